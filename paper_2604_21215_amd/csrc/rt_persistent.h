// Interface of the single-launch ("persistent") engine of the sequential loop.
#pragma once
#include "../../include/rt.h"
#include "rt_common.h"
#include <string>

namespace rt {

struct PersistentState {
    bool available = false;
    bool launched = false;
    void *slab = nullptr;
    size_t slab_bytes = 0;
    size_t exchange_bytes = 0;           // leading part of the slab that holds the counters and the exchange words
    int num_cu = 0;
    int grid = 0;
    size_t lds_bytes = 0;
    long long spin_limit = 0;
    // exchange buffers between the phases of a position (device)
    unsigned long long *bar = nullptr;   // [0] fenced-barrier counter, [8] abort word (non-zero once a wait expired)
    void *a_ll = nullptr, *h_ll = nullptr, *u_ll = nullptr, *z_ll = nullptr;
    void *kv_ll = nullptr, *zss_ll = nullptr, *zp_ll = nullptr;
    int win_rows = 0, upw = 1;
    int max_batch = 0;
    unsigned nonce = 0;                  // per-call tag prefix of the exchange words
    unsigned long long *trace = nullptr; // optional per-position phase clocks
    int trace_rows = 0;
};

rt_status persistent_create(PersistentState &P, const rt_config &cfg, const LayerDims &base);
void persistent_destroy(PersistentState &P);
size_t persistent_bytes(const PersistentState &P);
bool persistent_supported(const PersistentState &P, const LayerDims &D);
rt_status persistent_prefill(PersistentState &P, const LayerDims &D, const Weights &W, const Scratch &S, const void *x,
                             void *y, void *K, void *V, hipStream_t st, std::string &err);
int persistent_wait_expired(PersistentState &P);
int persistent_read_trace(PersistentState &P, unsigned long long *out, int rows);

}  // namespace rt
