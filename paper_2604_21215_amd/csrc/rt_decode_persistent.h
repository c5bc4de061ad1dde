// Interface of the single-launch decoding step (rt_decode_persistent.hip).
#pragma once
#include "../../include/rt.h"
#include "rt_common.h"
#include <string>

namespace rt {

struct DecodeCoopState {
    bool available = false;
    bool launched = false;
    void *slab = nullptr;             // counters and exchange words
    size_t slab_bytes = 0;
    int grid = 0;
    size_t lds_bytes = 0;
    int max_batch = 0;
    long long spin_limit = 0;
    unsigned nonce = 0;               // tag of the exchange words of the last call
    int d = 0, F = 0;
    bool cooperative = false;         // RT_DECODE_COOPERATIVE was set at rt_create: launch through the cooperative queue
    int split_override = 0;           // RT_DECODE_SPLIT: at most this many workgroups share the cache rows of one (b, h)
    bool want_trace = false;          // RT_DECODE_TRACE was set at rt_create: the kernel stamps its phases
};

rt_status decode_coop_create(DecodeCoopState &P, const rt_config &cfg, const LayerDims &base);
void decode_coop_destroy(DecodeCoopState &P);
size_t decode_coop_bytes(const DecodeCoopState &P);
bool decode_coop_supported(const DecodeCoopState &P, const LayerDims &D);
// one position t over the cache rows 0 .. t-1 of K, V; writes y_t and row t of K, V.  kv_row_elems: elements between two
// rows of the cache when the D.B sequences are a chunk of a larger batch (K, V then point at the chunk's first sequence
// inside row 0); 0: the rows hold these D.B sequences only
rt_status decode_coop_step(DecodeCoopState &P, const LayerDims &D, const Weights &W, const void *x_t, int t, void *y_t, void *K,
                           void *V, hipStream_t st, std::string &err, size_t kv_row_elems = 0);
int decode_coop_wait_expired(DecodeCoopState &P);
int decode_coop_read_trace(DecodeCoopState &P, unsigned long long *out, int workgroups);

}  // namespace rt
