// Interface of the single-launch ("persistent") engine of the sequential loop.
#pragma once
#include "../../include/rt.h"
#include "rt_common.h"
#include <string>

namespace rt {

struct PersistentState {
    bool available = false;
    void *slab = nullptr;
    size_t slab_bytes = 0;
    int *d_flags = nullptr;  // device: [0] abort flag, then barrier counters
    int *h_flags = nullptr;  // pinned host mirror of the abort flag
    int num_cu = 0;
    int grid = 0;
    size_t lds_bytes = 0;
};

rt_status persistent_create(PersistentState &P, const rt_config &cfg, const LayerDims &base);
void persistent_destroy(PersistentState &P);
size_t persistent_bytes(const PersistentState &P);
bool persistent_supported(const PersistentState &P, const LayerDims &D);
rt_status persistent_prefill(PersistentState &P, const LayerDims &D, const Weights &W, const Scratch &S, const void *x,
                             void *y, void *K, void *V, hipStream_t st, std::string &err);
int persistent_wait_expired(PersistentState &P);

}  // namespace rt
