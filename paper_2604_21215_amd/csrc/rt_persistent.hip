// Single-launch engine of the sequential loop (placeholder: reports "not available" so that the
// per-position engine is used).
#include "rt_persistent.h"

namespace rt {

rt_status persistent_create(PersistentState &P, const rt_config &, const LayerDims &)
{
    P.available = false;
    return RT_ERR_UNSUPPORTED;
}
void persistent_destroy(PersistentState &) {}
size_t persistent_bytes(const PersistentState &P) { return P.slab_bytes; }
bool persistent_supported(const PersistentState &P, const LayerDims &) { return P.available; }
rt_status persistent_prefill(PersistentState &, const LayerDims &, const Weights &, const Scratch &, const void *, void *,
                             void *, void *, hipStream_t, std::string &err)
{
    err = "persistent engine not available";
    return RT_ERR_UNSUPPORTED;
}
int persistent_wait_expired(PersistentState &) { return 0; }

}  // namespace rt
