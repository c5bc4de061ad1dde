// Internal interface of the backward pass (rt_backward.hip), paper Sec. 6.4.
#pragma once
#include "rt_common.h"
#include "rt_backward_persistent.h"

namespace rt {

// Where the parameter gradients go (device, fp32, written not accumulated; null = not wanted).
struct BwGrads {
    float *Wq, *Wk, *Wv, *Wo, *W1, *W2;
    float *g_attn, *g_mlp, *g_kv, *g_q, *g_k;
};

// bytes of scratch for sequences of B x N positions (E = bytes per element of the storage type)
size_t backward_scratch_bytes(size_t B, size_t N, size_t d, size_t F, size_t H, size_t E);

// x, z, gy [B][N][d]; gK, gV [N][B][H][64] or null (storage type T); dx [B][N][d] fp32.
// matrix_cores: with bf16 storage the batched products run on the matrix cores from bf16 copies of their operands.
// loop: the single-launch reverse loop (or null: one set of launches per position); its exchange words are part of ws
// and must have been zeroed once (backward_exchange_region).
template <typename T>
hipError_t backward_layer(const LayerDims &D, const Weights &W, const void *x, const void *z, const void *gy, const void *gK,
                          const void *gV, float *dx, const BwGrads &G, void *ws, bool matrix_cores, hipStream_t st,
                          BwpState *loop = nullptr);
// The attention-shaped passes on the matrix cores (rt_backward_attn.hip; fp32 rows [N][B H][64] in, bf16 head + remainder
// operands): dq += the keys' share, after the loop; one block of Algorithm 1 backwards, keys [k0, k0 + P) <- queries
// [q0, q0 + nq).  bw_attn_mfma_init once per process before the first of them.
hipError_t bw_attn_mfma_init();
hipError_t bw_dq_mfma(const LayerDims &D, const float *Qn, const float *Kp, const float *Vp, const float *dc, const float *lse,
                      const float *Ds, float *dq, hipStream_t st);
hipError_t bw_event_mfma(const LayerDims &D, const float *Qn, const float *Kp, const float *Vp, const float *dc, const float *lse,
                         const float *Ds, float *dK, float *dV, int k0, int P, int q0, int nq, hipStream_t st);
// where the exchange words of the single-launch loop lie inside a scratch area laid out for B x N positions
void backward_exchange_region(size_t B, size_t N, size_t d, size_t F, size_t H, size_t E, size_t *offset, size_t *bytes);

}  // namespace rt
