// The two operations a stack of RT layers needs around the layers themselves: the embedding lookup
// that produces the first layer's input, and the final RMS normalisation followed by the untied
// output projection ("LM head").  Neither is part of the layer recurrence (Sec. 6.1 leaves embedding
// and unembedding out of its cost model); both are bandwidth-bound single passes.
#include "rt_common.h"

namespace rt {

// x[b][n][:] = table[ids[b * ids_stride + first + n]][:]; one wavefront per row, 16-byte pieces.
template <typename T>
__global__ __launch_bounds__(256) void embed_rows_kernel(const T *__restrict__ table, const int32_t *__restrict__ ids,
                                                         T *__restrict__ x, int B, int N, int d, int vocab,
                                                         long long ids_stride, int first)
{
    const int lane = threadIdx.x & 63;
    const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= (long long)B * N) return;
    const int b = (int)(row / N), n = (int)(row % N);
    int id = ids[b * ids_stride + first + n];
    id = min(max(id, 0), vocab - 1);  // ids outside the table are clamped, never dereferenced
    constexpr int per = 16 / (int)sizeof(T);
    const uint4 *src = reinterpret_cast<const uint4 *>(table + (size_t)id * d);
    uint4 *dst = reinterpret_cast<uint4 *>(x + (size_t)row * d);
    for (int c = lane; c < d / per; c += 64) dst[c] = src[c];
}

// logits[b][v] = sum_k W[v][k] * (g[k] z[b][k] / rms(z[b])), fp32 out.  A workgroup first builds the
// normalised rows of one batch tile in LDS, then each of its wavefronts walks over vocabulary rows.
constexpr int kHeadLdsFloats = 12288;

template <typename T>
__global__ __launch_bounds__(256) void lm_head_kernel(const T *__restrict__ W, const T *__restrict__ g,
                                                      const T *__restrict__ z, long long z_stride, float *__restrict__ logits,
                                                      int B, int d, int vocab, float eps, int norm_free, int bt)
{
    __shared__ float zs[kHeadLdsFloats];
    __shared__ float red[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int b0 = 0; b0 < B; b0 += bt) {
        const int nb = min(bt, B - b0);
        __syncthreads();
        for (int b = 0; b < nb; ++b) {
            const T *zr = z + (size_t)(b0 + b) * z_stride;
            float ss = 0.f;
            for (int k = threadIdx.x; k < d; k += 256) {
                const float v = to_f32(zr[k]);
                zs[b * d + k] = v;
                ss = fmaf(v, v, ss);
            }
            ss = wave_sum(ss);
            if (lane == 0) red[wave] = ss;
            __syncthreads();
            const float tot = red[0] + red[1] + red[2] + red[3];
            const float rinv = norm_free ? 1.f : rsqrtf(tot / (float)d + eps);
            for (int k = threadIdx.x; k < d; k += 256) {
                const float gg = (g && !norm_free) ? to_f32(g[k]) : 1.f;
                zs[b * d + k] *= rinv * gg;
            }
            __syncthreads();
        }
        for (int v = blockIdx.x * 4 + wave; v < vocab; v += gridDim.x * 4) {
            const T *wr = W + (size_t)v * d;
            float acc[8];
#pragma unroll
            for (int b = 0; b < 8; ++b) acc[b] = 0.f;
            for (int k = lane * 8; k < d; k += 512) {
                float w[8];
                load8(wr + k, w);
#pragma unroll
                for (int b = 0; b < 8; ++b) {
                    if (b < nb) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[b] = fmaf(w[e], zs[b * d + k + e], acc[b]);
                    }
                }
            }
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                if (b < nb) {
                    const float s = wave_sum(acc[b]);
                    if (lane == 0) logits[(size_t)(b0 + b) * vocab + v] = s;
                }
            }
        }
    }
}

template <typename T>
hipError_t embed_rows_launch(const void *table, const int32_t *ids, void *x, int B, int N, int d, int vocab,
                             long long ids_stride, int first, hipStream_t st)
{
    const long long rows = (long long)B * N;
    hipLaunchKernelGGL(embed_rows_kernel<T>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, (const T *)table, ids, (T *)x,
                       B, N, d, vocab, ids_stride, first);
    return hipGetLastError();
}

template <typename T>
hipError_t lm_head_launch(const void *W, const void *g, const void *z, long long z_stride, float *logits, int B, int d,
                          int vocab, float eps, int norm_free, hipStream_t st)
{
    int bt = kHeadLdsFloats / d;
    if (bt > 8) bt = 8;
    int blocks = (vocab + 3) / 4;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(lm_head_kernel<T>, dim3(blocks), dim3(256), 0, st, (const T *)W, (const T *)g, (const T *)z, z_stride,
                       logits, B, d, vocab, eps, norm_free, bt);
    return hipGetLastError();
}

template hipError_t embed_rows_launch<float>(const void *, const int32_t *, void *, int, int, int, int, long long, int,
                                             hipStream_t);
template hipError_t embed_rows_launch<bf16_t>(const void *, const int32_t *, void *, int, int, int, int, long long, int,
                                              hipStream_t);
template hipError_t lm_head_launch<float>(const void *, const void *, const void *, long long, float *, int, int, int, float,
                                          int, hipStream_t);
template hipError_t lm_head_launch<bf16_t>(const void *, const void *, const void *, long long, float *, int, int, int, float,
                                           int, hipStream_t);

}  // namespace rt
