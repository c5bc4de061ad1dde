// Device body of the pre-pass projection GEMM on the matrix cores (bf16), shared by the whole-sequence launch
// and the per-chunk launch of the layer-wavefront engine.
#pragma once
#include "rt_mfma_device.h"

namespace rt {

// =============================================================================================
// Pre-pass GEMM: C[m][c] = sum_k (x[m][k] g_attn[k]) Wqkv[c][k], rows scaled by rinv[m], then qkRMS
// per head for the q and k_tmp parts.  Block tile 128 x 128, 4 wavefronts as 2 x 2, each 64 x 64
// (= one head of one output).  grid (ceil(M/128), ceil(3H/2)).
// =============================================================================================
// OWN_RINV: the 1/rms of the input rows is not read from rinv but formed from the A fragments on the way (every
// wavefront reads its 64 input rows in full).
template <bool OWN_RINV>
__device__ __forceinline__ void prepass_mfma_body(const bf16_t *__restrict__ x, const float *__restrict__ rinv,
                                                  const bf16_t *__restrict__ Wq, const bf16_t *__restrict__ Wk,
                                                  const bf16_t *__restrict__ Wv, const bf16_t *__restrict__ g_attn,
                                                  const bf16_t *__restrict__ g_q, const bf16_t *__restrict__ g_k,
                                                  bf16_t *__restrict__ Q, bf16_t *__restrict__ Kt,
                                                  bf16_t *__restrict__ Vt, float *__restrict__ Qf,
                                                  float *__restrict__ Ktf, int Bc, int Nc, size_t x_bstride,
                                                  int n0, int d, int H, float eps, int norm_free, int block_x,
                                                  int block_y)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l16 = lane & 15, g = lane >> 4;
    const int M = Bc * Nc;
    const int m0 = block_x * 128 + wm * 64;
    const int hb = block_y * 2 + wn;  // head slot in [q heads | k heads | v heads]
    if (hb >= 3 * H || m0 >= M) return;  // no barriers in this kernel
    const int which = hb / H, h = hb % H;
    const bf16_t *W = (which == 0 ? Wq : (which == 1 ? Wk : Wv)) + (size_t)h * kHeadDim * d;

    f32x4_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    const bf16_t *arow[4];
    const bf16_t *brow[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int mr = min(m0 + i * 16 + l16, M - 1);
        arow[i] = x + (size_t)(mr / Nc) * x_bstride + (size_t)(n0 + mr % Nc) * d + 8 * g;
        brow[i] = W + (size_t)(i * 16 + l16) * d + 8 * g;
    }
    const bool use_gain = (g_attn != nullptr) && !norm_free;
    float ssq[4] = {0.f, 0.f, 0.f, 0.f};   // OWN_RINV: sum of squares of input row l16 + 16 i over this lane's k slices

    for (int k0 = 0; k0 < d; k0 += 32) {
        Frag a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a[i].u = *reinterpret_cast<const uint4 *>(arow[i] + k0);
            b[i].u = *reinterpret_cast<const uint4 *>(brow[i] + k0);
        }
        if (OWN_RINV && !norm_free) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t w4[4] = {a[i].u.x, a[i].u.y, a[i].u.z, a[i].u.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float lo = __uint_as_float(w4[e] << 16), hi = __uint_as_float(w4[e] & 0xFFFF0000u);
                    ssq[i] = fmaf(lo, lo, fmaf(hi, hi, ssq[i]));
                }
            }
        }
        if (use_gain) {
            float gg[8];
            load8(g_attn + k0 + 8 * g, gg);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float xv[8];
                xv[0] = __uint_as_float(a[i].u.x << 16); xv[1] = __uint_as_float(a[i].u.x & 0xFFFF0000u);
                xv[2] = __uint_as_float(a[i].u.y << 16); xv[3] = __uint_as_float(a[i].u.y & 0xFFFF0000u);
                xv[4] = __uint_as_float(a[i].u.z << 16); xv[5] = __uint_as_float(a[i].u.z & 0xFFFF0000u);
                xv[6] = __uint_as_float(a[i].u.w << 16); xv[7] = __uint_as_float(a[i].u.w & 0xFFFF0000u);
                a[i].u.x = pack_bf16(xv[0] * gg[0], xv[1] * gg[1]);
                a[i].u.y = pack_bf16(xv[2] * gg[2], xv[3] * gg[3]);
                a[i].u.z = pack_bf16(xv[4] * gg[4], xv[5] * gg[5]);
                a[i].u.w = pack_bf16(xv[6] * gg[6], xv[7] * gg[7]);
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = mfma16(a[i], b[j], acc[i][j]);
    }

    if (OWN_RINV && !norm_free) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {   // join the four k slices of a row: afterwards every lane with this l16 holds the row's sum
            ssq[i] += __shfl_xor(ssq[i], 16, 64);
            ssq[i] += __shfl_xor(ssq[i], 32, 64);
            ssq[i] = rsqrtf(ssq[i] / (float)d + eps);
        }
    }
    const bf16_t *gn = which == 0 ? g_q : g_k;
    bf16_t *dst = which == 0 ? Q : (which == 1 ? Kt : Vt);
    float *dstf = which == 0 ? Qf : (which == 1 ? Ktf : nullptr);   // optional unrounded copies of q and k_tmp
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int m = m0 + i * 16 + 4 * g + r;
            // the output rows of this lane are 16 i + 4 g + r; their scale sits in the lanes whose l16 is 4 g + r
            const float rs = norm_free ? 1.f : (OWN_RINV ? __shfl(ssq[i], 4 * g + r, 64) : rinv[min(m, M - 1)]);
            float v[4];
            float ss = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) { v[j] = acc[i][j][r] * rs; ss = fmaf(v[j], v[j], ss); }
            float sc = 1.f;
            if (which < 2 && !norm_free) {
#pragma unroll
                for (int o = 8; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);  // the 16 lanes that share g
                sc = rsqrtf(ss / (float)kHeadDim + eps);
            }
            if (m < M) {
                const int b = m / Nc, n = n0 + m % Nc;
                const size_t oo = ((size_t)n * Bc + b) * d + h * kHeadDim + l16;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    float val = v[j] * sc;
                    if (which < 2 && !norm_free && gn) val *= bf16_to_f32(gn[h * kHeadDim + j * 16 + l16]);
                    dst[oo + j * 16] = f32_to_bf16(val);
                    if (dstf) dstf[oo + j * 16] = val;
                }
            }
        }
    }
}

}  // namespace rt
