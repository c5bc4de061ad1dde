// Main loop of the bf16 products C[m][n] = sum_k A[m][k] W[n][k] with both operands staged in LDS, for many rows
// (the layer's projections of Sec. 2.2 when all positions are known: pre-pass, and the loop-free layers of
// Sec. 2.1 / Sec. 6.1).
// Block tile 256 x 128, k-tiles of 64; four wavefronts as 2 x 2, each 128 x 64 = 4 x 2 tiles of
// v_mfma_f32_32x32x16_bf16 (128 accumulator registers); per 16-index step a wavefront reads 4 + 2 fragments from
// LDS for 8 matrix instructions (0.75 of the LDS rate at full matrix rate).  One LDS buffer (55 KB: two workgroups
// per compute unit); the next k-tile is fetched into registers (12 x 16 bytes per thread) while the current one
// is used.  Rows of the tiles are 72 elements apart (16-byte fragment reads of consecutive rows hit distinct banks).
#pragma once
#include "rt_mfma_device.h"
#include "rt_cross_tile.h"

namespace rt {

constexpr int kGtLd = 72;                      // row stride of the staged tiles in elements
constexpr int kGtRows = 256, kGtCols = 128;    // block tile

// Staging: piece p = tid + 256 i of a k-tile is row p / 8, 16-byte column p % 8.  ga[i] / gb[i] point at k = 0 of the
// piece's row of A (8 per thread, rows tid / 8 + 32 i of the block tile) and of W (4 per thread), already offset by
// 8 (tid % 8) elements.  gain (may be null): per-k factors applied to A while it is staged.  K is a multiple of 64.
// acc[mt][nt] register i afterwards: row 128 wm + 32 mt + 8 (i / 4) + 4 (lane / 32) + i % 4, column
// 64 wn + 32 nt + lane % 32 of the block tile, wm = wave / 2, wn = wave % 2.
__device__ __forceinline__ void tiled_mainloop(const bf16_t *const (&ga)[8], const bf16_t *const (&gb)[4],
                                               const bf16_t *__restrict__ gain, int K, bf16_t *__restrict__ As,
                                               bf16_t *__restrict__ Bs, f32x16_t (&acc)[4][2])
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, hi = lane >> 5;
    const int prow = tid >> 3, pc = tid & 7;
    const bool gained = gain != nullptr;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mt][nt][i] = 0.f;

    u32x4_t ra[8], rb[4];
#define RT_GT_FETCH(k0)                                                                                     \
    _Pragma("unroll") for (int i = 0; i < 8; ++i) ra[i] = *reinterpret_cast<const u32x4_t *>(ga[i] + (k0)); \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) rb[i] = *reinterpret_cast<const u32x4_t *>(gb[i] + (k0));
#define RT_GT_STAGE(k0)                                                                                  \
    {                                                                                                    \
        float gg[8];                                                                                     \
        if (gained) load8(gain + (k0) + pc * 8, gg);                                                     \
        _Pragma("unroll") for (int i = 0; i < 8; ++i)                                                    \
        {                                                                                                \
            u32x4_t v = ra[i];                                                                           \
            if (gained) {                                                                                \
                _Pragma("unroll") for (int e = 0; e < 4; ++e)                                            \
                    v[e] = pack_bf16(__uint_as_float(v[e] << 16) * gg[2 * e],                            \
                                     __uint_as_float(v[e] & 0xFFFF0000u) * gg[2 * e + 1]);               \
            }                                                                                            \
            *reinterpret_cast<u32x4_t *>(As + (prow + 32 * i) * kGtLd + pc * 8) = v;                     \
        }                                                                                                \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                    \
            *reinterpret_cast<u32x4_t *>(Bs + (prow + 32 * i) * kGtLd + pc * 8) = rb[i];                 \
    }

    RT_GT_FETCH(0)
    RT_GT_STAGE(0)
    __syncthreads();
    for (int k0 = 0; k0 < K; k0 += 64) {
        const bool more = k0 + 64 < K;
        if (more) { RT_GT_FETCH(k0 + 64) }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            uint4 fa[4], fb[2];
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
                fa[mt] = *reinterpret_cast<const uint4 *>(As + (wm * 128 + mt * 32 + l32) * kGtLd + ks * 16 + 8 * hi);
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
                fb[nt] = *reinterpret_cast<const uint4 *>(Bs + (wn * 64 + nt * 32 + l32) * kGtLd + ks * 16 + 8 * hi);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) acc[mt][nt] = mfma32u(fa[mt], fb[nt], acc[mt][nt]);
        }
        __syncthreads();   // everyone is done reading the tiles
        if (more) {
            RT_GT_STAGE(k0 + 64)
            __syncthreads();
        }
    }
#undef RT_GT_FETCH
#undef RT_GT_STAGE
}

}  // namespace rt
