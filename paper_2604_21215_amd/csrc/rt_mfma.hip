// bf16 MFMA kernels (gfx950, v_mfma_f32_16x16x32_bf16): the pre-pass projection GEMM and the
// cross-block UpdateTile (Appendix C, Algorithm 2) as a flash-style contraction.
//
// Operand layout of v_mfma_f32_16x16x32_bf16 (D = A*B + C, A 16x32, B 32x16, 64 lanes, g = lane/16):
//   A: lane holds A[row = lane%16][k = 8g .. 8g+7]          (8 bf16 = 16 bytes)
//   B: lane holds B[k = 8g .. 8g+7][col = lane%16]
//   D: lane holds D[row = 4g + r][col = lane%16], r = 0..3   (4 fp32)
// Both operands want the contraction index contiguous per lane, which is how x, the weights, q and k
// rows are stored, so those fragments are loaded straight from global memory.
#include "rt_mfma_device.h"
#include "rt_cross_tile.h"
#include "rt_prepass_device.h"
#include "rt_gemm_tiled.h"

namespace rt {

// =============================================================================================
// Pre-pass GEMM (prepass_mfma_body): grid (ceil(M/128), ceil(3H/2)), block 256.
// =============================================================================================
__global__ __launch_bounds__(256) void prepass_mfma_kernel(const bf16_t *__restrict__ x, const float *__restrict__ rinv,
                                                           const bf16_t *__restrict__ Wq, const bf16_t *__restrict__ Wk,
                                                           const bf16_t *__restrict__ Wv, const bf16_t *__restrict__ g_attn,
                                                           const bf16_t *__restrict__ g_q, const bf16_t *__restrict__ g_k,
                                                           bf16_t *__restrict__ Q, bf16_t *__restrict__ Kt,
                                                           bf16_t *__restrict__ Vt, float *__restrict__ Qf,
                                                           float *__restrict__ Ktf, int Bc, int Nc, size_t x_bstride,
                                                           int n0, int d, int H, float eps, int norm_free)
{
    prepass_mfma_body<false>(x, rinv, Wq, Wk, Wv, g_attn, g_q, g_k, Q, Kt, Vt, Qf, Ktf, Bc, Nc, x_bstride, n0, d, H, eps, norm_free,
                             blockIdx.x, blockIdx.y);
}

// The same projection with both operands staged in LDS (tiled_mainloop), for many rows and d a multiple of 128: a
// wavefront's 64 columns are one head of q, k_tmp or v_tmp, so the qkRMS of a row is a sum over its two column
// tiles and the 32 lanes of its half of the wavefront.  grid (ceil(M / 256), 3 d / 128), block 256.
__global__ __launch_bounds__(256) void prepass_tiled_kernel(const bf16_t *__restrict__ x, const float *__restrict__ rinv,
                                                            const bf16_t *__restrict__ Wq, const bf16_t *__restrict__ Wk,
                                                            const bf16_t *__restrict__ Wv, const bf16_t *__restrict__ g_attn,
                                                            const bf16_t *__restrict__ g_q, const bf16_t *__restrict__ g_k,
                                                            bf16_t *__restrict__ Q, bf16_t *__restrict__ Kt,
                                                            bf16_t *__restrict__ Vt, float *__restrict__ Qf,
                                                            float *__restrict__ Ktf, int Bc, int Nc, size_t x_bstride,
                                                            int n0, int d, int H, float eps, int norm_free)
{
    __shared__ __align__(16) bf16_t As[kGtRows * kGtLd];
    __shared__ __align__(16) bf16_t Bs[kGtCols * kGtLd];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, hi = lane >> 5;
    const int M = Bc * Nc;
    const int m0 = blockIdx.x * kGtRows;
    const int c0 = blockIdx.y * kGtCols;          // first of the block's columns of [q | k_tmp | v_tmp]
    const int bw = c0 / d;                         // d is a multiple of 128: a block lies within one of the three
    const bf16_t *Wb = (bw == 0 ? Wq : (bw == 1 ? Wk : Wv)) + (size_t)(c0 - bw * d) * d;
    const int prow = tid >> 3, pc = tid & 7;
    const bf16_t *ga[8], *gb[4];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int mr = min(m0 + prow + 32 * i, M - 1);
        ga[i] = x + (size_t)(mr / Nc) * x_bstride + (size_t)(n0 + mr % Nc) * d + pc * 8;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) gb[i] = Wb + (size_t)(prow + 32 * i) * d + pc * 8;

    f32x16_t acc[4][2];
    tiled_mainloop(ga, gb, (g_attn != nullptr && !norm_free) ? g_attn : nullptr, d, As, Bs, acc);

    const int hcol = c0 - bw * d + wn * 64;        // first column of this wavefront's head within its output
    const bool normed = bw < 2 && !norm_free;
    const bf16_t *gn = bw == 0 ? g_q : g_k;
    bf16_t *dst = bw == 0 ? Q : (bw == 1 ? Kt : Vt);
    float *dstf = bw == 0 ? Qf : (bw == 1 ? Ktf : nullptr);   // optional unrounded copies of q and k_tmp
    float gc[2] = {1.f, 1.f};
    if (normed && gn) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) gc[nt] = bf16_to_f32(gn[hcol + nt * 32 + l32]);
    }
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int m = m0 + wm * 128 + mt * 32 + 8 * (i / 4) + 4 * hi + (i % 4);
            const float rs = norm_free ? 1.f : rinv[min(m, M - 1)];
            const float v0 = acc[mt][0][i] * rs, v1 = acc[mt][1][i] * rs;
            float sc = 1.f;
            if (normed) {
                float ss = fmaf(v0, v0, v1 * v1);
#pragma unroll
                for (int o = 16; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);   // the 32 lanes that share hi
                sc = rsqrtf(ss / (float)kHeadDim + eps);
            }
            if (m < M) {
                const int b = m / Nc, n = n0 + m % Nc;
                const size_t oo = ((size_t)n * Bc + b) * d + hcol + l32;
                const float o0 = v0 * sc * gc[0], o1 = v1 * sc * gc[1];
                dst[oo] = f32_to_bf16(o0);
                dst[oo + 32] = f32_to_bf16(o1);
                if (dstf) { dstf[oo] = o0; dstf[oo + 32] = o1; }
            }
        }
    }
}

// out[r][k] = bf16(W[r][k] * g[k]) for the three d x d projection matrices stacked: the tiled pre-pass then stages its input
// rows as they are (vector work in the staging step is on that kernel's critical path).  grid ceil(3 d d / 8 / 256), block 256.
__global__ __launch_bounds__(256) void scale_qkv_columns_kernel(const bf16_t *__restrict__ Wq, const bf16_t *__restrict__ Wk,
                                                                const bf16_t *__restrict__ Wv, const bf16_t *__restrict__ g,
                                                                bf16_t *__restrict__ out, int d)
{
    const size_t per = (size_t)d * d / 8;           // 16-byte pieces per matrix
    const size_t q = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (q >= 3 * per) return;
    const int which = (int)(q / per);
    const size_t e = (q - which * per) * 8;         // element offset within the matrix
    const int k = (int)(e % (size_t)d);
    const bf16_t *W = which == 0 ? Wq : (which == 1 ? Wk : Wv);
    float w[8], gg[8];
    load8(W + e, w);
    load8(g + k, gg);
    *reinterpret_cast<uint4 *>(out + (size_t)which * d * d + e) =
        make_uint4(pack_bf16(w[0] * gg[0], w[1] * gg[1]), pack_bf16(w[2] * gg[2], w[3] * gg[3]),
                   pack_bf16(w[4] * gg[4], w[5] * gg[5]), pack_bf16(w[6] * gg[6], w[7] * gg[7]));
}

constexpr int kTiledMinRows = 2048;   // below this the untiled kernel's smaller block tiles fill the chip better

hipError_t prepass_mfma_launch(const LayerDims &D, const Weights &W, const Scratch &S, const void *x, int Bc, int Nc,
                               size_t x_bstride, int n0, hipStream_t st)
{
    const int M = Bc * Nc;
    if (M >= kTiledMinRows && D.d % 128 == 0) {
        const bf16_t *wq = (const bf16_t *)W.Wq, *wk = (const bf16_t *)W.Wk, *wv = (const bf16_t *)W.Wv, *ga = (const bf16_t *)W.g_attn;
        if (ga && !D.norm_free && S.wg_qkv) {   // the gain goes into the matrices' columns
            const size_t pieces = 3 * (size_t)D.d * D.d / 8;
            hipLaunchKernelGGL(scale_qkv_columns_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st, wq, wk, wv, ga,
                               S.wg_qkv, D.d);
            wq = S.wg_qkv; wk = wq + (size_t)D.d * D.d; wv = wk + (size_t)D.d * D.d; ga = nullptr;
        }
        hipLaunchKernelGGL(prepass_tiled_kernel, dim3((M + kGtRows - 1) / kGtRows, 3 * D.d / kGtCols), dim3(256), 0, st,
                           (const bf16_t *)x, S.rinv, wq, wk, wv, ga, (const bf16_t *)W.g_q, (const bf16_t *)W.g_k, (bf16_t *)S.Q,
                           (bf16_t *)S.Kt, (bf16_t *)S.Vt, S.Qf, S.Ktf, Bc, Nc, x_bstride, n0, D.d, D.H, D.eps, D.norm_free);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(prepass_mfma_kernel, dim3((M + 127) / 128, (3 * D.H + 1) / 2), dim3(256), 0, st, (const bf16_t *)x,
                       S.rinv, (const bf16_t *)W.Wq, (const bf16_t *)W.Wk, (const bf16_t *)W.Wv, (const bf16_t *)W.g_attn,
                       (const bf16_t *)W.g_q, (const bf16_t *)W.g_k, (bf16_t *)S.Q, (bf16_t *)S.Kt, (bf16_t *)S.Vt, S.Qf, S.Ktf,
                       Bc, Nc, x_bstride, n0, D.d, D.H, D.eps, D.norm_free);
    return hipGetLastError();
}

// =============================================================================================
// Cross-block UpdateTile as a stand-alone launch: queries [t1, t1+nq) against keys [t1-P, t1).
// A wavefront owns 32 queries (two 16-query tiles); a block is 4 wavefronts = 128 queries.
// grid (ceil(nq/128), B*H).  HP: unrounded queries Qf, keys as head K plus remainder Klo (three products per
// logit tile).  ALIBI: linear positional bias with the head's slope 2^(-alibi (h+1)/H).
// =============================================================================================
template <bool HP, bool ALIBI>
__global__ __launch_bounds__(256) void cross_mfma_kernel(const bf16_t *__restrict__ Q, const float *__restrict__ Qf,
                                                         const bf16_t *__restrict__ K, const bf16_t *__restrict__ Klo,
                                                         const bf16_t *__restrict__ VT, int vt_stride,
                                                         float *__restrict__ pm, float *__restrict__ pl,
                                                         float *__restrict__ po, int BH, int t1, int P, int nq, int level,
                                                         int level_rel, int slots, float scale, float alibi, int H)
{
    const int wave = threadIdx.x >> 6;
    const int q0 = blockIdx.x * 128 + wave * 32;  // first query of this wavefront, relative to t1
    if (q0 >= nq) return;                         // no barriers in this kernel
    cross_mfma_wave<HP, ALIBI>(Q, Qf, K, Klo, VT, vt_stride, pm, pl, po, BH, blockIdx.y, t1, 0, t1 - P, P, q0, nq, level,
                               level_rel, slots, scale, ALIBI ? alibi_slope(alibi, (int)blockIdx.y % H, H) : 0.f);
}

// Same tile with K and V^T staged in LDS for the four wavefronts (128 queries) of a workgroup, blocks of
// 64 keys and more.  Workgroups are dealt to the 8 XCDs round-robin by the dispatcher, so the index is
// decoded such that all query blocks of one (b, h) land on the same XCD and its key/value tiles are
// fetched into that L2 once.  The HP form's three LDS tiles per buffer leave room for two workgroups per compute unit.
#define RT_CROSS_TILE_KERNEL(NAME, HPv, WAVES)                                                                              \
    template <bool ALIBI, int VAR = kCtVarDefault>                                                                          \
    __global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(WAVES, WAVES))) void NAME(                        \
        const bf16_t *__restrict__ Q, const float *__restrict__ Qf, const bf16_t *__restrict__ K,                          \
        const bf16_t *__restrict__ Klo, const bf16_t *__restrict__ VT, int vt_stride, float *__restrict__ pm,              \
        float *__restrict__ pl, float *__restrict__ po, int BH, int t1, int P, int nq, int nqb, int level, int level_rel,  \
        int slots, float scale, float alibi, int H)                                                                         \
    {                                                                                                                       \
        __shared__ __align__(16) unsigned char lds[2 * cross_tile_lds_bytes<HPv>()];                                        \
        const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;                                                                \
        const int bh = (j / nqb) * 8 + xcd, qb = j % nqb;                                                                   \
        if (bh >= BH) return; /* the whole workgroup leaves together */                                                     \
        cross_tile_wg<HPv, 4, 2, ALIBI, HPv, VAR>(Q, Qf, K, Klo, VT, vt_stride, pm, pl, po, BH, bh, t1, 0, t1 - P, P,       \
                                        qb * 128 + (int)(threadIdx.x >> 6) * 32, nq, level, level_rel, slots, scale, lds,   \
                                        (int)threadIdx.x, ALIBI ? alibi_slope(alibi, bh % H, H) : 0.f);                     \
    }
RT_CROSS_TILE_KERNEL(cross_tile_kernel, false, 4)
RT_CROSS_TILE_KERNEL(cross_tile_hp_kernel, true, 4)
#undef RT_CROSS_TILE_KERNEL

hipError_t cross_mfma_launch(const LayerDims &D, const Scratch &S, const void *K, int t1, int P, int nq, bool hp,
                             hipStream_t st)
{
    int level = 0;
    while ((1 << level) < P) ++level;
    const int nqb = (nq + 127) / 128;
    const int BH = D.B * D.H, bh8 = (BH + 7) / 8 * 8;
    const bool al = D.alibi > 0.f;
    const bf16_t *Q = (const bf16_t *)S.Q, *Kb = (const bf16_t *)K;
#define RT_TILE_ARGS Q, S.Qf, Kb, (hp ? reinterpret_cast<const bf16_t *>(S.Kh) : S.Klo), S.VT, S.vt_stride, S.pm, S.pl, S.po, BH, t1, P, nq, nqb, level, level - D.log2_pmin, S.slots, D.scale, D.alibi, D.H
#define RT_WAVE_ARGS Q, S.Qf, Kb, S.Klo, S.VT, S.vt_stride, S.pm, S.pl, S.po, BH, t1, P, nq, level, level - D.log2_pmin, S.slots, D.scale, D.alibi, D.H
    if (P >= kKC) {
        const dim3 grid(bh8 * nqb);
        if (hp && al) hipLaunchKernelGGL(cross_tile_hp_kernel<true>, grid, dim3(256), 0, st, RT_TILE_ARGS);
        else if (hp) hipLaunchKernelGGL(cross_tile_hp_kernel<false>, grid, dim3(256), 0, st, RT_TILE_ARGS);
        else if (al) hipLaunchKernelGGL(cross_tile_kernel<true>, grid, dim3(256), 0, st, RT_TILE_ARGS);
        else hipLaunchKernelGGL(cross_tile_kernel<false>, grid, dim3(256), 0, st, RT_TILE_ARGS);
    } else {
        const dim3 grid(nqb, BH);
        if (hp && al) hipLaunchKernelGGL((cross_mfma_kernel<true, true>), grid, dim3(256), 0, st, RT_WAVE_ARGS);
        else if (hp) hipLaunchKernelGGL((cross_mfma_kernel<true, false>), grid, dim3(256), 0, st, RT_WAVE_ARGS);
        else if (al) hipLaunchKernelGGL((cross_mfma_kernel<false, true>), grid, dim3(256), 0, st, RT_WAVE_ARGS);
        else hipLaunchKernelGGL((cross_mfma_kernel<false, false>), grid, dim3(256), 0, st, RT_WAVE_ARGS);
    }
#undef RT_TILE_ARGS
#undef RT_WAVE_ARGS
    return hipGetLastError();
}

}  // namespace rt
