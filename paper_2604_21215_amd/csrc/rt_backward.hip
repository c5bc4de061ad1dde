// Backward pass of one RT layer (paper Sec. 6.4, "The backward pass"), with the forward intermediates recomputed
// from the layer's input x and output z (Sec. 6.1, "Activation checkpointing").
//
// For L = <gy, y> + <gK, K> + <gV, V> the gradients with respect to x, the six matrices and the five gain vectors.
// Structure, as Sec. 6.4 describes it:
//   (A) recompute, all positions at once: with z given every persistent pair k_i, v_i = proj(RMS(z_i)) is known, so
//       queries, temporary pairs, the attention of every position (output and log-sum-exp), h and the MLP's
//       pre-activations are batched products and one pass per (b, h, position);
//   (B) the reverse loop over positions, which carries ONLY the gradients of the persistent pairs (dK, dV): position i
//       completes dz_i = gy_i + (what arrives through k_i, v_i), takes it back through the MLP, the residuals and Wo to
//       the attention output, and adds the softmax's contribution to dK_j, dV_j of the earlier positions.  The earlier
//       positions are reached in the blocks of Appendix C, Algorithm 1, run backwards: the keys [t-P+1, t] receive the
//       contribution of the queries [t+1, t+P] as one tile, after the last of those queries and before position t is
//       visited; blocks below kBwPmin keys are handled directly by each query (its "window");
//   (C) after the loop, batched: dq over all (query, key) pairs, the gradients of the temporary pairs, x through the
//       three projections and RMS, and every parameter sum as one product over all B N rows.
// Everything outside the batched products is fp32 on the vector ALUs; the storage type T decides how x, z, gy, gK, gV and
// the weights are read.  The batched products are fp32 LDS-tiled kernels for fp32 storage; for bf16 storage (the
// configurations' "bf16 compute with fp32 accumulation") they run on the matrix cores from bf16 copies of their
// operands - the recompute's activations as bf16 head + bf16 remainder (two products: no rounding of q, k, h or the
// MLP pre-activations that the forward engines avoid either), gradients rounded once.  Internal tensors are
// position-first: row r = n B + b.
#include "rt_base_case.h"
#include "rt_gemm_tiled.h"
#include "rt_backward.h"
#include <cstdlib>

namespace rt {

constexpr int kBwPmin = 32;      // keys closer than this are handled by the query's own wavefront in the reverse loop
constexpr int kTileLdF = 65;     // row stride (floats) of the 64 x 64 LDS tiles of the attention-gradient kernels

// ------------------------------------------------------------------------------------------------ small helpers
template <typename T>
__global__ __launch_bounds__(256) void bw_to_f32_kernel(const T *__restrict__ in, float *__restrict__ out, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) out[i] = to_f32(in[i]);
}

__global__ __launch_bounds__(256) void bw_fill_kernel(float *__restrict__ out, size_t n, float v)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) out[i] = v;
}

// out[c * ldo + col0 + r] = in[r * cols + c]  (r < rows, c < cols); grid (ceil(cols / 32), ceil(rows / 32)), block (32, 8)
template <typename T>
__global__ __launch_bounds__(256) void bw_transpose_kernel(const T *__restrict__ in, T *__restrict__ out, int rows, int cols,
                                                           size_t ldo, int col0)
{
    __shared__ T tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
    for (int j = ty; j < 32; j += 8)
        if (r0 + j < rows && c0 + tx < cols) tile[j][tx] = in[(size_t)(r0 + j) * cols + c0 + tx];
    __syncthreads();
    for (int j = ty; j < 32; j += 8)
        if (c0 + j < cols && r0 + tx < rows) out[(size_t)(c0 + j) * ldo + col0 + r0 + tx] = tile[tx][j];
}

// gradients handed in for K, V ([N][B][H][64], storage type) -> fp32 accumulators; null = zero
template <typename T>
__global__ __launch_bounds__(256) void bw_init_pairs_kernel(const T *__restrict__ gK, const T *__restrict__ gV,
                                                            float *__restrict__ dK, float *__restrict__ dV, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        dK[i] = gK ? to_f32(gK[i]) : 0.f;
        dV[i] = gV ? to_f32(gV[i]) : 0.f;
    }
}

__device__ __forceinline__ float block_sum_256(float v, float *red)
{   // sum over the 256 threads of a workgroup (red: 4 floats of LDS); every thread gets the result
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// ------------------------------------------------------------------------------------------------ (A) recompute
// Row r = n B + b:  v = src[b][n][:] (+ alpha add[r][:]);  rinv = 1 / sqrt(mean(v^2) + eps);  unit = v rinv;
// ng = unit * gain (ng == unit when there is no gain).  norm_free: unit = ng = v, rinv = 1.  grid M, block 256.
template <typename T>
__global__ __launch_bounds__(256) void bw_rows_norm_kernel(const T *__restrict__ src, const float *__restrict__ add, float alpha,
                                                           const T *__restrict__ gain, float *__restrict__ unit,
                                                           float *__restrict__ ng, float *__restrict__ rinv, int B, int N, int d,
                                                           float eps, int norm_free)
{
    __shared__ float red[4];
    const int r = blockIdx.x, n = r / B, b = r % B;
    const T *s = src + ((size_t)b * N + n) * d;
    const float *a = add ? add + (size_t)r * d : nullptr;
    float ss = 0.f;
    for (int k = threadIdx.x; k < d; k += 256) {
        const float v = to_f32(s[k]) + (a ? alpha * a[k] : 0.f);
        ss = fmaf(v, v, ss);
    }
    ss = block_sum_256(ss, red);
    const float ri = norm_free ? 1.f : rsqrtf(ss / (float)d + eps);
    if (threadIdx.x == 0) rinv[r] = ri;
    const bool use_g = gain != nullptr && !norm_free;
    for (int k = threadIdx.x; k < d; k += 256) {
        const float v = to_f32(s[k]) + (a ? alpha * a[k] : 0.f);
        const float u = v * ri;
        unit[(size_t)r * d + k] = u;
        if (ng != unit) ng[(size_t)r * d + k] = use_g ? u * to_f32(gain[k]) : u;
    }
}

// Per-head normalisation of one part of a raw projection: raw[r][col0 + 64 h + lane] -> unit (in place), out = unit * g,
// rh[r][h] = 1 / rms of the head.  rh == null: a value part, copied as it is.  grid (M, H), block 64.
template <typename T>
__global__ __launch_bounds__(64) void bw_head_norm_kernel(float *__restrict__ raw, int ld, int col0, const T *__restrict__ g,
                                                          float *__restrict__ out, float *__restrict__ rh, int H, float eps,
                                                          int norm_free)
{
    const int r = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    const size_t ro = (size_t)r * ld + col0 + h * kHeadDim + lane;
    const size_t oo = ((size_t)r * H + h) * kHeadDim + lane;
    const float v = raw[ro];
    if (rh == nullptr) {
        out[oo] = v;
        return;
    }
    const float ri = norm_free ? 1.f : rsqrtf(wave_sum(v * v) / (float)kHeadDim + eps);
    const float u = v * ri;
    raw[ro] = u;
    out[oo] = (g && !norm_free) ? u * to_f32(g[h * kHeadDim + lane]) : u;
    if (lane == 0) rh[(size_t)r * H + h] = ri;
}

// Attention of every position (Sec. 2.2): query i against the persistent pairs j < i and its own temporary pair.
// One wavefront per (b, h, i); output c (normalised) and the log-sum-exp of the logits.  grid (B H, N), block 64.
__global__ __launch_bounds__(64) void bw_attn_fwd_kernel(const float *__restrict__ Qn, const float *__restrict__ Ktn,
                                                         const float *__restrict__ Vt, const float *__restrict__ Kp,
                                                         const float *__restrict__ Vp, float *__restrict__ c,
                                                         float *__restrict__ lse, int B, int H, float scale, float alibi)
{
    const int bh = blockIdx.x, i = (int)gridDim.y - 1 - (int)blockIdx.y, lane = threadIdx.x;   // long rows first
    const size_t rs = (size_t)B * H * kHeadDim;
    const size_t off = (size_t)i * rs + (size_t)bh * kHeadDim + lane;
    const float q = Qn[off];
    float m = scale * wave_sum(q * Ktn[off]), l = 1.f, o = Vt[off];
    if (i > 0)
        attend_keys<float, false>(q, Kp + (size_t)bh * kHeadDim, Vp + (size_t)bh * kHeadDim, rs, i, scale, m, l, o, nullptr,
                                  alibi_slope(alibi, bh % H, H), i);
    c[off] = o / l;
    if (lane == 0) lse[(size_t)i * B * H + bh] = m + logf(l);
}

// act = gelu(pre), gp = gelu'(pre) (exact erf form); pre and gp may be the same buffer.
__global__ __launch_bounds__(256) void bw_gelu_kernel(const float *pre, float *__restrict__ act, float *gp, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const float p = pre[i];
        const float cdf = 0.5f * (1.0f + erff(p * 0.70710678118654752440f));
        act[i] = p * cdf;
        gp[i] = cdf + p * 0.39894228040143267794f * expf(-0.5f * p * p);
    }
}

// ------------------------------------------------------------------------------------------------ products
// C[i][j] (+)= alpha sum_k A[i a_rs + k a_cs] Bm[j b_rs + k b_cs],  i < M, j < Nn, k < K: any of the layouts the
// backward pass needs (activations times weights, times transposed weights, and sums over rows for the parameter
// gradients) through the strides.  64 x 64 tile per workgroup, k-steps of 16 staged in LDS, 4 x 4 outputs per thread.
// grid (ceil(Nn / 64), ceil(M / 64)), block 256.
__global__ __launch_bounds__(256) void bw_gemm_kernel(const float *__restrict__ A, long a_rs, long a_cs,
                                                      const float *__restrict__ Bm, long b_rs, long b_cs, float *__restrict__ C,
                                                      long c_rs, int M, int Nn, int K, float alpha, int accumulate)
{
    __shared__ float As[16][68], Bs[16][68];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
    float acc[4][4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[r][c] = 0.f;
    for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int e = tid + 256 * s;
            int r, kk;
            if (a_cs == 1) { r = e >> 4; kk = e & 15; } else { kk = e >> 6; r = e & 63; }
            const int gi = i0 + r, gk = k0 + kk;
            As[kk][r] = (gi < M && gk < K) ? A[(size_t)gi * a_rs + (size_t)gk * a_cs] : 0.f;
            if (b_cs == 1) { r = e >> 4; kk = e & 15; } else { kk = e >> 6; r = e & 63; }
            const int gj = j0 + r, gk2 = k0 + kk;
            Bs[kk][r] = (gj < Nn && gk2 < K) ? Bm[(size_t)gj * b_rs + (size_t)gk2 * b_cs] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) a[r] = As[kk][ty + 16 * r];
#pragma unroll
            for (int c = 0; c < 4; ++c) b[c] = Bs[kk][tx + 16 * c];
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[r][c] = fmaf(a[r], b[c], acc[r][c]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int gi = i0 + ty + 16 * r;
        if (gi >= M) continue;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int gj = j0 + tx + 16 * c;
            if (gj < Nn) {
                float *p = C + (size_t)gi * c_rs + gj;
                *p = accumulate ? *p + alpha * acc[r][c] : alpha * acc[r][c];
            }
        }
    }
}

static void gemm(hipStream_t st, const float *A, long a_rs, long a_cs, const float *Bm, long b_rs, long b_cs, float *C, long c_rs,
                 int M, int Nn, int K, float alpha, bool accumulate)
{
    hipLaunchKernelGGL(bw_gemm_kernel, dim3((unsigned)((Nn + 63) / 64), (unsigned)((M + 63) / 64)), dim3(256), 0, st, A, a_rs, a_cs,
                       Bm, b_rs, b_cs, C, c_rs, M, Nn, K, alpha, accumulate ? 1 : 0);
}


// ------------------------------------------------------------------------------------------------ matrix-core products
// C[m][n] (+)= alpha sum_k A[m][k] W[n][k] with A, W bf16 and the contraction index contiguous in both (rows lda, ldb
// apart, K a multiple of 64), fp32 C, on the LDS-tiled main loop of the loop-free layers (256 x 128 block tile).
// blockIdx.z = contraction slice (the parameter gradients contract over all B N rows but have few outputs): slice z
// covers k in [z Ks, (z + 1) Ks) and, when gridDim.z > 1, writes its tile to part + z * M * Nn (dense, reduced afterwards).
__global__ __launch_bounds__(256) void bw_mm_kernel(const bf16_t *__restrict__ A, size_t lda, const bf16_t *__restrict__ W, size_t ldb,
                                                    float *__restrict__ C, size_t ldc, float *__restrict__ part, int M, int Nn, int Ks,
                                                    float alpha, int accumulate)
{
    __shared__ __align__(16) bf16_t As[kGtRows * kGtLd];
    __shared__ __align__(16) bf16_t Bs[kGtCols * kGtLd];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, hi = lane >> 5;
    const int m0 = blockIdx.x * kGtRows, nb0 = blockIdx.y * kGtCols;
    const size_t k0 = (size_t)blockIdx.z * Ks;
    const int prow = tid >> 3, pc = tid & 7;
    const bf16_t *ga[8], *gb[4];
#pragma unroll
    for (int i = 0; i < 8; ++i) ga[i] = A + (size_t)min(m0 + prow + 32 * i, M - 1) * lda + k0 + pc * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) gb[i] = W + (size_t)min(nb0 + prow + 32 * i, Nn - 1) * ldb + k0 + pc * 8;
    f32x16_t acc[4][2];
    tiled_mainloop(ga, gb, nullptr, Ks, As, Bs, acc);
    const bool split = gridDim.z > 1;
    float *out = split ? part + (size_t)blockIdx.z * M * Nn : C;
    const size_t ldo = split ? (size_t)Nn : ldc;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int m = m0 + wm * 128 + mt * 32 + 8 * (i / 4) + 4 * hi + (i % 4);
            if (m >= M) continue;
#pragma unroll
            for (int nt = 0; nt < 2; ++nt) {
                const int n = nb0 + wn * 64 + nt * 32 + l32;
                if (n >= Nn) continue;
                float *p = out + (size_t)m * ldo + n;
                if (split) *p = acc[mt][nt][i];
                else *p = accumulate ? *p + alpha * acc[mt][nt][i] : alpha * acc[mt][nt][i];
            }
        }
}

// C[m][n] (+)= alpha sum_z part[z][m][n]  (fixed order: runs are bit-reproducible)
__global__ __launch_bounds__(256) void bw_mm_reduce_kernel(const float *__restrict__ part, int S, float *__restrict__ C, size_t ldc,
                                                           int M, int Nn, float alpha, int accumulate)
{
    const size_t n_el = (size_t)M * Nn;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n_el; e += (size_t)gridDim.x * 256) {
        float s = 0.f;
        for (int z = 0; z < S; ++z) s += part[(size_t)z * n_el + e];
        float *p = C + (e / Nn) * ldc + e % Nn;
        *p = accumulate ? *p + alpha * s : alpha * s;
    }
}

// fp32 rows -> bf16 head (and, if lo is given, the bf16 remainder v - head): in [R][ldi], out [R][ldo]
__global__ __launch_bounds__(256) void bw_split_rows_kernel(const float *__restrict__ in, size_t ldi, bf16_t *__restrict__ hi_out,
                                                            bf16_t *__restrict__ lo_out, size_t ldo, int R, int Cn)
{
    const size_t n_el = (size_t)R * Cn;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n_el; e += (size_t)gridDim.x * 256) {
        const size_t r = e / Cn, c = e % Cn;
        const float v = in[r * ldi + c];
        const bf16_t h = f32_to_bf16(v);
        hi_out[r * ldo + c] = h;
        if (lo_out) lo_out[r * ldo + c] = f32_to_bf16(v - bf16_to_f32(h));
    }
}

// fp32 [R][ldi] (columns c0 .. c0 + Cn - 1) -> bf16 transposed [Cn][ldo], columns R .. Rp - 1 of the output zero.
// grid (ceil(Rp / 64), ceil(Cn / 64)), block 256.
__global__ __launch_bounds__(256) void bw_transpose_bf16_kernel(const float *__restrict__ in, size_t ldi, int c0, bf16_t *__restrict__ out,
                                                                size_t ldo, int R, int Rp, int Cn)
{
    __shared__ float tile[64][65];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int r0 = blockIdx.x * 64, cb = blockIdx.y * 64;
    for (int j = ty; j < 64; j += 4) {
        const int r = r0 + j, c = cb + tx;
        tile[j][tx] = (r < R && c < Cn) ? in[(size_t)r * ldi + c0 + c] : 0.f;
    }
    __syncthreads();
    for (int j = ty; j < 64; j += 4) {
        const int c = cb + j, r = r0 + tx;
        if (c < Cn && r < Rp) out[(size_t)c * ldo + r] = f32_to_bf16(tile[tx][j]);
    }
}

// small-M product of the reverse loop: out[b][o] = epilogue(sum_k W[o][k] in[b][k]) with the forward's gemv_body
template <typename T> struct OneMatrix {
    const T *W;
    int n_in;
    __device__ __forceinline__ const T *row(int o) const { return W + (size_t)o * n_in; }
    __device__ __forceinline__ const T *gain() const { return nullptr; }
};

template <typename T, int EPI, int KS>
__global__ __launch_bounds__(256) void bw_gemv_kernel(const T *__restrict__ W, int n_out, int n_in, const float *__restrict__ in,
                                                      size_t in_stride, int Bn, const float *__restrict__ res_f,
                                                      float *__restrict__ out_f)
{
    __shared__ float part[4][kGemvPart];
    const OneMatrix<T> rows{W, n_in};
    gemv_body<T, float, EPI, KS>(rows, blockIdx.x, n_out, n_in, in, in_stride, Bn, 0.f, 0, 1.f, (const T *)nullptr, 0, res_f, out_f,
                                 (T *)nullptr, 0, part);
}

template <typename T, int EPI>
static void gemv(hipStream_t st, const T *W, int n_out, int n_in, const float *in, size_t in_stride, int B, const float *res_f,
                 float *out_f)
{
    for (int b0 = 0; b0 < B; b0 += kBatchTile) {
        const int Bn = (B - b0 < kBatchTile) ? B - b0 : kBatchTile;
        const float *rf = res_f ? res_f + (size_t)b0 * n_out : nullptr;
        if (n_in <= 1024)
            hipLaunchKernelGGL((bw_gemv_kernel<T, EPI, 2>), dim3((n_out + 2 * kGemvRows - 1) / (2 * kGemvRows)), dim3(256), 0, st, W,
                               n_out, n_in, in + (size_t)b0 * in_stride, in_stride, Bn, rf, out_f + (size_t)b0 * n_out);
        else
            hipLaunchKernelGGL((bw_gemv_kernel<T, EPI, 4>), dim3((n_out + kGemvRows - 1) / kGemvRows), dim3(256), 0, st, W, n_out,
                               n_in, in + (size_t)b0 * in_stride, in_stride, Bn, rf, out_f + (size_t)b0 * n_out);
    }
}

// ------------------------------------------------------------------------------------------------ (B) reverse loop
// Position i, one wavefront per (b, h): dK_i, dV_i are complete.  Through the per-head normalisation of the persistent
// key (k = unit * g_k, unit = raw * rk):  dkraw = rk (w - unit mean(unit w)), w = dK_i g_k.  Writes dkraw of the row
// and the input [dkraw | dV_i] of the product with [Wk; Wv]^T.  grid B H, block 64.
template <typename T>
__global__ __launch_bounds__(64) void bw_pair_grad_kernel(const float *__restrict__ dK, const float *__restrict__ dV,
                                                          const float *__restrict__ unit_k, const float *__restrict__ rk,
                                                          const T *__restrict__ g_k, float *__restrict__ dkraw,
                                                          float *__restrict__ in_kv, int i, int B, int H, int norm_free)
{
    const int bh = blockIdx.x, b = bh / H, h = bh % H, lane = threadIdx.x;
    const int d = H * kHeadDim;
    const size_t r = (size_t)i * B + b;
    const size_t off = r * d + h * kHeadDim + lane;
    const float dk = dK[off];
    float du = dk;
    if (!norm_free) {
        const float w = g_k ? dk * to_f32(g_k[h * kHeadDim + lane]) : dk;
        const float u = unit_k[r * 2 * d + h * kHeadDim + lane];
        du = rk[r * H + h] * (w - u * (wave_sum(u * w) / (float)kHeadDim));
    }
    dkraw[off] = du;
    in_kv[(size_t)b * 2 * d + h * kHeadDim + lane] = du;
    in_kv[(size_t)b * 2 * d + d + h * kHeadDim + lane] = dV[off];
}

// out_row = base_row + rinv (w - unit mean(unit w)), w = g_in * gain: the transpose Jacobian of RMS applied to the
// gradient g_in of the normalised row, added to `base` (gy_i for dz_i: T storage [B][N][d]; Gz for dh_i: fp32 rows).
// Also out_scaled[b] = alpha * out_row, the input of the next product.  grid B, block 256.
template <typename T, typename BASE_T>
__global__ __launch_bounds__(256) void bw_norm_bw_row_kernel(const float *__restrict__ g_in, const float *__restrict__ unit,
                                                             const float *__restrict__ rinv, const T *__restrict__ gain,
                                                             const BASE_T *__restrict__ base, size_t base_bstride,
                                                             float *__restrict__ out_row, float *__restrict__ out_scaled,
                                                             float alpha, int i, int B, int d, int norm_free)
{
    __shared__ float red[4];
    constexpr int kPer = 8;   // elements per thread held in registers: every load of the row is issued before the reduction
    const int b = blockIdx.x;
    const size_t r = (size_t)i * B + b;
    const float *gi = g_in + r * d, *un = unit + r * d;
    const BASE_T *bs = base + (size_t)b * base_bstride;
    const bool use_g = gain != nullptr && !norm_free;
    const float ri = rinv[r];
    if (d <= 256 * kPer) {
        float w[kPer], u[kPer], bv[kPer];
#pragma unroll
        for (int e = 0; e < kPer; ++e) {
            const int k = threadIdx.x + 256 * e;
            const bool in = k < d;
            const float g = in ? gi[k] : 0.f;
            w[e] = (use_g && in) ? g * to_f32(gain[k]) : g;
            u[e] = in ? un[k] : 0.f;
            bv[e] = in ? to_f32(bs[k]) : 0.f;
        }
        float dot = 0.f;
        if (!norm_free) {
#pragma unroll
            for (int e = 0; e < kPer; ++e) dot = fmaf(u[e], w[e], dot);
            dot = block_sum_256(dot, red) / (float)d;
        }
#pragma unroll
        for (int e = 0; e < kPer; ++e) {
            const int k = threadIdx.x + 256 * e;
            if (k < d) {
                const float v = bv[e] + (norm_free ? w[e] : ri * (w[e] - u[e] * dot));
                out_row[r * d + k] = v;
                out_scaled[(size_t)b * d + k] = alpha * v;
            }
        }
        return;
    }
    float dot = 0.f;
    if (!norm_free) {
        for (int k = threadIdx.x; k < d; k += 256) dot = fmaf(un[k], use_g ? gi[k] * to_f32(gain[k]) : gi[k], dot);
        dot = block_sum_256(dot, red) / (float)d;
    }
    for (int k = threadIdx.x; k < d; k += 256) {
        const float w = use_g ? gi[k] * to_f32(gain[k]) : gi[k];
        const float v = to_f32(bs[k]) + (norm_free ? w : ri * (w - un[k] * dot));
        out_row[r * d + k] = v;
        out_scaled[(size_t)b * d + k] = alpha * v;
    }
}

// Softmax backward of query i for its own temporary pair and its window (the persistent keys of the positions
// i - (i mod kBwPmin) .. i - 1), one wavefront per (b, h):
//   Dsum = <dc, c>;  p = exp(logit - lse);  dp = <dc, v>;  ds = p (dp - Dsum);
//   dV_j += p_j dc,  dK_j += scale ds_j q   (window keys);   dvt_i = p_own dc,  dkt_i = scale ds_own q,
//   dq_i = scale ds_own kt_i (the keys' share of dq_i is added after the loop).  grid B H, block 64.
template <typename T>
__global__ __launch_bounds__(64) void bw_attn_row_kernel(const float *__restrict__ Qn, const float *__restrict__ Ktn,
                                                         const float *__restrict__ Vt, const float *__restrict__ Kp,
                                                         const float *__restrict__ Vp, const float *__restrict__ cbuf,
                                                         const float *__restrict__ dc, const float *__restrict__ lse,
                                                         float *__restrict__ Ds, float *dK, float *dV,
                                                         float *__restrict__ dq, float *__restrict__ dkt, float *__restrict__ dvt,
                                                         int i, int B, int H, float scale, float alibi,
                                                         // when fuse_pair: the per-head normalisation backward of position i - 1
                                                         // (bw_pair_grad_kernel's work) by the same wavefront, whose own window
                                                         // update was the last contribution to dK, dV of that position
                                                         int fuse_pair, const float *__restrict__ unit_k, const float *__restrict__ rk,
                                                         const T *__restrict__ g_k, float *__restrict__ dkraw, float *__restrict__ in_kv,
                                                         int norm_free)
{
    const int bh = blockIdx.x, lane = threadIdx.x;
    const size_t rs = (size_t)B * H * kHeadDim;
    const size_t off = (size_t)i * rs + (size_t)bh * kHeadDim + lane;
    const float q = Qn[off], kt = Ktn[off], vt = Vt[off], g = dc[off], cv = cbuf[off];
    const float L = lse[(size_t)i * B * H + bh];
    const float Dsum = wave_sum(g * cv);
    const float p_own = expf(scale * wave_sum(q * kt) - L);
    const float ds_own = p_own * (wave_sum(g * vt) - Dsum);
    dvt[off] = p_own * g;
    dkt[off] = scale * ds_own * q;
    dq[off] = scale * ds_own * kt;
    if (lane == 0) Ds[(size_t)i * B * H + bh] = Dsum;
    const int w = i & (kBwPmin - 1);
    float dk_prev = 0.f, dv_prev = 0.f;   // dK, dV of position i - 1 after this query's update (fuse_pair needs w > 0)
    if (w > 0) {
        const int j0 = i - w;
        const size_t kb = (size_t)(j0 + min(lane, w - 1)) * rs + (size_t)bh * kHeadDim;   // lane j < w owns key j0 + j
        float s = 0.f, dp = 0.f;
#pragma unroll
        for (int c8 = 0; c8 < 8; ++c8) {
            float kk[8], vv[8];
            load8(Kp + kb + c8 * 8, kk);
            load8(Vp + kb + c8 * 8, vv);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                s = fmaf(lane_bcast(q, c8 * 8 + e), kk[e], s);
                dp = fmaf(lane_bcast(g, c8 * 8 + e), vv[e], dp);
            }
        }
        const float slope = alibi_slope(alibi, bh % H, H);
        const float p = lane < w ? expf(fmaf(-slope, (float)(w - lane), s * scale) - L) : 0.f;
        const float ds = p * (dp - Dsum);
        // eight rows at a time: all their loads are issued before the first store (the rows are distinct)
        for (int jb = 0; jb < w; jb += 8) {
            float av[8], ak[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const size_t o = (size_t)(j0 + min(jb + e, w - 1)) * rs + (size_t)bh * kHeadDim + lane;
                av[e] = dV[o];
                ak[e] = dK[o];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int j = jb + e;
                if (j < w) {   // wave-uniform
                    const size_t o = (size_t)(j0 + j) * rs + (size_t)bh * kHeadDim + lane;
                    const float nv = fmaf(lane_bcast(p, j), g, av[e]);
                    const float nk = fmaf(scale * lane_bcast(ds, j), q, ak[e]);
                    dV[o] = nv;
                    dK[o] = nk;
                    if (j == w - 1) { dv_prev = nv; dk_prev = nk; }
                }
            }
        }
    }
    if (fuse_pair && w > 0) {
        const int b = bh / H, h = bh % H, d = H * kHeadDim;
        const size_t r = (size_t)(i - 1) * B + b;
        const size_t po = r * d + h * kHeadDim + lane;
        float du = dk_prev;
        if (!norm_free) {
            const float wv = g_k ? dk_prev * to_f32(g_k[h * kHeadDim + lane]) : dk_prev;
            const float u = unit_k[r * 2 * d + h * kHeadDim + lane];
            du = rk[r * H + h] * (wv - u * (wave_sum(u * wv) / (float)kHeadDim));
        }
        dkraw[po] = du;
        in_kv[(size_t)b * 2 * d + h * kHeadDim + lane] = du;
        in_kv[(size_t)b * 2 * d + d + h * kHeadDim + lane] = dv_prev;
    }
}

// One block of Algorithm 1 backwards: the keys [k0, k0 + P) receive the contribution of the queries [q0, q0 + nq).
// A workgroup owns 64 keys of one (b, h) (K, V rows in LDS) and walks the queries in chunks of 64:
//   S = K Q^T, dP = V dC^T  ->  Pm = exp(scale S - bias - lse_q), dS = Pm (dP - Dsum_q)   (64 x 64, in LDS)
//   dV += Pm dC,  dK += scale dS Q     (accumulated in registers, added to the global rows at the end)
// thread (tx, ty) = (tid % 16, tid / 16): keys ty + 16 kk, queries / columns tx + 16 qq.  grid (ceil(P / 64), B H), block 256.
__global__ __launch_bounds__(256) void bw_event_kernel(const float *__restrict__ Qn, const float *__restrict__ Kp,
                                                       const float *__restrict__ Vp, const float *__restrict__ dc,
                                                       const float *__restrict__ lse, const float *__restrict__ Ds,
                                                       float *__restrict__ dK, float *__restrict__ dV, int B, int H, int k0, int P,
                                                       int q0, int nq, float scale, float alibi)
{
    extern __shared__ __align__(16) float ev_lds[];
    float *Ks = ev_lds, *Vs = Ks + 64 * kTileLdF, *Qs = Vs + 64 * kTileLdF, *Cs = Qs + 64 * kTileLdF;
    float *Ps = Cs + 64 * kTileLdF, *Ss = Ps + 64 * kTileLdF, *lse_s = Ss + 64 * kTileLdF, *ds_s = lse_s + 64;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int bh = blockIdx.y, kb = k0 + blockIdx.x * 64, nk = min(64, k0 + P - kb);
    const size_t rs = (size_t)B * H * kHeadDim;
    const float slope = alibi_slope(alibi, bh % H, H);
    for (int e = tid; e < 64 * 64; e += 256) {
        const int r = e >> 6, c = e & 63;
        const size_t o = (size_t)(kb + min(r, nk - 1)) * rs + (size_t)bh * kHeadDim + c;
        Ks[r * kTileLdF + c] = r < nk ? Kp[o] : 0.f;
        Vs[r * kTileLdF + c] = r < nk ? Vp[o] : 0.f;
    }
    float adv[4][4], adk[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int c = 0; c < 4; ++c) adv[a][c] = adk[a][c] = 0.f;
    for (int qc = 0; qc < nq; qc += 64) {
        const int nqc = min(64, nq - qc);
        __syncthreads();   // the previous chunk's tiles are no longer read
        for (int e = tid; e < 64 * 64; e += 256) {
            const int r = e >> 6, c = e & 63;
            const size_t o = (size_t)(q0 + qc + min(r, nqc - 1)) * rs + (size_t)bh * kHeadDim + c;
            Qs[r * kTileLdF + c] = r < nqc ? Qn[o] : 0.f;
            Cs[r * kTileLdF + c] = r < nqc ? dc[o] : 0.f;
        }
        if (tid < 64) {
            const size_t o = (size_t)(q0 + qc + min(tid, nqc - 1)) * B * H + bh;
            lse_s[tid] = lse[o];
            ds_s[tid] = Ds[o];
        }
        __syncthreads();
        float s[4][4], dp[4][4];
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int c = 0; c < 4; ++c) s[a][c] = dp[a][c] = 0.f;
        for (int c = 0; c < 64; ++c) {
            float kv[4], vv[4], qv[4], gv[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                kv[a] = Ks[(ty + 16 * a) * kTileLdF + c];
                vv[a] = Vs[(ty + 16 * a) * kTileLdF + c];
                qv[a] = Qs[(tx + 16 * a) * kTileLdF + c];
                gv[a] = Cs[(tx + 16 * a) * kTileLdF + c];
            }
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b2 = 0; b2 < 4; ++b2) {
                    s[a][b2] = fmaf(kv[a], qv[b2], s[a][b2]);
                    dp[a][b2] = fmaf(vv[a], gv[b2], dp[a][b2]);
                }
        }
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b2 = 0; b2 < 4; ++b2) {
                const int key = ty + 16 * a, qi = tx + 16 * b2;
                const bool valid = key < nk && qi < nqc;
                const float dist = (float)((q0 + qc + qi) - (kb + key));
                const float p = valid ? expf(fmaf(-slope, dist, scale * s[a][b2]) - lse_s[qi]) : 0.f;
                Ps[key * kTileLdF + qi] = p;
                Ss[key * kTileLdF + qi] = p * (dp[a][b2] - ds_s[qi]);
            }
        __syncthreads();
        for (int qi = 0; qi < 64; ++qi) {
            float pk[4], sk[4], gc[4], qcv[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                pk[a] = Ps[(ty + 16 * a) * kTileLdF + qi];
                sk[a] = Ss[(ty + 16 * a) * kTileLdF + qi];
                gc[a] = Cs[qi * kTileLdF + tx + 16 * a];
                qcv[a] = Qs[qi * kTileLdF + tx + 16 * a];
            }
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    adv[a][c] = fmaf(pk[a], gc[c], adv[a][c]);
                    adk[a][c] = fmaf(sk[a], qcv[c], adk[a][c]);
                }
        }
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int key = ty + 16 * a;
        if (key >= nk) continue;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const size_t o = (size_t)(kb + key) * rs + (size_t)bh * kHeadDim + tx + 16 * c;
            dV[o] += adv[a][c];
            dK[o] = fmaf(scale, adk[a][c], dK[o]);
        }
    }
}
constexpr size_t kEventLds = (size_t)(6 * 64 * kTileLdF + 128) * 4;

// ------------------------------------------------------------------------------------------------ (C) after the loop
// dq of 64 queries of one (b, h) over all persistent keys before them: dq_i += scale sum_{j < i} dS_ij k_j with dS as
// above (every quantity of every position is known now).  grid (ceil(N / 64), B H), block 256.
__global__ __launch_bounds__(256) void bw_dq_kernel(const float *__restrict__ Qn, const float *__restrict__ Kp,
                                                    const float *__restrict__ Vp, const float *__restrict__ dc,
                                                    const float *__restrict__ lse, const float *__restrict__ Ds,
                                                    float *__restrict__ dq, int B, int H, int N, float scale, float alibi)
{
    extern __shared__ __align__(16) float ev_lds[];
    float *Ks = ev_lds, *Vs = Ks + 64 * kTileLdF, *Qs = Vs + 64 * kTileLdF, *Cs = Qs + 64 * kTileLdF;
    float *Ss = Cs + 64 * kTileLdF, *lse_s = Ss + 64 * kTileLdF, *ds_s = lse_s + 64;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int bh = blockIdx.y, qb = ((int)gridDim.x - 1 - (int)blockIdx.x) * 64, nqc = min(64, N - qb);   // long blocks first
    const size_t rs = (size_t)B * H * kHeadDim;
    const float slope = alibi_slope(alibi, bh % H, H);
    for (int e = tid; e < 64 * 64; e += 256) {
        const int r = e >> 6, c = e & 63;
        const size_t o = (size_t)(qb + min(r, nqc - 1)) * rs + (size_t)bh * kHeadDim + c;
        Qs[r * kTileLdF + c] = r < nqc ? Qn[o] : 0.f;
        Cs[r * kTileLdF + c] = r < nqc ? dc[o] : 0.f;
    }
    if (tid < 64) {
        const size_t o = (size_t)(qb + min(tid, nqc - 1)) * B * H + bh;
        lse_s[tid] = lse[o];
        ds_s[tid] = Ds[o];
    }
    float acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[a][c] = 0.f;
    const int kend = qb + nqc - 1;   // keys 0 .. kend - 1 precede some query of the block
    for (int kc = 0; kc < kend; kc += 64) {
        const int nk = min(64, kend - kc);
        __syncthreads();
        for (int e = tid; e < 64 * 64; e += 256) {
            const int r = e >> 6, c = e & 63;
            const size_t o = (size_t)(kc + min(r, nk - 1)) * rs + (size_t)bh * kHeadDim + c;
            Ks[r * kTileLdF + c] = r < nk ? Kp[o] : 0.f;
            Vs[r * kTileLdF + c] = r < nk ? Vp[o] : 0.f;
        }
        __syncthreads();
        float s[4][4], dp[4][4];
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int c = 0; c < 4; ++c) s[a][c] = dp[a][c] = 0.f;
        for (int c = 0; c < 64; ++c) {
            float kv[4], vv[4], qv[4], gv[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                kv[a] = Ks[(ty + 16 * a) * kTileLdF + c];
                vv[a] = Vs[(ty + 16 * a) * kTileLdF + c];
                qv[a] = Qs[(tx + 16 * a) * kTileLdF + c];
                gv[a] = Cs[(tx + 16 * a) * kTileLdF + c];
            }
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b2 = 0; b2 < 4; ++b2) {
                    s[a][b2] = fmaf(kv[a], qv[b2], s[a][b2]);
                    dp[a][b2] = fmaf(vv[a], gv[b2], dp[a][b2]);
                }
        }
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b2 = 0; b2 < 4; ++b2) {
                const int key = ty + 16 * a, qi = tx + 16 * b2;
                const int dist = (qb + qi) - (kc + key);
                const bool valid = key < nk && qi < nqc && dist > 0;
                const float p = valid ? expf(fmaf(-slope, (float)dist, scale * s[a][b2]) - lse_s[qi]) : 0.f;
                Ss[key * kTileLdF + qi] = p * (dp[a][b2] - ds_s[qi]);
            }
        __syncthreads();
        // dq[query ty + 16 a][column tx + 16 c] += sum_key dS[key][query] K[key][column]
        for (int key = 0; key < 64; ++key) {
            float sq[4], kc4[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                sq[a] = Ss[key * kTileLdF + ty + 16 * a];
                kc4[a] = Ks[key * kTileLdF + tx + 16 * a];
            }
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[a][c] = fmaf(sq[a], kc4[c], acc[a][c]);
        }
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int qi = ty + 16 * a;
        if (qi >= nqc) continue;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const size_t o = (size_t)(qb + qi) * rs + (size_t)bh * kHeadDim + tx + 16 * c;
            dq[o] = fmaf(scale, acc[a][c], dq[o]);
        }
    }
}
constexpr size_t kDqLds = (size_t)(5 * 64 * kTileLdF + 128) * 4;

// Transpose Jacobian of the per-head normalisation for every row: out[r][colo + 64 h + lane] = rh (w - unit mean(unit w)),
// w = dy g; rh == null: a value part, copied.  unit rows are `ldu` apart starting at column colu.  grid (M, H), block 64.
template <typename T>
__global__ __launch_bounds__(64) void bw_head_norm_bw_kernel(const float *__restrict__ dy, const float *__restrict__ unit, int ldu,
                                                             int colu, const float *__restrict__ rh, const T *__restrict__ g,
                                                             float *__restrict__ out, int ldo, int colo, int H, int norm_free)
{
    const int r = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    const float v = dy[((size_t)r * H + h) * kHeadDim + lane];
    float du = v;
    if (rh != nullptr && !norm_free) {
        const float w = g ? v * to_f32(g[h * kHeadDim + lane]) : v;
        const float u = unit[(size_t)r * ldu + colu + h * kHeadDim + lane];
        du = rh[(size_t)r * H + h] * (w - u * (wave_sum(u * w) / (float)kHeadDim));
    }
    out[(size_t)r * ldo + colo + h * kHeadDim + lane] = du;
}

// dx[b][n][:] = dh[r][:] + rinv_x (w - unit_x mean(unit_x w)), w = dn g_attn.  grid M, block 256.
template <typename T>
__global__ __launch_bounds__(256) void bw_dx_kernel(const float *__restrict__ dn, const float *__restrict__ unit,
                                                    const float *__restrict__ rinv, const T *__restrict__ gain,
                                                    const float *__restrict__ dh, float *__restrict__ dx, int B, int N, int d,
                                                    int norm_free)
{
    __shared__ float red[4];
    const int r = blockIdx.x, n = r / B, b = r % B;
    const float *gi = dn + (size_t)r * d, *un = unit + (size_t)r * d;
    const bool use_g = gain != nullptr && !norm_free;
    float dot = 0.f;
    if (!norm_free) {
        for (int k = threadIdx.x; k < d; k += 256) dot = fmaf(un[k], use_g ? gi[k] * to_f32(gain[k]) : gi[k], dot);
        dot = block_sum_256(dot, red) / (float)d;
    }
    const float ri = rinv[r];
    float *o = dx + ((size_t)b * N + n) * d;
    for (int k = threadIdx.x; k < d; k += 256) {
        const float w = use_g ? gi[k] * to_f32(gain[k]) : gi[k];
        o[k] = dh[(size_t)r * d + k] + (norm_free ? w : ri * (w - un[k] * dot));
    }
}

// out[col] (+)= sum_r A[r lda + col] Bm[r ldb + col]  (gain gradients: column sums of gradient times normalised value).
// grid ceil(ncol / 64), block 256 (four row phases per column, joined in LDS in a fixed order).
__global__ __launch_bounds__(256) void bw_colsum_kernel(const float *__restrict__ A, size_t lda, const float *__restrict__ Bm,
                                                        size_t ldb, int M, int ncol, float *__restrict__ out, int accumulate)
{
    __shared__ float part[4][64];
    const int cx = threadIdx.x & 63, ry = threadIdx.x >> 6, col = blockIdx.x * 64 + cx;
    float s = 0.f;
    if (col < ncol)
        for (int r = ry; r < M; r += 4) s = fmaf(A[(size_t)r * lda + col], Bm[(size_t)r * ldb + col], s);
    part[ry][cx] = s;
    __syncthreads();
    if (ry == 0 && col < ncol) {
        const float t = (part[0][cx] + part[1][cx]) + (part[2][cx] + part[3][cx]);
        out[col] = accumulate ? out[col] + t : t;
    }
}

// ------------------------------------------------------------------------------------------------ host side
namespace {
struct Carver {
    char *base;
    size_t off = 0;
    template <typename U> U *take(size_t count)
    {
        const size_t o = off;
        off = (off + count * sizeof(U) + 255) / 256 * 256;
        return base ? reinterpret_cast<U *>(base + o) : nullptr;
    }
};

struct BwBufs {
    float *Wqkv_f, *Wo_f, *W1_f, *W2_f;
    void *WkvT, *W2T, *W1T, *WoT;
    float *unit_x, *nxg, *rinv_x, *unit_z, *nzg, *rinv_z;
    float *qkv, *Qn, *Ktn, *Vt, *rq, *rkt;       // qkv: [M][3d] raw -> unit (q, k parts)
    float *kv, *Kp, *Vp, *rk;                    // kv: [M][2d] raw -> unit (k part)
    float *c, *lse, *a, *unit_h, *hg, *rinv_h, *gp, *act;
    float *dK, *dV, *in_kv, *dkraw, *d_rz, *Gz, *dmo, *dpre, *t1, *d_h, *da, *dc, *Ds, *dq, *dkt, *dvt;
    float *G3, *dn;
    // matrix-core path (bf16 storage): bf16 copies of the products' operands
    bf16_t *op_hi, *op_lo;   // [M][d] head and remainder of the recompute's activations, one product at a time
    bf16_t *G3_b;            // [M][3d]
    bf16_t *WqkvT_b;         // [d][3d]
    bf16_t *tA, *tB;         // transposed operands of the parameter sums, [rows][Mp]
    float *part;             // contraction slices of a parameter sum
    // single-launch reverse loop: the loop-independent halves of its products (rt_backward_persistent.hip) and its
    // exchange words
    bf16_t *gy_pf;           // [M][d] gy with position-first rows
    float *A_gy, *A_uz;      // [M][F]
    float *C_gy, *C_uz, *C_uh;   // [M][d]
    char *flash;             // bf16 copies of the pairs for the recompute's attention on the matrix cores
    char *exchange;
};

// contraction slices of the parameter sums over M rows: as many as keep 512 rows and more per slice, at most 16
int bw_slices(size_t M)
{
    int S = 1;
    while (S < 16 && M / (2 * (size_t)S) >= 512) S *= 2;
    return S;
}

size_t carve_bufs(BwBufs &Bf, char *base, size_t B, size_t N, size_t d, size_t F, size_t H, size_t E, bool gains)
{
    Carver cv{base};
    const size_t M = B * N;
    // the exchange words of the single-launch loop come first: their place does not depend on the call's B and N
    // (they are zeroed once, when the scratch is allocated)
    Bf.exchange = E == 2 ? cv.take<char>(bwp_exchange_bytes((int)d, (int)F)) : nullptr;
    Bf.Wqkv_f = cv.take<float>(3 * d * d); Bf.Wo_f = cv.take<float>(d * d); Bf.W1_f = cv.take<float>(F * d); Bf.W2_f = cv.take<float>(d * F);
    Bf.WkvT = cv.take<char>(2 * d * d * E); Bf.W2T = cv.take<char>(F * d * E); Bf.W1T = cv.take<char>(d * F * E); Bf.WoT = cv.take<char>(d * d * E);
    Bf.unit_x = cv.take<float>(M * d); Bf.nxg = gains ? cv.take<float>(M * d) : Bf.unit_x; Bf.rinv_x = cv.take<float>(M);
    Bf.unit_z = cv.take<float>(M * d); Bf.nzg = gains ? cv.take<float>(M * d) : Bf.unit_z; Bf.rinv_z = cv.take<float>(M);
    Bf.qkv = cv.take<float>(M * 3 * d); Bf.Qn = cv.take<float>(M * d); Bf.Ktn = cv.take<float>(M * d); Bf.Vt = cv.take<float>(M * d);
    Bf.rq = cv.take<float>(M * H); Bf.rkt = cv.take<float>(M * H);
    Bf.kv = cv.take<float>(M * 2 * d); Bf.Kp = cv.take<float>(M * d); Bf.Vp = cv.take<float>(M * d); Bf.rk = cv.take<float>(M * H);
    Bf.c = cv.take<float>(M * d); Bf.lse = cv.take<float>(M * H); Bf.a = cv.take<float>(M * d);
    Bf.unit_h = cv.take<float>(M * d); Bf.hg = gains ? cv.take<float>(M * d) : Bf.unit_h; Bf.rinv_h = cv.take<float>(M);
    Bf.gp = cv.take<float>(M * F); Bf.act = cv.take<float>(M * F);
    Bf.dK = cv.take<float>(M * d); Bf.dV = cv.take<float>(M * d); Bf.in_kv = cv.take<float>(B * 2 * d); Bf.dkraw = cv.take<float>(M * d);
    Bf.d_rz = cv.take<float>(M * d); Bf.Gz = cv.take<float>(M * d); Bf.dmo = cv.take<float>(B * d); Bf.dpre = cv.take<float>(M * F);
    Bf.t1 = cv.take<float>(M * d); Bf.d_h = cv.take<float>(M * d); Bf.da = cv.take<float>(B * d); Bf.dc = cv.take<float>(M * d);
    Bf.Ds = cv.take<float>(M * H); Bf.dq = cv.take<float>(M * d); Bf.dkt = cv.take<float>(M * d); Bf.dvt = cv.take<float>(M * d);
    Bf.G3 = cv.take<float>(M * 3 * d); Bf.dn = cv.take<float>(M * d);
    const size_t Mp = M + 64 * 16, wide = 3 * d > F ? 3 * d : F;
    Bf.op_hi = cv.take<bf16_t>(M * d); Bf.op_lo = cv.take<bf16_t>(M * d);
    Bf.G3_b = cv.take<bf16_t>(M * 3 * d); Bf.WqkvT_b = cv.take<bf16_t>(3 * d * d);
    Bf.tA = cv.take<bf16_t>(wide * Mp); Bf.tB = cv.take<bf16_t>((F > d ? F : d) * Mp);
    Bf.part = cv.take<float>(16 * d * d > 4 * F * d ? 16 * d * d : 4 * F * d);
    if (E == 2) {
        Bf.gy_pf = cv.take<bf16_t>(M * d);
        Bf.A_gy = cv.take<float>(M * F); Bf.A_uz = cv.take<float>(M * F);
        Bf.C_gy = cv.take<float>(M * d); Bf.C_uz = cv.take<float>(M * d); Bf.C_uh = cv.take<float>(M * d);
        Bf.flash = cv.take<char>(flash_recompute_scratch_bytes(B, N, d, H));
    } else {
        Bf.gy_pf = nullptr; Bf.A_gy = Bf.A_uz = Bf.C_gy = Bf.C_uz = Bf.C_uh = nullptr;
        Bf.flash = nullptr;
    }
    return cv.off;
}

bool g_lds_raised = false;
hipError_t raise_lds()
{
    if (g_lds_raised) return hipSuccess;
    hipError_t e = hipFuncSetAttribute((const void *)bw_event_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kEventLds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)bw_dq_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kDqLds);
    if (e != hipSuccess) return e;
    g_lds_raised = true;
    return hipSuccess;
}
}  // namespace

size_t backward_scratch_bytes(size_t B, size_t N, size_t d, size_t F, size_t H, size_t E)
{
    BwBufs tmp;
    return carve_bufs(tmp, nullptr, B, N, d, F, H, E, true);
}

void backward_exchange_region(size_t B, size_t N, size_t d, size_t F, size_t H, size_t E, size_t *offset, size_t *bytes)
{
    (void)B; (void)N; (void)H;
    *offset = 0;
    *bytes = E == 2 ? bwp_exchange_bytes((int)d, (int)F) : 0;
}

// rows of a [B][N][d] tensor in position-first order (row n B + b), bf16
__global__ __launch_bounds__(256) void bw_rows_pf_kernel(const bf16_t *__restrict__ in, bf16_t *__restrict__ out, int B, int N, int d)
{
    const size_t n_el = (size_t)B * N * d;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n_el; e += (size_t)gridDim.x * 256) {
        const size_t r = e / d, c = e % d;
        const size_t n = r / B, b = r % B;
        out[e] = in[(b * N + n) * d + c];
    }
}

template <typename T>
hipError_t backward_layer(const LayerDims &D, const Weights &W, const void *x_, const void *z_, const void *gy_, const void *gK_,
                          const void *gV_, float *dx, const BwGrads &G, void *ws, bool matrix_cores, hipStream_t st, BwpState *loop)
{
    const int B = D.B, N = D.N, d = D.d, F = D.F, H = D.H, M = B * N, BH = B * H, nf = D.norm_free;
    const T *x = (const T *)x_, *z = (const T *)z_, *gy = (const T *)gy_;
    const T *g_attn = (const T *)W.g_attn, *g_mlp = (const T *)W.g_mlp, *g_q = (const T *)W.g_q, *g_k = (const T *)W.g_k;
    const T *g_kv = W.g_kv ? (const T *)W.g_kv : g_attn;
    BwBufs Bf;
    carve_bufs(Bf, (char *)ws, B, N, d, F, H, sizeof(T), true);
    if (!g_attn || nf) Bf.nxg = Bf.unit_x;
    if (!g_kv || nf) Bf.nzg = Bf.unit_z;
    if (!g_mlp || nf) Bf.hg = Bf.unit_h;
    hipError_t e = raise_lds();
    if (e != hipSuccess) return e;
    const dim3 blk(256);
    auto grid1 = [](size_t n) { return dim3((unsigned)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096)); };
    const size_t dd = (size_t)d * d, dF = (size_t)d * F;
    // bf16 storage: the batched products on the matrix cores
    const bool mm = matrix_cores && sizeof(T) == 2 && F % 64 == 0;
    // C[M][Nn] = A_bf16 [M][K] (rows lda) times W_bf16 [Nn][K]^T (rows ldb), optionally sliced over the contraction
    auto mm_nt = [&](const bf16_t *A, size_t lda, const bf16_t *Wb, size_t ldb, float *C, size_t ldc, int Mo, int Nn, int K, float alpha,
                     bool accumulate, int slices) {
        const dim3 g((unsigned)((Mo + kGtRows - 1) / kGtRows), (unsigned)((Nn + kGtCols - 1) / kGtCols), (unsigned)slices);
        hipLaunchKernelGGL(bw_mm_kernel, g, blk, 0, st, A, lda, Wb, ldb, C, ldc, Bf.part, Mo, Nn, K / slices, alpha, accumulate ? 1 : 0);
        if (slices > 1)
            hipLaunchKernelGGL(bw_mm_reduce_kernel, grid1((size_t)Mo * Nn), blk, 0, st, Bf.part, slices, C, ldc, Mo, Nn, alpha,
                               accumulate ? 1 : 0);
    };
    // recompute product C[M][Nn] = Act [M][d] Wt^T with the activation as bf16 head + remainder (Wt: the caller's bf16 matrix)
    auto act_times_w = [&](const float *Act, const void *Wt, const float *Wf, float *C, size_t ldc, int Nn) {
        if (mm) {
            hipLaunchKernelGGL(bw_split_rows_kernel, grid1((size_t)M * d), blk, 0, st, Act, (size_t)d, Bf.op_hi, Bf.op_lo, (size_t)d, M, d);
            mm_nt(Bf.op_lo, d, (const bf16_t *)Wt, d, C, ldc, M, Nn, d, 1.f, false, 1);
            mm_nt(Bf.op_hi, d, (const bf16_t *)Wt, d, C, ldc, M, Nn, d, 1.f, true, 1);
        } else {
            gemm(st, Act, d, 1, Wf, d, 1, C, (long)ldc, M, Nn, d, 1.f, false);
        }
    };

    // ---- weights: fp32 copies for the products, transposed copies (storage type) for the loop's small-M products
    if (!mm) {
        hipLaunchKernelGGL(bw_to_f32_kernel<T>, grid1(dd), blk, 0, st, (const T *)W.Wq, Bf.Wqkv_f, dd);
        hipLaunchKernelGGL(bw_to_f32_kernel<T>, grid1(dd), blk, 0, st, (const T *)W.Wk, Bf.Wqkv_f + dd, dd);
        hipLaunchKernelGGL(bw_to_f32_kernel<T>, grid1(dd), blk, 0, st, (const T *)W.Wv, Bf.Wqkv_f + 2 * dd, dd);
        hipLaunchKernelGGL(bw_to_f32_kernel<T>, grid1(dd), blk, 0, st, (const T *)W.Wo, Bf.Wo_f, dd);
        hipLaunchKernelGGL(bw_to_f32_kernel<T>, grid1(dF), blk, 0, st, (const T *)W.W1, Bf.W1_f, dF);
        hipLaunchKernelGGL(bw_to_f32_kernel<T>, grid1(dF), blk, 0, st, (const T *)W.W2, Bf.W2_f, dF);
    }
    auto transpose = [&](const void *in, void *out, int rows, int cols, size_t ldo, int col0) {
        hipLaunchKernelGGL(bw_transpose_kernel<T>, dim3((unsigned)((cols + 31) / 32), (unsigned)((rows + 31) / 32)), blk, 0, st,
                           (const T *)in, (T *)out, rows, cols, ldo, col0);
    };
    transpose(W.Wk, Bf.WkvT, d, d, 2 * (size_t)d, 0);   // WkvT[c][r] = Wk[r][c], WkvT[c][d + r] = Wv[r][c]
    transpose(W.Wv, Bf.WkvT, d, d, 2 * (size_t)d, d);
    transpose(W.W2, Bf.W2T, d, F, (size_t)d, 0);         // W2 [d][F] -> [F][d]
    transpose(W.W1, Bf.W1T, F, d, (size_t)F, 0);         // W1 [F][d] -> [d][F]
    transpose(W.Wo, Bf.WoT, d, d, (size_t)d, 0);
    if (mm) {   // [Wq; Wk; Wv]^T as [d][3d]
        transpose(W.Wq, Bf.WqkvT_b, d, d, 3 * (size_t)d, 0);
        transpose(W.Wk, Bf.WqkvT_b, d, d, 3 * (size_t)d, d);
        transpose(W.Wv, Bf.WqkvT_b, d, d, 3 * (size_t)d, 2 * d);
    }

    // ---- (A) recompute
    hipLaunchKernelGGL(bw_rows_norm_kernel<T>, dim3(M), blk, 0, st, x, (const float *)nullptr, 0.f, g_attn, Bf.unit_x, Bf.nxg, Bf.rinv_x,
                       B, N, d, D.eps, nf);
    if (mm) {
        hipLaunchKernelGGL(bw_split_rows_kernel, grid1((size_t)M * d), blk, 0, st, Bf.nxg, (size_t)d, Bf.op_hi, Bf.op_lo, (size_t)d, M, d);
        const void *w3[3] = {W.Wq, W.Wk, W.Wv};
        for (int j = 0; j < 3; ++j) {
            mm_nt(Bf.op_lo, d, (const bf16_t *)w3[j], d, Bf.qkv + (size_t)j * d, 3 * (size_t)d, M, d, d, 1.f, false, 1);
            mm_nt(Bf.op_hi, d, (const bf16_t *)w3[j], d, Bf.qkv + (size_t)j * d, 3 * (size_t)d, M, d, d, 1.f, true, 1);
        }
    } else {
        gemm(st, Bf.nxg, d, 1, Bf.Wqkv_f, d, 1, Bf.qkv, 3 * d, M, 3 * d, d, 1.f, false);
    }
    hipLaunchKernelGGL(bw_head_norm_kernel<T>, dim3(M, H), dim3(64), 0, st, Bf.qkv, 3 * d, 0, g_q, Bf.Qn, Bf.rq, H, D.eps, nf);
    hipLaunchKernelGGL(bw_head_norm_kernel<T>, dim3(M, H), dim3(64), 0, st, Bf.qkv, 3 * d, d, g_k, Bf.Ktn, Bf.rkt, H, D.eps, nf);
    hipLaunchKernelGGL(bw_head_norm_kernel<T>, dim3(M, H), dim3(64), 0, st, Bf.qkv, 3 * d, 2 * d, (const T *)nullptr, Bf.Vt,
                       (float *)nullptr, H, D.eps, nf);
    hipLaunchKernelGGL(bw_rows_norm_kernel<T>, dim3(M), blk, 0, st, z, (const float *)nullptr, 0.f, g_kv, Bf.unit_z, Bf.nzg, Bf.rinv_z,
                       B, N, d, D.eps, nf);
    if (mm) {
        hipLaunchKernelGGL(bw_split_rows_kernel, grid1((size_t)M * d), blk, 0, st, Bf.nzg, (size_t)d, Bf.op_hi, Bf.op_lo, (size_t)d, M, d);
        const void *w2[2] = {W.Wk, W.Wv};
        for (int j = 0; j < 2; ++j) {
            mm_nt(Bf.op_lo, d, (const bf16_t *)w2[j], d, Bf.kv + (size_t)j * d, 2 * (size_t)d, M, d, d, 1.f, false, 1);
            mm_nt(Bf.op_hi, d, (const bf16_t *)w2[j], d, Bf.kv + (size_t)j * d, 2 * (size_t)d, M, d, d, 1.f, true, 1);
        }
    } else {
        gemm(st, Bf.nzg, d, 1, Bf.Wqkv_f + dd, d, 1, Bf.kv, 2 * d, M, 2 * d, d, 1.f, false);
    }
    hipLaunchKernelGGL(bw_head_norm_kernel<T>, dim3(M, H), dim3(64), 0, st, Bf.kv, 2 * d, 0, g_k, Bf.Kp, Bf.rk, H, D.eps, nf);
    hipLaunchKernelGGL(bw_head_norm_kernel<T>, dim3(M, H), dim3(64), 0, st, Bf.kv, 2 * d, d, (const T *)nullptr, Bf.Vp,
                       (float *)nullptr, H, D.eps, nf);
    const bool mfma_attn = mm && Bf.flash && getenv("RT_BWD_ALU_ATTENTION") == nullptr;
    if (mfma_attn && (e = bw_attn_mfma_init()) != hipSuccess) return e;
    // one block of Algorithm 1 backwards: keys [k0, k0 + P) <- queries [q0, q0 + nq)
    auto run_event = [&](int k0, int P, int q0, int nq) -> hipError_t {
        if (mfma_attn) return bw_event_mfma(D, Bf.Qn, Bf.Kp, Bf.Vp, Bf.dc, Bf.lse, Bf.Ds, Bf.dK, Bf.dV, k0, P, q0, nq, st);
        hipLaunchKernelGGL(bw_event_kernel, dim3((unsigned)((P + 63) / 64), BH), blk, kEventLds, st, Bf.Qn, Bf.Kp, Bf.Vp, Bf.dc, Bf.lse,
                           Bf.Ds, Bf.dK, Bf.dV, B, H, k0, P, q0, nq, D.scale, D.alibi);
        return hipSuccess;
    };
    if (mfma_attn) {
        e = flash_recompute_f32(D, Bf.Qn, Bf.Ktn, Bf.Vt, Bf.Kp, Bf.Vp, Bf.c, Bf.lse, Bf.flash, st);
        if (e != hipSuccess) return e;
    } else {
        hipLaunchKernelGGL(bw_attn_fwd_kernel, dim3(BH, N), dim3(64), 0, st, Bf.Qn, Bf.Ktn, Bf.Vt, Bf.Kp, Bf.Vp, Bf.c, Bf.lse, B, H, D.scale,
                           D.alibi);
    }
    act_times_w(Bf.c, W.Wo, Bf.Wo_f, Bf.a, (size_t)d, d);
    hipLaunchKernelGGL(bw_rows_norm_kernel<T>, dim3(M), blk, 0, st, x, Bf.a, D.alpha, g_mlp, Bf.unit_h, Bf.hg, Bf.rinv_h, B, N, d, D.eps,
                       nf);
    act_times_w(Bf.hg, W.W1, Bf.W1_f, Bf.gp, (size_t)F, F);
    hipLaunchKernelGGL(bw_gelu_kernel, grid1((size_t)M * F), blk, 0, st, Bf.gp, Bf.act, Bf.gp, (size_t)M * F);

    // ---- (B) the reverse loop
    hipLaunchKernelGGL(bw_init_pairs_kernel<T>, grid1((size_t)M * d), blk, 0, st, (const T *)gK_, (const T *)gV_, Bf.dK, Bf.dV,
                       (size_t)M * d);
    const bool single_launch = mm && loop != nullptr && Bf.exchange != nullptr && bwp_supported(*loop, D);
    if (single_launch) {
        // the halves of the loop's products that do not depend on the loop (see rt_backward_persistent.hip): with gy and
        // the normalised rows of z and h known for all positions, W2^T and Wo^T of them are batched products here
        const bf16_t *W2T = (const bf16_t *)Bf.W2T, *WoT = (const bf16_t *)Bf.WoT;
        hipLaunchKernelGGL(bw_rows_pf_kernel, grid1((size_t)M * d), blk, 0, st, (const bf16_t *)gy, Bf.gy_pf, B, N, d);
        mm_nt(Bf.gy_pf, d, W2T, d, Bf.A_gy, (size_t)F, M, F, d, 1.f, false, 1);
        mm_nt(Bf.gy_pf, d, WoT, d, Bf.C_gy, (size_t)d, M, d, d, 1.f, false, 1);
        hipLaunchKernelGGL(bw_split_rows_kernel, grid1((size_t)M * d), blk, 0, st, Bf.unit_z, (size_t)d, Bf.op_hi, Bf.op_lo, (size_t)d, M, d);
        mm_nt(Bf.op_lo, d, W2T, d, Bf.A_uz, (size_t)F, M, F, d, 1.f, false, 1);
        mm_nt(Bf.op_hi, d, W2T, d, Bf.A_uz, (size_t)F, M, F, d, 1.f, true, 1);
        mm_nt(Bf.op_lo, d, WoT, d, Bf.C_uz, (size_t)d, M, d, d, 1.f, false, 1);
        mm_nt(Bf.op_hi, d, WoT, d, Bf.C_uz, (size_t)d, M, d, d, 1.f, true, 1);
        hipLaunchKernelGGL(bw_split_rows_kernel, grid1((size_t)M * d), blk, 0, st, Bf.unit_h, (size_t)d, Bf.op_hi, Bf.op_lo, (size_t)d, M, d);
        mm_nt(Bf.op_lo, d, WoT, d, Bf.C_uh, (size_t)d, M, d, d, 1.f, false, 1);
        mm_nt(Bf.op_hi, d, WoT, d, Bf.C_uh, (size_t)d, M, d, d, 1.f, true, 1);
        BwpTensors Tn;
        Tn.WkvT = (const bf16_t *)Bf.WkvT; Tn.W2T = W2T; Tn.W1T = (const bf16_t *)Bf.W1T; Tn.WoT = WoT;
        Tn.g_kv = (const bf16_t *)g_kv; Tn.g_mlp = (const bf16_t *)g_mlp; Tn.g_k = (const bf16_t *)g_k;
        Tn.gy = (const bf16_t *)gy;
        Tn.unit_k = Bf.kv; Tn.rk = Bf.rk; Tn.unit_z = Bf.unit_z; Tn.rinv_z = Bf.rinv_z; Tn.unit_h = Bf.unit_h; Tn.rinv_h = Bf.rinv_h;
        Tn.gp = Bf.gp; Tn.A_gy = Bf.A_gy; Tn.A_uz = Bf.A_uz; Tn.C_gy = Bf.C_gy; Tn.C_uz = Bf.C_uz; Tn.C_uh = Bf.C_uh;
        Tn.Qn = Bf.Qn; Tn.Ktn = Bf.Ktn; Tn.Vt = Bf.Vt; Tn.Kp = Bf.Kp; Tn.Vp = Bf.Vp; Tn.c = Bf.c; Tn.lse = Bf.lse;
        Tn.dK = Bf.dK; Tn.dV = Bf.dV; Tn.dkraw = Bf.dkraw; Tn.d_rz = Bf.d_rz; Tn.Gz = Bf.Gz; Tn.dpre = Bf.dpre; Tn.t1 = Bf.t1;
        Tn.d_h = Bf.d_h; Tn.dc = Bf.dc; Tn.Ds = Bf.Ds; Tn.dq = Bf.dq; Tn.dkt = Bf.dkt; Tn.dvt = Bf.dvt;
        // one launch per block of kBwPmin positions, last block first; the block of Algorithm 1 that ends just before a
        // launch's first position takes that launch's (and the later ones') queries to the earlier keys
        for (int i_lo = ((N - 1) / kBwPmin) * kBwPmin; i_lo >= 0; i_lo -= kBwPmin) {
            const int i_hi = i_lo + kBwPmin - 1 < N - 1 ? i_lo + kBwPmin - 1 : N - 1;
            e = bwp_run_block(*loop, D, Tn, Bf.exchange, i_hi, i_lo, st);
            if (e != hipSuccess) return e;
            if (i_lo > 0) {
                const int P = i_lo & -i_lo, nq = P < N - i_lo ? P : N - i_lo;
                if ((e = run_event(i_lo - P, P, i_lo, nq)) != hipSuccess) return e;
            }
        }
    }
    if (!single_launch) {
    bool pair_done = false;   // [dkraw | dV] of position i was already prepared by the query after it
    for (int i = N - 1; i >= 0; --i) {
        const size_t ro = (size_t)i * B;
        if (!pair_done)
            hipLaunchKernelGGL(bw_pair_grad_kernel<T>, dim3(BH), dim3(64), 0, st, Bf.dK, Bf.dV, Bf.kv, Bf.rk, g_k, Bf.dkraw, Bf.in_kv, i, B,
                               H, nf);
        gemv<T, EPI_KV>(st, (const T *)Bf.WkvT, d, 2 * d, Bf.in_kv, 2 * (size_t)d, B, nullptr, Bf.d_rz + ro * d);
        hipLaunchKernelGGL((bw_norm_bw_row_kernel<T, T>), dim3(B), blk, 0, st, Bf.d_rz, Bf.unit_z, Bf.rinv_z, g_kv, gy + (size_t)i * d,
                           (size_t)N * d, Bf.Gz, Bf.dmo, D.alpha, i, B, d, nf);
        gemv<T, EPI_MUL>(st, (const T *)Bf.W2T, F, d, Bf.dmo, (size_t)d, B, Bf.gp + ro * F, Bf.dpre + ro * F);
        gemv<T, EPI_KV>(st, (const T *)Bf.W1T, d, F, Bf.dpre + ro * F, (size_t)F, B, nullptr, Bf.t1 + ro * d);
        hipLaunchKernelGGL((bw_norm_bw_row_kernel<T, float>), dim3(B), blk, 0, st, Bf.t1, Bf.unit_h, Bf.rinv_h, g_mlp, Bf.Gz + ro * d,
                           (size_t)d, Bf.d_h, Bf.da, D.alpha, i, B, d, nf);
        gemv<T, EPI_KV>(st, (const T *)Bf.WoT, d, d, Bf.da, (size_t)d, B, nullptr, Bf.dc + ro * d);
        // position i - 1 lies in this query's window unless i opens a block of kBwPmin positions (then a tile follows below,
        // or i = 0): its pair gradient is complete after this query's update and is finished by the same wavefront
        const int fuse = (i & (kBwPmin - 1)) != 0 ? 1 : 0;
        hipLaunchKernelGGL(bw_attn_row_kernel<T>, dim3(BH), dim3(64), 0, st, Bf.Qn, Bf.Ktn, Bf.Vt, Bf.Kp, Bf.Vp, Bf.c, Bf.dc, Bf.lse, Bf.Ds,
                           Bf.dK, Bf.dV, Bf.dq, Bf.dkt, Bf.dvt, i, B, H, D.scale, D.alibi, fuse, Bf.kv, Bf.rk, g_k, Bf.dkraw, Bf.in_kv, nf);
        pair_done = fuse != 0;
        const int P = i & -i;   // Algorithm 1's block that ends with key i - 1 (0-based): keys [i - P, i), queries [i, i + P)
        if (i > 0 && P >= kBwPmin) {
            const int nq = P < N - i ? P : N - i;
            if ((e = run_event(i - P, P, i, nq)) != hipSuccess) return e;
        }
    }
    }

    // ---- (C) batched remainder
    if (mfma_attn) {
        if ((e = bw_dq_mfma(D, Bf.Qn, Bf.Kp, Bf.Vp, Bf.dc, Bf.lse, Bf.Ds, Bf.dq, st)) != hipSuccess) return e;
    } else {
        hipLaunchKernelGGL(bw_dq_kernel, dim3((unsigned)((N + 63) / 64), BH), blk, kDqLds, st, Bf.Qn, Bf.Kp, Bf.Vp, Bf.dc, Bf.lse, Bf.Ds,
                           Bf.dq, B, H, N, D.scale, D.alibi);
    }
    // gain gradients that need the normalised values (before anything is overwritten)
    auto colsum = [&](const float *A, size_t lda, const float *Bm, size_t ldb, float *out, bool acc) {
        hipLaunchKernelGGL(bw_colsum_kernel, dim3((unsigned)((d + 63) / 64)), blk, 0, st, A, lda, Bm, ldb, M, d, out, acc ? 1 : 0);
    };
    const size_t ld3 = 3 * (size_t)d;
    hipLaunchKernelGGL(bw_head_norm_bw_kernel<T>, dim3(M, H), dim3(64), 0, st, Bf.dq, Bf.qkv, 3 * d, 0, Bf.rq, g_q, Bf.G3, 3 * d, 0, H, nf);
    hipLaunchKernelGGL(bw_head_norm_bw_kernel<T>, dim3(M, H), dim3(64), 0, st, Bf.dkt, Bf.qkv, 3 * d, d, Bf.rkt, g_k, Bf.G3, 3 * d, d, H,
                       nf);
    hipLaunchKernelGGL(bw_head_norm_bw_kernel<T>, dim3(M, H), dim3(64), 0, st, Bf.dvt, Bf.qkv, 3 * d, 0, (const float *)nullptr,
                       (const T *)nullptr, Bf.G3, 3 * d, 2 * d, H, nf);
    // dn = [dq_raw | dkt_raw | dvt] [Wq; Wk; Wv]
    if (mm) {
        hipLaunchKernelGGL(bw_split_rows_kernel, grid1((size_t)M * 3 * d), blk, 0, st, Bf.G3, 3 * (size_t)d, Bf.G3_b, (bf16_t *)nullptr,
                           3 * (size_t)d, M, 3 * d);
        mm_nt(Bf.G3_b, 3 * (size_t)d, Bf.WqkvT_b, 3 * (size_t)d, Bf.dn, (size_t)d, M, d, 3 * d, 1.f, false, 1);
    } else {
        gemm(st, Bf.G3, 3 * d, 1, Bf.Wqkv_f, 1, d, Bf.dn, d, M, d, 3 * d, 1.f, false);
    }
    hipLaunchKernelGGL(bw_dx_kernel<T>, dim3(M), blk, 0, st, Bf.dn, Bf.unit_x, Bf.rinv_x, g_attn, Bf.d_h, dx, B, N, d, nf);
    // parameter sums over all rows:  dW[n][k] = sum_r G[r][n] In[r][k]
    if (mm) {
        const int S = bw_slices((size_t)M), SF = S >= 4 ? S / 4 : 1;
        const int Ks = (int)((((size_t)M + S - 1) / S + 63) / 64 * 64), Mp = S * Ks;
        // transposed bf16 copy [Cn][Mp] of columns c0.. of a [M][ld] tensor (the tail M..Mp is zero)
        auto tr = [&](const float *in, size_t ld, int c0, int Cn, bf16_t *out) {
            hipLaunchKernelGGL(bw_transpose_bf16_kernel, dim3((unsigned)((Mp + 63) / 64), (unsigned)((Cn + 63) / 64)), blk, 0, st, in, ld, c0,
                               out, (size_t)Mp, M, Mp, Cn);
        };
        auto wsum = [&](int rowsA, int rowA0, int rowsB, float *C, float alpha, bool acc, int slices) {
            mm_nt(Bf.tA + (size_t)rowA0 * Mp, (size_t)Mp, Bf.tB, (size_t)Mp, C, (size_t)rowsB, rowsA, rowsB, Mp, alpha, acc, slices);
        };
        if (G.Wq || G.Wk || G.Wv) {
            tr(Bf.G3, 3 * (size_t)d, 0, 3 * d, Bf.tA);
            tr(Bf.nxg, (size_t)d, 0, d, Bf.tB);
            if (G.Wq) wsum(d, 0, d, G.Wq, 1.f, false, S);
            if (G.Wk) wsum(d, d, d, G.Wk, 1.f, false, S);
            if (G.Wv) wsum(d, 2 * d, d, G.Wv, 1.f, false, S);
        }
        if (G.Wk || G.Wv) {
            tr(Bf.nzg, (size_t)d, 0, d, Bf.tB);
            if (G.Wk) { tr(Bf.dkraw, (size_t)d, 0, d, Bf.tA); wsum(d, 0, d, G.Wk, 1.f, true, S); }
            if (G.Wv) { tr(Bf.dV, (size_t)d, 0, d, Bf.tA); wsum(d, 0, d, G.Wv, 1.f, true, S); }
        }
        if (G.Wo) { tr(Bf.d_h, (size_t)d, 0, d, Bf.tA); tr(Bf.c, (size_t)d, 0, d, Bf.tB); wsum(d, 0, d, G.Wo, D.alpha, false, S); }
        if (G.W1) { tr(Bf.dpre, (size_t)F, 0, F, Bf.tA); tr(Bf.hg, (size_t)d, 0, d, Bf.tB); wsum(F, 0, d, G.W1, 1.f, false, SF); }
        if (G.W2) { tr(Bf.Gz, (size_t)d, 0, d, Bf.tA); tr(Bf.act, (size_t)F, 0, F, Bf.tB); wsum(d, 0, F, G.W2, D.alpha, false, SF); }
    } else {
    if (G.Wq) gemm(st, Bf.G3, 1, 3 * d, Bf.nxg, 1, d, G.Wq, d, d, d, M, 1.f, false);
    if (G.Wk) {
        gemm(st, Bf.G3 + d, 1, 3 * d, Bf.nxg, 1, d, G.Wk, d, d, d, M, 1.f, false);
        gemm(st, Bf.dkraw, 1, d, Bf.nzg, 1, d, G.Wk, d, d, d, M, 1.f, true);
    }
    if (G.Wv) {
        gemm(st, Bf.G3 + 2 * d, 1, 3 * d, Bf.nxg, 1, d, G.Wv, d, d, d, M, 1.f, false);
        gemm(st, Bf.dV, 1, d, Bf.nzg, 1, d, G.Wv, d, d, d, M, 1.f, true);
    }
    if (G.Wo) gemm(st, Bf.d_h, 1, d, Bf.c, 1, d, G.Wo, d, d, d, M, D.alpha, false);
    if (G.W1) gemm(st, Bf.dpre, 1, F, Bf.hg, 1, d, G.W1, d, F, d, M, 1.f, false);
    if (G.W2) gemm(st, Bf.Gz, 1, d, Bf.act, 1, F, G.W2, F, d, F, M, D.alpha, false);
    }
    // gains
    if (nf) {
        float *gs[5] = {G.g_attn, G.g_mlp, G.g_kv, G.g_q, G.g_k};
        for (float *p : gs)
            if (p) hipLaunchKernelGGL(bw_fill_kernel, grid1((size_t)d), blk, 0, st, p, (size_t)d, 0.f);
    } else {
        if (G.g_q) colsum(Bf.dq, d, Bf.qkv, ld3, G.g_q, false);
        if (G.g_k) {
            colsum(Bf.dkt, d, Bf.qkv + d, ld3, G.g_k, false);
            colsum(Bf.dK, d, Bf.kv, 2 * (size_t)d, G.g_k, true);
        }
        if (G.g_mlp) colsum(Bf.t1, d, Bf.unit_h, d, G.g_mlp, false);
        if (G.g_attn) colsum(Bf.dn, d, Bf.unit_x, d, G.g_attn, false);
        if (W.g_kv == nullptr) {   // RMS(z) shares the gain of RMS(x)
            if (G.g_attn) colsum(Bf.d_rz, d, Bf.unit_z, d, G.g_attn, true);
            if (G.g_kv) hipLaunchKernelGGL(bw_fill_kernel, grid1((size_t)d), blk, 0, st, G.g_kv, (size_t)d, 0.f);
        } else if (G.g_kv) {
            colsum(Bf.d_rz, d, Bf.unit_z, d, G.g_kv, false);
        }
    }
    return hipGetLastError();
}

template hipError_t backward_layer<float>(const LayerDims &, const Weights &, const void *, const void *, const void *, const void *,
                                          const void *, float *, const BwGrads &, void *, bool, hipStream_t, BwpState *);
template hipError_t backward_layer<bf16_t>(const LayerDims &, const Weights &, const void *, const void *, const void *, const void *,
                                           const void *, float *, const BwGrads &, void *, bool, hipStream_t, BwpState *);

}  // namespace rt
