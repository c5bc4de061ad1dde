// Whole-sequence evaluation without the sequential loop, for the two cases in which every key-value pair is
// known in advance:
//   * Sec. 6.1 ("activation checkpointing"): given a layer's input x AND its output z, the persistent pairs are
//     k_i, v_i = proj(RMS(z_i)) for all i at once, and every intermediate (and z itself) follows from batched
//     matrix products and one causal attention with the temporary pair on the diagonal;
//   * Sec. 2.1: the standard Transformer layer, whose keys and values come from the layer input - the same
//     computation with the persistent pair of a position equal to its temporary pair.
// Steps, all on one stream, bf16 storage with matrix-core kernels throughout:
//   pre-pass GEMM over the source of the pairs -> export K, V (+ key remainder and V^T for the tiles)
//   pre-pass GEMM over x -> q, temporary pairs (recompute only; for the Transformer layer they are the same rows)
//   one masked flash-style launch for the attention of all positions (cache rows j < i plus the temporary pair)
//   h = x + alpha Wo a;  u = gelu(W1 RMS(h));  y = h + alpha W2 u   as three GEMMs with fused epilogues.
#include "rt_base_case.h"
#include "rt_mfma_device.h"
#include "rt_gemm_tiled.h"

namespace rt {

// ---------------------------------------------------------------------------------------------
// C[m][n] = sum_k A[m][k] W[n][k], A [M][K] and W [Nn][K] bf16 row-major, fp32 accumulation.
// Block tile 128 x 128, 4 wavefronts as 2 x 2 of 64 x 64, fragments straight from global memory
// (v_mfma_f32_16x16x32_bf16: both operands want the contraction index contiguous per lane).
//   PG_WO: out_f = out_b = res_b + alpha C                       (h = x + alpha Wo a)
//   PG_W1: out_b = gelu(rinv_m * C), A rows multiplied by `gain` on the way, rinv_m = 1/rms of the raw A row,
//          formed from the fragments (u = gelu(W1 RMS(h; g_mlp)))
//   PG_W2: out_b = res_f + alpha C                               (y = h + alpha W2 u)
// Rows: the M rows are positions n0 .. n0 + Nc - 1 of every batch row of [B][N][*] tensors (A, res, out alike):
// row m lives at tensor row (m / Nc) * N + n0 + m % Nc  (Nc = N, n0 = 0: the whole tensor).
// grid (ceil(M / 128), Nn / 128 rounded up), Nn a multiple of 64.
// ---------------------------------------------------------------------------------------------
enum { PG_WO = 0, PG_W1 = 1, PG_W2 = 2 };

template <int EPI>
__global__ __launch_bounds__(256) void par_gemm_kernel(const bf16_t *__restrict__ A, const bf16_t *__restrict__ W, int M, int Nn,
                                                       int K, int Nc, int N, int n0, const bf16_t *__restrict__ gain, float eps,
                                                       int norm_free,
                                                       float alpha, const bf16_t *__restrict__ res_b,
                                                       const float *__restrict__ res_f, float *__restrict__ out_f,
                                                       bf16_t *__restrict__ out_b)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l16 = lane & 15, g = lane >> 4;
    const int m0 = blockIdx.x * 128 + wm * 64, nb0 = blockIdx.y * 128 + wn * 64;
    if (m0 >= M || nb0 >= Nn) return;   // no barriers in this kernel

    f32x4_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const bf16_t *arow[4], *brow[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int mr = min(m0 + i * 16 + l16, M - 1);
        arow[i] = A + ((size_t)(mr / Nc) * N + n0 + mr % Nc) * K + 8 * g;
        brow[i] = W + (size_t)(nb0 + i * 16 + l16) * K + 8 * g;
    }
    const bool normed = EPI == PG_W1 && !norm_free;
    const bool use_gain = normed && gain != nullptr;
    float ssq[4] = {0.f, 0.f, 0.f, 0.f};   // PG_W1: sum of squares of A row l16 + 16 i over this lane's k slices

    for (int k0 = 0; k0 < K; k0 += 32) {
        Frag a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a[i].u = *reinterpret_cast<const uint4 *>(arow[i] + k0);
            b[i].u = *reinterpret_cast<const uint4 *>(brow[i] + k0);
        }
        if (normed) {
            float gg[8] = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f};
            if (use_gain) load8(gain + k0 + 8 * g, gg);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t w4[4] = {a[i].u.x, a[i].u.y, a[i].u.z, a[i].u.w};
                uint32_t o4[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float lo = __uint_as_float(w4[e] << 16), hi = __uint_as_float(w4[e] & 0xFFFF0000u);
                    ssq[i] = fmaf(lo, lo, fmaf(hi, hi, ssq[i]));
                    o4[e] = pack_bf16(lo * gg[2 * e], hi * gg[2 * e + 1]);
                }
                if (use_gain) a[i].u = make_uint4(o4[0], o4[1], o4[2], o4[3]);
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] = mfma16(a[i], b[j], acc[i][j]);
    }
    if (normed) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {   // join the four k slices of a row: every lane with this l16 then holds the row's scale
            ssq[i] += __shfl_xor(ssq[i], 16, 64);
            ssq[i] += __shfl_xor(ssq[i], 32, 64);
            ssq[i] = rsqrtf(ssq[i] / (float)K + eps);
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int m = m0 + i * 16 + 4 * g + r;
            // this lane's output rows are 16 i + 4 g + r; their scale sits in the lanes whose l16 is 4 g + r
            const float rs = normed ? __shfl(ssq[i], 4 * g + r, 64) : 1.f;
            if (m < M) {
                const size_t row = (size_t)(m / Nc) * N + n0 + m % Nc;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const size_t o = row * Nn + nb0 + j * 16 + l16;
                    const float c = acc[i][j][r];
                    if (EPI == PG_WO) {
                        const float h = bf16_to_f32(res_b[o]) + alpha * c;
                        out_f[o] = h;
                        out_b[o] = f32_to_bf16(h);
                    } else if (EPI == PG_W1) {
                        out_b[o] = f32_to_bf16(gelu_erf(c * rs));
                    } else {
                        out_b[o] = f32_to_bf16(res_f[o] + alpha * c);
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// The same products with both operands staged in LDS (tiled_mainloop), for many rows and Nn a multiple of 128, K of 64.
//   PG_WO: h = res_b + alpha C -> out_f (fp32) and out_b = bf16(h * gain): the A operand of the next product with its
//          RMS gain already applied (gain may be null)
//   PG_W1: out_b = gelu(rinv_m C); rinv_m = 1/rms of row m of h (par_rinv_kernel on the fp32 copy)
//   PG_W2: out_b = res_f + alpha C
// grid (ceil(M / 256), Nn / 128), block 256.
// ---------------------------------------------------------------------------------------------
template <int EPI>
__global__ __launch_bounds__(256) void tiled_gemm_kernel(const bf16_t *__restrict__ A, const bf16_t *__restrict__ W, int M, int Nn,
                                                         int K, int Nc, int N, int n0, const bf16_t *__restrict__ gain,
                                                         const float *__restrict__ rinv, int norm_free, float alpha,
                                                         const bf16_t *__restrict__ res_b, const float *__restrict__ res_f,
                                                         float *__restrict__ out_f, bf16_t *__restrict__ out_b)
{
    __shared__ __align__(16) bf16_t As[kGtRows * kGtLd];
    __shared__ __align__(16) bf16_t Bs[kGtCols * kGtLd];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, hi = lane >> 5;
    const int m0 = blockIdx.x * kGtRows, nb0 = blockIdx.y * kGtCols;
    const int prow = tid >> 3, pc = tid & 7;
    const bf16_t *ga[8], *gb[4];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int mr = min(m0 + prow + 32 * i, M - 1);
        ga[i] = A + ((size_t)(mr / Nc) * N + n0 + mr % Nc) * K + pc * 8;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) gb[i] = W + (size_t)(nb0 + prow + 32 * i) * K + pc * 8;

    f32x16_t acc[4][2];
    tiled_mainloop(ga, gb, nullptr, K, As, Bs, acc);

    float gcol[2] = {1.f, 1.f};
    if (EPI == PG_WO && gain != nullptr && !norm_free) {
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) gcol[nt] = bf16_to_f32(gain[nb0 + wn * 64 + nt * 32 + l32]);
    }
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int m = m0 + wm * 128 + mt * 32 + 8 * (i / 4) + 4 * hi + (i % 4);
            if (m < M) {
                const size_t row = (size_t)(m / Nc) * N + n0 + m % Nc;
                const float rs = (EPI == PG_W1 && !norm_free) ? rinv[m] : 1.f;
#pragma unroll
                for (int nt = 0; nt < 2; ++nt) {
                    const size_t o = row * Nn + nb0 + wn * 64 + nt * 32 + l32;
                    const float c = acc[mt][nt][i];
                    if (EPI == PG_WO) {
                        const float h = bf16_to_f32(res_b[o]) + alpha * c;
                        out_f[o] = h;
                        out_b[o] = f32_to_bf16(h * gcol[nt]);
                    } else if (EPI == PG_W1) {
                        out_b[o] = f32_to_bf16(gelu_bf16_out(c * rs));
                    } else {
                        out_b[o] = f32_to_bf16(res_f[o] + alpha * c);
                    }
                }
            }
        }
    }
}

// 1 / rms of rows n0 .. n0 + Nc - 1 of every batch row of a [B][N][d] fp32 tensor, rinv[m] for m = b Nc + n.
// grid ceil(M / 4), block 256: one wavefront per row.  d is a multiple of 4.
__global__ __launch_bounds__(256) void par_rinv_kernel(const float *__restrict__ x, float *__restrict__ rinv, int M, int Nc, int N,
                                                       int n0, int d, float eps)
{
    const int lane = threadIdx.x & 63, m = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (m >= M) return;
    const float *xr = x + ((size_t)(m / Nc) * N + n0 + m % Nc) * d;
    float ss = 0.f;
    for (int k = lane * 4; k < d; k += 256) {
        const float4 v = *reinterpret_cast<const float4 *>(xr + k);
        ss = fmaf(v.x, v.x, fmaf(v.y, v.y, fmaf(v.z, v.z, fmaf(v.w, v.w, ss))));
    }
    ss = wave_sum(ss);
    if (lane == 0) rinv[m] = rsqrtf(ss / (float)d + eps);
}

// ---------------------------------------------------------------------------------------------
// The same products for FEW rows (a block of the blocked recurrence: M = block x B, tens to a few hundred rows),
// where the kernel above is latency-bound: few workgroups, and every wavefront walks the whole contraction in
// dependent steps.  Here a workgroup owns a 64 x 64 output tile and its NWV = 4 or 8 wavefronts split the contraction
// (each the full tile over K / NWV); a wavefront issues the loads of four steps (128 indices: 32 fragments) before
// their 64 matrix instructions; the partial tiles and the partial row statistics meet in LDS (four tile slots:
// wavefronts 4..7 add theirs onto the slots of wavefronts 0..3), then thread (row, quarter) of the first 256
// finishes 16 consecutive outputs of one row.  CT = 32 / 16: tiles of 64 x 32 / 64 x 16 outputs (8 / 4 per thread) - two /
// four times the workgroups, for products of so few rows that 64-column tiles do not keep the memory system busy.
//   PG_PRE: the pre-pass projection: W = [Wq; Wk; Wv] by column block (one head each), A rows RMS-normalised with
//           `gain`, then qkRMS per head for q and k_tmp; rows go to Q / Kt / Vt (and fp32 Qf / Ktf) position-first.
// grid (ceil(M / 64), Nn / 64), block 64 NWV, 70 KB of LDS.
// ---------------------------------------------------------------------------------------------
constexpr int PG_PRE = 3;
constexpr int kSkLd = 68;   // row stride of a partial tile in floats

struct PreOut {   // PG_PRE only
    const bf16_t *Wq, *Wk, *Wv, *g_q, *g_k;
    bf16_t *Q, *Kt, *Vt;
    float *Qf, *Ktf;
    int H, Bc;
    // y0: first column block ([q heads | k heads | v heads]): H skips the queries.  With K set the pairs go straight into the
    // cache rows (K, its bf16 remainder Klo, V and the transposed copy VT) instead of the pre-pass buffers.
    int y0;
    bf16_t *K, *Klo, *V, *VT;
    uint16_t *Kh;
    int vt_stride;
};

template <int EPI, int NWV, int CT = 64>
__global__ __launch_bounds__(64 * NWV) void blk_gemm_kernel(const bf16_t *__restrict__ A, const bf16_t *__restrict__ W, int M, int Nn,
                                                       int K, int Nc, int N, int n0, const bf16_t *__restrict__ gain, float eps,
                                                       int norm_free, float alpha, const bf16_t *__restrict__ res_b,
                                                       const float *__restrict__ res_f, float *__restrict__ out_f,
                                                       bf16_t *__restrict__ out_b, PreOut po)
{
    extern __shared__ __align__(16) unsigned char blk_smem[];
    float *part = reinterpret_cast<float *>(blk_smem);               // [4][64][kSkLd]
    float *ssq_s = part + 4 * 64 * kSkLd;                             // [8][64]
    const int tid = threadIdx.x, lane = tid & 63, kw = tid >> 6;
    const int l16 = lane & 15, g = lane >> 4;
    static_assert(CT == 64 || ((CT == 32 || CT == 16) && EPI != PG_PRE), "the pre-pass form owns whole heads");
    constexpr int NJ = CT / 16, PER = CT / 4;   // column fragments per wavefront; outputs per epilogue thread
    const int m0 = blockIdx.x * 64, nb0 = blockIdx.y * CT;
    const bf16_t *Wt = W;
    if (EPI == PG_PRE) {
        const int by = (int)blockIdx.y + po.y0;
        const int which = by / po.H, h = by % po.H;
        Wt = (which == 0 ? po.Wq : (which == 1 ? po.Wk : po.Wv)) + (size_t)h * kHeadDim * K - (size_t)nb0 * K;
    }
    const int klen = K / NWV, kbeg = kw * klen;
    f32x4_t acc[4][NJ];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const bf16_t *arow[4], *brow[NJ];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int mr = min(m0 + i * 16 + l16, M - 1);
        arow[i] = A + ((size_t)(mr / Nc) * N + n0 + mr % Nc) * K + kbeg + 8 * g;
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) brow[j] = Wt + (size_t)(nb0 + j * 16 + l16) * K + kbeg + 8 * g;
    const bool normed = (EPI == PG_W1 || EPI == PG_PRE) && !norm_free;
    const bool use_gain = normed && gain != nullptr;
    float ssq[4] = {0.f, 0.f, 0.f, 0.f};

#define RT_SK_STEP(av, bv, kk)                                                                                  \
    {                                                                                                           \
        if (normed) {                                                                                           \
            float gg[8] = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f};                                             \
            if (use_gain) load8(gain + kbeg + (kk) + 8 * g, gg);                                                \
            _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                       \
            {                                                                                                   \
                const uint32_t w4[4] = {av[i].u.x, av[i].u.y, av[i].u.z, av[i].u.w};                            \
                uint32_t o4[4];                                                                                 \
                _Pragma("unroll") for (int e = 0; e < 4; ++e)                                                   \
                {                                                                                               \
                    const float lo = __uint_as_float(w4[e] << 16), hi = __uint_as_float(w4[e] & 0xFFFF0000u);   \
                    ssq[i] = fmaf(lo, lo, fmaf(hi, hi, ssq[i]));                                                \
                    o4[e] = pack_bf16(lo * gg[2 * e], hi * gg[2 * e + 1]);                                      \
                }                                                                                               \
                if (use_gain) av[i].u = make_uint4(o4[0], o4[1], o4[2], o4[3]);                                 \
            }                                                                                                   \
        }                                                                                                       \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                           \
            _Pragma("unroll") for (int j = 0; j < NJ; ++j) acc[i][j] = mfma16(av[i], bv[j], acc[i][j]);         \
    }
    int k = 0;
    for (; k + 128 <= klen; k += 128) {   // four steps: 32 fragment loads in flight, then their 64 matrix instructions
        Frag a[4][4], b[4][NJ];
#pragma unroll
        for (int st = 0; st < 4; ++st) {
#pragma unroll
            for (int i = 0; i < 4; ++i) a[st][i].u = *reinterpret_cast<const uint4 *>(arow[i] + k + 32 * st);
#pragma unroll
            for (int j = 0; j < NJ; ++j) b[st][j].u = *reinterpret_cast<const uint4 *>(brow[j] + k + 32 * st);
        }
#pragma unroll
        for (int st = 0; st < 4; ++st) RT_SK_STEP(a[st], b[st], k + 32 * st)
    }
    for (; k < klen; k += 32) {
        Frag a[4], b[NJ];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i].u = *reinterpret_cast<const uint4 *>(arow[i] + k);
#pragma unroll
        for (int j = 0; j < NJ; ++j) b[j].u = *reinterpret_cast<const uint4 *>(brow[j] + k);
        RT_SK_STEP(a, b, k)
    }
#undef RT_SK_STEP
    // partial tile and partial row statistics of this wavefront
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (normed) {
            ssq[i] += __shfl_xor(ssq[i], 16, 64);
            ssq[i] += __shfl_xor(ssq[i], 32, 64);
            if (g == 0) ssq_s[kw * 64 + i * 16 + l16] = ssq[i];
        }
        if (kw < 4) {
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) part[(kw * 64 + i * 16 + 4 * g + r) * kSkLd + j * 16 + l16] = acc[i][j][r];
        }
    }
    __syncthreads();
    if (NWV == 8) {
        if (kw >= 4) {   // onto the slot of wavefront kw - 4: every element has one writer
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r) part[((kw - 4) * 64 + i * 16 + 4 * g + r) * kSkLd + j * 16 + l16] += acc[i][j][r];
        }
        __syncthreads();
        if (kw >= 4) return;   // no barrier below
    }
    // thread (row, quarter): PER consecutive outputs of one row
    const int row = tid >> 2, qc = (tid & 3) * PER;
    const int m = m0 + row;
    float v[16];
#pragma unroll
    for (int c4 = 0; c4 < PER / 4; ++c4) {
        float4 s4 = *reinterpret_cast<const float4 *>(part + (size_t)row * kSkLd + qc + 4 * c4);
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const float4 t4 = *reinterpret_cast<const float4 *>(part + (size_t)(w * 64 + row) * kSkLd + qc + 4 * c4);
            s4.x += t4.x; s4.y += t4.y; s4.z += t4.z; s4.w += t4.w;
        }
        v[4 * c4] = s4.x; v[4 * c4 + 1] = s4.y; v[4 * c4 + 2] = s4.z; v[4 * c4 + 3] = s4.w;
    }
    float rs = 1.f;
    if (normed) {
        float tot = (ssq_s[row] + ssq_s[64 + row]) + (ssq_s[128 + row] + ssq_s[192 + row]);
        if (NWV == 8) tot += (ssq_s[256 + row] + ssq_s[320 + row]) + (ssq_s[384 + row] + ssq_s[448 + row]);
        rs = rsqrtf(tot / (float)K + eps);
    }
    if (EPI == PG_PRE) {
        const int by = (int)blockIdx.y + po.y0;
        const int which = by / po.H, h = by % po.H;
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) { v[e] *= rs; ss = fmaf(v[e], v[e], ss); }
        ss += __shfl_xor(ss, 1, 64);   // the four threads of a row are adjacent lanes
        ss += __shfl_xor(ss, 2, 64);
        const bool qk = which < 2 && !norm_free;
        const float sc = qk ? rsqrtf(ss / (float)kHeadDim + eps) : 1.f;
        const bf16_t *gn = which == 0 ? po.g_q : po.g_k;
        if (m < M) {
            const int bb = m / Nc, n = n0 + m % Nc;
            const size_t oo = ((size_t)n * po.Bc + bb) * K + h * kHeadDim + qc;   // the projection is square: row length = K = d
            if (po.K != nullptr && which > 0) {   // straight into the cache: the rows of the pre-pass buffers are laid out like it
                bf16_t *vt = po.VT ? po.VT + ((size_t)(bb * po.H + h) * kHeadDim + qc) * po.vt_stride + n : nullptr;
                uint32_t hb[8], lb[8], fb[8];   // the 16 outputs as bf16 head, bf16 remainder and fp16 pairs: 32-byte runs per array
#pragma unroll
                for (int e2 = 0; e2 < 8; ++e2) {
                    float v0 = v[2 * e2] * sc, v1 = v[2 * e2 + 1] * sc;
                    if (qk && gn) {
                        v0 *= bf16_to_f32(gn[h * kHeadDim + qc + 2 * e2]);
                        v1 *= bf16_to_f32(gn[h * kHeadDim + qc + 2 * e2 + 1]);
                    }
                    hb[e2] = pack_bf16(v0, v1);
                    lb[e2] = pack_bf16(v0 - __uint_as_float(hb[e2] << 16), v1 - __uint_as_float(hb[e2] & 0xFFFF0000u));
                    fb[e2] = pack_f16(v0, v1);
                    if (which == 2 && vt) {   // else the caller transposes whole runs of positions later
                        vt[(size_t)(2 * e2) * po.vt_stride] = (bf16_t)(hb[e2] & 0xFFFFu);
                        vt[(size_t)(2 * e2 + 1) * po.vt_stride] = (bf16_t)(hb[e2] >> 16);
                    }
                }
                bf16_t *row = (which == 1 ? po.K : po.V) + oo;
                *reinterpret_cast<uint4 *>(row) = make_uint4(hb[0], hb[1], hb[2], hb[3]);
                *reinterpret_cast<uint4 *>(row + 8) = make_uint4(hb[4], hb[5], hb[6], hb[7]);
                if (which == 1) {
                    *reinterpret_cast<uint4 *>(po.Klo + oo) = make_uint4(lb[0], lb[1], lb[2], lb[3]);
                    *reinterpret_cast<uint4 *>(po.Klo + oo + 8) = make_uint4(lb[4], lb[5], lb[6], lb[7]);
                    *reinterpret_cast<uint4 *>(po.Kh + oo) = make_uint4(fb[0], fb[1], fb[2], fb[3]);
                    *reinterpret_cast<uint4 *>(po.Kh + oo + 8) = make_uint4(fb[4], fb[5], fb[6], fb[7]);
                }
                return;
            }
            bf16_t *dst = which == 0 ? po.Q : (which == 1 ? po.Kt : po.Vt);
            float *dstf = which == 0 ? po.Qf : (which == 1 ? po.Ktf : nullptr);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float val = v[e] * sc;
                if (qk && gn) val *= bf16_to_f32(gn[h * kHeadDim + qc + e]);
                dst[oo + e] = f32_to_bf16(val);
                if (dstf) dstf[oo + e] = val;
            }
        }
        return;
    }
    if (m >= M) return;
    const size_t o = ((size_t)(m / Nc) * N + n0 + m % Nc) * Nn + nb0 + qc;
    // PER consecutive outputs: loads and stores in pieces of four elements (8 bytes of bf16, 16 bytes of fp32)
#pragma unroll
    for (int e4 = 0; e4 < PER / 4; ++e4) {
        float r[4];
        if (EPI == PG_WO) {
            const uint2 xr = *reinterpret_cast<const uint2 *>(res_b + o + 4 * e4);
            const float x4[4] = {__uint_as_float(xr.x << 16), __uint_as_float(xr.x & 0xFFFF0000u), __uint_as_float(xr.y << 16),
                                 __uint_as_float(xr.y & 0xFFFF0000u)};
#pragma unroll
            for (int e = 0; e < 4; ++e) r[e] = x4[e] + alpha * v[4 * e4 + e];
            *reinterpret_cast<float4 *>(out_f + o + 4 * e4) = make_float4(r[0], r[1], r[2], r[3]);
        } else if (EPI == PG_W1) {
#pragma unroll
            for (int e = 0; e < 4; ++e) r[e] = gelu_erf(v[4 * e4 + e] * rs);
        } else {
            const float4 h4 = *reinterpret_cast<const float4 *>(res_f + o + 4 * e4);
            r[0] = h4.x + alpha * v[4 * e4]; r[1] = h4.y + alpha * v[4 * e4 + 1];
            r[2] = h4.z + alpha * v[4 * e4 + 2]; r[3] = h4.w + alpha * v[4 * e4 + 3];
        }
        *reinterpret_cast<uint2 *>(out_b + o + 4 * e4) = make_uint2(pack_bf16(r[0], r[1]), pack_bf16(r[2], r[3]));
    }
}

constexpr size_t kBlkLds = (size_t)(4 * 64 * kSkLd + 8 * 64) * 4;
constexpr int kNarrowM = 512, kNarrow16M = 64;
template <int EPI, int NWV, int CT = 64>
static hipError_t blk_gemm_launch_n(dim3 grid, hipStream_t st, const bf16_t *A, const bf16_t *W, int M, int Nn, int K, int Nc, int N,
                                    int n0, const bf16_t *gain, float eps, int norm_free, float alpha, const bf16_t *res_b,
                                    const float *res_f, float *out_f, bf16_t *out_b, const PreOut &po)
{
    static bool raised = false;   // more than the default 64 KB of dynamic LDS
    if (!raised) {
        hipError_t e = hipFuncSetAttribute((const void *)blk_gemm_kernel<EPI, NWV, CT>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)kBlkLds);
        if (e != hipSuccess) return e;
        raised = true;
    }
    hipLaunchKernelGGL((blk_gemm_kernel<EPI, NWV, CT>), grid, dim3(64 * NWV), kBlkLds, st, A, W, M, Nn, K, Nc, N, n0, gain, eps,
                       norm_free, alpha, res_b, res_f, out_f, out_b, po);
    return hipSuccess;
}
// eight wavefronts when every share of the contraction is still a whole number of 32-index steps
template <int EPI>
static hipError_t blk_gemm_launch(dim3 grid, hipStream_t st, const bf16_t *A, const bf16_t *W, int M, int Nn, int K, int Nc, int N,
                                  int n0, const bf16_t *gain, float eps, int norm_free, float alpha, const bf16_t *res_b,
                                  const float *res_f, float *out_f, bf16_t *out_b, const PreOut &po)
{
    if constexpr (EPI != PG_PRE) {
        // few rows: 64-column tiles are then too few workgroups for the weight stream.  Tiles of 32 columns up to kNarrowM
        // rows (MI355X, d = 1024, one position of B sequences: B = 128 52.1 -> 42.0 ms per 512 positions, B = 512 76.6 -> 73.5,
        // B = 1024 139 -> 154), of 16 columns up to kNarrow16M (32 rows: 35.1 -> 31.7 ms per 2048 positions in blocks of 4;
        // 128 rows: 42.3 -> 47.4)
        if (M <= kNarrow16M && K % 256 == 0 && Nn % 32 == 0) {
            grid.y = (unsigned)(Nn / 16);
            return blk_gemm_launch_n<EPI, 8, 16>(grid, st, A, W, M, Nn, K, Nc, N, n0, gain, eps, norm_free, alpha, res_b, res_f, out_f,
                                                 out_b, po);
        }
        if (M <= kNarrowM && K % 256 == 0 && Nn % 32 == 0) {
            grid.y = (unsigned)(Nn / 32);
            return blk_gemm_launch_n<EPI, 8, 32>(grid, st, A, W, M, Nn, K, Nc, N, n0, gain, eps, norm_free, alpha, res_b, res_f, out_f,
                                                 out_b, po);
        }
    }
    // eight shares of a contraction of 1024 are one step group each: with many row tiles four wavefronts (two groups each, one
    // pass less through LDS) are faster (1024 rows, d = 1024: 123.1 -> 121.8 ms per 512 positions)
    if (K % 256 == 0 && !(M >= kNarrowM && K <= 1024))
        return blk_gemm_launch_n<EPI, 8>(grid, st, A, W, M, Nn, K, Nc, N, n0, gain, eps, norm_free, alpha, res_b, res_f, out_f, out_b, po);
    return blk_gemm_launch_n<EPI, 4>(grid, st, A, W, M, Nn, K, Nc, N, n0, gain, eps, norm_free, alpha, res_b, res_f, out_f, out_b, po);
}

// K, V of positions t0 .. t0 + gridDim.y - 1 from the pre-pass outputs (rows (t, b, h)): the caller's cache rows, the bf16 remainder
// of the keys and the transposed values for the tiles.  grid (B*H, N), block 64.
__global__ __launch_bounds__(64) void par_export_kernel(const bf16_t *__restrict__ Ks, const float *__restrict__ Kf,
                                                        const bf16_t *__restrict__ Vs, bf16_t *__restrict__ K,
                                                        bf16_t *__restrict__ V, bf16_t *__restrict__ Klo, uint16_t *__restrict__ Kh,
                                                        bf16_t *__restrict__ VT, int vt_stride, int BH, int t0)
{
    const int lane = threadIdx.x, bh = blockIdx.x, t = t0 + blockIdx.y;
    const size_t off = ((size_t)t * BH + bh) * kHeadDim + lane;
    const bf16_t k = Ks[off], v = Vs[off];
    K[off] = k;
    V[off] = v;
    Klo[off] = f32_to_bf16(Kf[off] - bf16_to_f32(k));
    Kh[off] = f32_to_f16_bits(Kf[off]);
    VT[((size_t)bh * kHeadDim + lane) * vt_stride + t] = v;
}

// The same export for all N positions, 64 positions of one (b, h) per workgroup: every global access is a run of
// 32 bytes or more (the kernel above writes V^T two bytes at a time); the values are transposed through LDS.
// V^T columns N .. 64 ceil(N / 64) - 1 are written as zeros.  grid (B*H, ceil(N / 64)), block 256.
__global__ __launch_bounds__(256) void par_export_tile_kernel(const bf16_t *__restrict__ Ks, const float *__restrict__ Kf,
                                                              const bf16_t *__restrict__ Vs, bf16_t *__restrict__ K,
                                                              bf16_t *__restrict__ V, bf16_t *__restrict__ Klo, uint16_t *__restrict__ Kh,
                                                              bf16_t *__restrict__ VT, int vt_stride, int BH, int N)
{
    constexpr int kLd = 72;
    __shared__ __align__(16) bf16_t tile[64 * kLd];
    const int tid = threadIdx.x, r = tid >> 2, c = tid & 3, bh = blockIdx.x, t0 = blockIdx.y * 64;
    const int t = t0 + r;
    uint4 v0 = make_uint4(0u, 0u, 0u, 0u), v1 = v0;
    if (t < N) {
        const size_t off = ((size_t)t * BH + bh) * kHeadDim + 16 * c;
        const uint4 k0 = *reinterpret_cast<const uint4 *>(Ks + off), k1 = *reinterpret_cast<const uint4 *>(Ks + off + 8);
        v0 = *reinterpret_cast<const uint4 *>(Vs + off);
        v1 = *reinterpret_cast<const uint4 *>(Vs + off + 8);
        float kf[16];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float4 f = *reinterpret_cast<const float4 *>(Kf + off + 4 * j);
            kf[4 * j] = f.x; kf[4 * j + 1] = f.y; kf[4 * j + 2] = f.z; kf[4 * j + 3] = f.w;
        }
        const uint32_t kw[8] = {k0.x, k0.y, k0.z, k0.w, k1.x, k1.y, k1.z, k1.w};
        uint32_t lo[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
            lo[j] = pack_bf16(kf[2 * j] - __uint_as_float(kw[j] << 16), kf[2 * j + 1] - __uint_as_float(kw[j] & 0xFFFF0000u));
        *reinterpret_cast<uint4 *>(K + off) = k0;
        *reinterpret_cast<uint4 *>(K + off + 8) = k1;
        *reinterpret_cast<uint4 *>(V + off) = v0;
        *reinterpret_cast<uint4 *>(V + off + 8) = v1;
        *reinterpret_cast<uint4 *>(Klo + off) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
        *reinterpret_cast<uint4 *>(Klo + off + 8) = make_uint4(lo[4], lo[5], lo[6], lo[7]);
        uint32_t kh[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) kh[j] = pack_f16(kf[2 * j], kf[2 * j + 1]);
        *reinterpret_cast<uint4 *>(Kh + off) = make_uint4(kh[0], kh[1], kh[2], kh[3]);
        *reinterpret_cast<uint4 *>(Kh + off + 8) = make_uint4(kh[4], kh[5], kh[6], kh[7]);
    }
    *reinterpret_cast<uint4 *>(tile + r * kLd + 16 * c) = v0;
    *reinterpret_cast<uint4 *>(tile + r * kLd + 16 * c + 8) = v1;
    __syncthreads();
    // row r of V^T (head dimension r), positions t0 + 16 c .. + 15
    uint32_t w[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
        w[j] = (uint32_t)tile[(16 * c + 2 * j) * kLd + r] | ((uint32_t)tile[(16 * c + 2 * j + 1) * kLd + r] << 16);
    bf16_t *dst = VT + ((size_t)bh * kHeadDim + r) * vt_stride + t0 + 16 * c;
    *reinterpret_cast<uint4 *>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
    *reinterpret_cast<uint4 *>(dst + 8) = make_uint4(w[4], w[5], w[6], w[7]);
}

// a_t of positions t0 .. t0 + gridDim.y - 1 (merge_body) as bf16 rows of [B][N][d].  grid (B*H, positions), block 64.
__global__ __launch_bounds__(64) void par_merge_kernel(const bf16_t *__restrict__ Q, const float *__restrict__ Qf,
                                                       const bf16_t *__restrict__ Kt, const float *__restrict__ Ktf,
                                                       const bf16_t *__restrict__ Vt, const bf16_t *__restrict__ K,
                                                       const bf16_t *__restrict__ Klo, const bf16_t *__restrict__ V,
                                                       const float *__restrict__ pm, const float *__restrict__ pl,
                                                       const float *__restrict__ po, bf16_t *__restrict__ a_out, int BH, int H,
                                                       int N, int p_min, int log2_pmin, int levels, int slots, float scale,
                                                       float alibi, int t0)
{
    const int bh = blockIdx.x, t = t0 + blockIdx.y;
    const float a = merge_body<bf16_t, true>(Q, Qf, Kt, Ktf, Vt, K, Klo, V, pm, pl, po, nullptr, BH, H, bh, t, t, p_min, log2_pmin,
                                             levels, slots, -1, scale, -1, 0, nullptr, alibi);
    const int b = bh / H, h = bh % H;
    a_out[((size_t)b * N + t) * ((size_t)H * kHeadDim) + h * kHeadDim + threadIdx.x] = f32_to_bf16(a);
}

// ---------------------------------------------------------------------------------------------
// Attention of ALL positions in one launch when every key-value pair is known in advance (Sec. 6.1 recompute,
// Sec. 2.1 Transformer layer): query i against the cache rows j < i plus its own temporary pair, as one masked
// flash-style pass instead of Algorithm 1's blocks (no partial states to write and merge).  The inner loop is the one
// of cross_tile_wg (key and V^T chunks of 64 keys staged in LDS and shared by four wavefronts of 32 queries; logits
// from unrounded operands: with F16 the queries (fp32, times scale log2 e) and the keys (the fp16 copy of the cache,
// passed in the Klo argument; K is then not read) are rounded once to fp16 and S^T is one product, as in the tiles of
// the sequential engines; without it bf16 head + remainder and three products per tile); additionally
//   - the state of a query starts from its temporary pair (m = its logit from the unrounded q and k_tmp, l = 1,
//     o = v_tmp), so that every query has a finite reference before the first key,
//   - chunks that reach a wavefront's own positions mask keys j >= i with -inf,
//   - with ALIBI the bias slope (j - i) is applied per (key, query),
//   - the result is normalised and written as bf16 rows of a [B][N][d].
// One workgroup per (128 queries, b, h).  grid ceil(N / 128) * B*H, block 256, LDS 2 x 27 KB.  When B*H is a multiple of
// 8 the workgroups are numbered so that all query tiles of one (b, h) run on the same XCD one after the other (their
// keys and values then come out of that XCD's L2), the longest first.
// ---------------------------------------------------------------------------------------------
// F32OUT (the backward pass's recompute): the result goes out as fp32 rows c_out[(i B H + bh) 64 ..] together with the
// log-sum-exp of the query's logits (natural log), lse_out[i B H + bh], instead of bf16 rows of a_out.
template <bool ALIBI, bool F32OUT = false, bool F16 = !F32OUT>
__global__ __launch_bounds__(256) void par_flash_kernel(const float *__restrict__ Qf, const float *__restrict__ Ktf,
                                                        const bf16_t *__restrict__ Vt, const bf16_t *__restrict__ K,
                                                        const bf16_t *__restrict__ Klo, const bf16_t *__restrict__ VT,
                                                        int vt_stride, bf16_t *__restrict__ a_out, int BH, int H, int N,
                                                        int ntiles, float scale, float alibi, float *__restrict__ c_out = nullptr,
                                                        float *__restrict__ lse_out = nullptr, const bf16_t *__restrict__ VTlo = nullptr,
                                                        const float *__restrict__ Vt32 = nullptr)
{
    extern __shared__ __align__(16) unsigned char flash_lds[];
    constexpr int T = 256, PPT = 2;
    static_assert(!(F32OUT && F16), "the fp32-output form keeps the three-product logits");
    constexpr int TILE = kKC * kTileLd, BUF = (F32OUT ? 4 : (F16 ? 2 : 3)) * TILE;   // keys, V^T[, key remainder[, V^T remainder]]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    int bh, qt;
    {
        const int L = blockIdx.x;
        if (BH % 8 == 0) {
            const int xcd = L & 7, idx = L >> 3;
            bh = xcd + 8 * (idx / ntiles);
            qt = ntiles - 1 - idx % ntiles;
        } else {
            bh = L / ntiles;
            qt = ntiles - 1 - L % ntiles;
        }
    }
    const int q0w = qt * 128 + 32 * wave;          // first query of this wavefront
    const bool active = q0w < N;                    // wave-uniform
    const int qpos = q0w + l32;                     // this lane's query (its partner lane hi ^ 1 holds the same one)
    const int qi = min(qpos, N - 1);
    const size_t rs = (size_t)BH * kHeadDim;
    bf16_t *tiles = reinterpret_cast<bf16_t *>(flash_lds);
    const float c2 = scale * kLog2e;
    const float s2 = ALIBI ? alibi_slope(alibi, bh % H, H) * kLog2e : 0.f;

    // ---- queries as B fragments (head + remainder), and the temporary pair's logit
    uint4 bq[4], bql[4];
    float m2, lsum = hi == 0 ? 1.f : 0.f;
    f32x16_t O[2];
    {
        const size_t qo = (size_t)qi * rs + (size_t)bh * kHeadDim;
        float dot = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            float f[8], r[8], kf[8];
            load8(Qf + qo + 8 * hi + ks * 16, f);
            load8(Ktf + qo + 8 * hi + ks * 16, kf);
#pragma unroll
            for (int e = 0; e < 8; ++e) dot = fmaf(f[e], kf[e], dot);
            if (F16) {   // the product then delivers the logits in log2 units
                bq[ks] = make_uint4(cvt_pk_f16(f[0] * c2, f[1] * c2), cvt_pk_f16(f[2] * c2, f[3] * c2), cvt_pk_f16(f[4] * c2, f[5] * c2),
                                    cvt_pk_f16(f[6] * c2, f[7] * c2));
                bql[ks] = bq[ks];   // not used
                continue;
            }
            uint32_t h2[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                h2[e] = cvt_pk_bf16(f[2 * e], f[2 * e + 1]);
                r[2 * e] = f[2 * e] - __uint_as_float(h2[e] << 16);
                r[2 * e + 1] = f[2 * e + 1] - __uint_as_float(h2[e] & 0xFFFF0000u);
            }
            bq[ks] = make_uint4(h2[0], h2[1], h2[2], h2[3]);
            bql[ks] = make_uint4(cvt_pk_bf16(r[0], r[1]), cvt_pk_bf16(r[2], r[3]), cvt_pk_bf16(r[4], r[5]), cvt_pk_bf16(r[6], r[7]));
        }
        dot += __shfl_xor(dot, 32, 64);
        m2 = dot * c2;                              // distance 0: no bias
        // register i of tile dt is head dimension 32dt + 8(i/4) + 4hi + i%4
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (F32OUT) {   // the temporary value unrounded
                    const float4 v4 = *reinterpret_cast<const float4 *>(Vt32 + qo + 32 * dt + 8 * j + 4 * hi);
                    O[dt][4 * j] = v4.x; O[dt][4 * j + 1] = v4.y; O[dt][4 * j + 2] = v4.z; O[dt][4 * j + 3] = v4.w;
                    continue;
                }
                const uint2 v = *reinterpret_cast<const uint2 *>(Vt + qo + 32 * dt + 8 * j + 4 * hi);
                O[dt][4 * j] = __uint_as_float(v.x << 16);
                O[dt][4 * j + 1] = __uint_as_float(v.x & 0xFFFF0000u);
                O[dt][4 * j + 2] = __uint_as_float(v.y << 16);
                O[dt][4 * j + 3] = __uint_as_float(v.y & 0xFFFF0000u);
            }
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- staging of one chunk: thread -> 16-byte piece, 8 consecutive threads cover one row; key rows past the last
    // position are read from the last one (they are masked), V^T columns up to vt_stride exist and hold finite values
    u32x4_t rk[PPT], rl[PPT], rv[PPT], rv2[PPT];
    const int prow = tid >> 3, pc16 = tid & 7;
    const bf16_t *gv = VT + ((size_t)bh * kHeadDim + prow) * vt_stride + pc16 * 8;
    const bf16_t *gv2 = F32OUT ? VTlo + ((size_t)bh * kHeadDim + prow) * vt_stride + pc16 * 8 : nullptr;
    const int lds_off = prow * kTileLd + pc16 * 8, lds_off_v = prow * kVLd + pc16 * 8;
#define RT_FL_FETCH(kc)                                                                                               \
    _Pragma("unroll") for (int i = 0; i < PPT; ++i)                                                                   \
    {                                                                                                                 \
        const size_t ro = (size_t)min((kc) + prow + i * (T / 8), N - 1) * rs + (size_t)bh * kHeadDim + pc16 * 8;      \
        rk[i] = *reinterpret_cast<const u32x4_t *>((F16 ? Klo : K) + ro);                                             \
        if (!F16) rl[i] = *reinterpret_cast<const u32x4_t *>(Klo + ro);                                               \
        rv[i] = *reinterpret_cast<const u32x4_t *>(gv + (size_t)(i * (T / 8)) * vt_stride + (kc));                    \
        if (F32OUT) rv2[i] = *reinterpret_cast<const u32x4_t *>(gv2 + (size_t)(i * (T / 8)) * vt_stride + (kc));      \
    }
#define RT_FL_STAGE(buf)                                                                                              \
    _Pragma("unroll") for (int i = 0; i < PPT; ++i)                                                                   \
    {                                                                                                                 \
        bf16_t *dst = tiles + (size_t)(buf) * BUF + lds_off + i * (T / 8) * kTileLd;                                  \
        *reinterpret_cast<u32x4_t *>(dst) = rk[i];                                                                    \
        bf16_t *dv = tiles + (size_t)(buf) * BUF + TILE + lds_off_v + i * (T / 8) * kVLd;                             \
        *reinterpret_cast<uint2 *>(dv) = make_uint2(rv[i][0], rv[i][1]);                                              \
        *reinterpret_cast<uint2 *>(dv + 4) = make_uint2(rv[i][2], rv[i][3]);                                          \
        if (!F16) *reinterpret_cast<u32x4_t *>(dst + 2 * TILE) = rl[i];                                               \
        if (F32OUT) {                                                                                                 \
            bf16_t *dv2 = tiles + (size_t)(buf) * BUF + 3 * TILE + lds_off_v + i * (T / 8) * kVLd;                    \
            *reinterpret_cast<uint2 *>(dv2) = make_uint2(rv2[i][0], rv2[i][1]);                                       \
            *reinterpret_cast<uint2 *>(dv2 + 4) = make_uint2(rv2[i][2], rv2[i][3]);                                   \
        }                                                                                                             \
    }

    const int kend = min(qt * 128 + 128, N);        // keys 0 .. kend - 2 are needed by some query of the tile
    const int nchunks = (kend - 1 + kKC - 1) / kKC; // workgroup-uniform; 0 for the single position 0
    if (nchunks > 0) {
        RT_FL_FETCH(0)
        RT_FL_STAGE(0)
    }
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
        const int cur = c & 1;
        if (c + 1 < nchunks) { RT_FL_FETCH((c + 1) * kKC) }
        if (active && c * kKC < q0w + 31) {          // some key of the chunk precedes some query of the wavefront
            const bf16_t *Ks = tiles + (size_t)cur * BUF, *Vs = Ks + TILE;
            f32x16_t S[2];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                const bf16_t *krow = Ks + (kt * 32 + l32) * kTileLd + 8 * hi;
                uint4 ka[4];
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) ka[ks] = *reinterpret_cast<const uint4 *>(krow + ks * 16);
                f32x16_t acc;
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[i] = 0.f;
                if (F16) {
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) acc = mfma32h(ka[ks], bq[ks], acc);
                } else {
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)      // small terms first
                        acc = mfma32u(*reinterpret_cast<const uint4 *>(krow + 2 * TILE + ks * 16), bq[ks], acc);
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) acc = mfma32u(ka[ks], bql[ks], acc);
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) acc = mfma32u(ka[ks], bq[ks], acc);
                }
                S[kt] = acc;
            }
            // register i of tile kt is key 64c + 32kt + 8(i/4) + 4hi + i%4; from here on S is in log2 units
            if (ALIBI || !F16) {
                const float base = ALIBI ? s2 * (float)(c * kKC + 4 * hi - qpos) : 0.f;
                const float cs = F16 ? 1.f : c2;
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        S[kt][i] = ALIBI ? fmaf(S[kt][i], cs, fmaf(s2, (float)(32 * kt + 8 * (i / 4) + (i % 4)), base)) : S[kt][i] * cs;
            }
            if (c * kKC + kKC > q0w) {               // the chunk reaches this wavefront's own positions: keys j >= i out
                const int lim = qpos - (c * kKC + 4 * hi);   // valid iff 32kt + 8(i/4) + i%4 < lim
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        if (32 * kt + 8 * (i / 4) + (i % 4) >= lim) S[kt][i] = -INFINITY;
            }
            float lmax = fmaxf(fmaxf(S[0][0], S[0][1]), S[0][2]);
#pragma unroll
            for (int i = 3; i < 15; i += 2) lmax = fmaxf(fmaxf(lmax, S[0][i]), S[0][i + 1]);
            lmax = fmaxf(fmaxf(lmax, S[0][15]), S[1][0]);
#pragma unroll
            for (int i = 1; i < 15; i += 2) lmax = fmaxf(fmaxf(lmax, S[1][i]), S[1][i + 1]);
            lmax = fmaxf(lmax, S[1][15]);
            const bool over = lmax > m2 + kSlack;
            if (__any(over)) {
                const float mx = fmaxf(lmax, __shfl_xor(lmax, 32, 64));
                const float m_new = fmaxf(m2, mx);
                const float resc = __builtin_amdgcn_exp2f(m2 - m_new);   // m2 is finite from the start
                m2 = m_new;
                lsum *= resc;
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) O[dt] *= resc;
            }
            uint4 bp[4], bpl[4];
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                float pw[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) pw[e] = __builtin_amdgcn_exp2f(S[s4 >> 1][8 * (s4 & 1) + e] - m2);
                bp[s4] = make_uint4(cvt_pk_bf16(pw[0], pw[1]), cvt_pk_bf16(pw[2], pw[3]), cvt_pk_bf16(pw[4], pw[5]), cvt_pk_bf16(pw[6], pw[7]));
                lsum += ((pw[0] + pw[1]) + (pw[2] + pw[3])) + ((pw[4] + pw[5]) + (pw[6] + pw[7]));
                if (F32OUT) {   // what the bf16 weights lost: the weights and the values both enter as head + remainder
                    const uint32_t hw[4] = {bp[s4].x, bp[s4].y, bp[s4].z, bp[s4].w};
                    uint32_t lw[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        lw[e] = cvt_pk_bf16(pw[2 * e] - __uint_as_float(hw[e] << 16), pw[2 * e + 1] - __uint_as_float(hw[e] & 0xFFFF0000u));
                    bpl[s4] = make_uint4(lw[0], lw[1], lw[2], lw[3]);
                }
            }
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) {
                    const bf16_t *vrow = Vs + (dt * 32 + l32) * kVLd + s4 * 16 + 4 * hi;
                    const uint2 v0 = *reinterpret_cast<const uint2 *>(vrow), v1 = *reinterpret_cast<const uint2 *>(vrow + 8);
                    if (F32OUT) {   // small terms first
                        const bf16_t *vrow2 = vrow + 2 * TILE;   // the remainder tile
                        const uint2 u0 = *reinterpret_cast<const uint2 *>(vrow2), u1 = *reinterpret_cast<const uint2 *>(vrow2 + 8);
                        O[dt] = mfma32u(make_uint4(u0.x, u0.y, u1.x, u1.y), bp[s4], O[dt]);
                        O[dt] = mfma32u(make_uint4(v0.x, v0.y, v1.x, v1.y), bpl[s4], O[dt]);
                    }
                    O[dt] = mfma32u(make_uint4(v0.x, v0.y, v1.x, v1.y), bp[s4], O[dt]);
                }
            }
        }
        if (c + 1 < nchunks) {
            RT_FL_STAGE(cur ^ 1)
            __syncthreads();
        }
    }
#undef RT_FL_FETCH
#undef RT_FL_STAGE

    if (F32OUT) {
        if (active && qpos < N) {
            const float lt = lsum + __shfl_xor(lsum, 32, 64), inv = 1.f / lt;
            float *crow = c_out + ((size_t)qpos * BH + bh) * kHeadDim + 4 * hi;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    *reinterpret_cast<float4 *>(crow + dt * 32 + 8 * j) =
                        make_float4(O[dt][4 * j] * inv, O[dt][4 * j + 1] * inv, O[dt][4 * j + 2] * inv, O[dt][4 * j + 3] * inv);
            if (hi == 0) lse_out[(size_t)qpos * BH + bh] = m2 * kLn2 + logf(lt);
        }
        return;
    }
    if (active && qpos < N) {
        const float inv = 1.f / (lsum + __shfl_xor(lsum, 32, 64));
        const int b = bh / H, h = bh % H;
        bf16_t *arow = a_out + ((size_t)b * N + qpos) * ((size_t)H * kHeadDim) + h * kHeadDim + 4 * hi;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                *reinterpret_cast<uint2 *>(arow + dt * 32 + 8 * j) =
                    make_uint2(cvt_pk_bf16(O[dt][4 * j] * inv, O[dt][4 * j + 1] * inv), cvt_pk_bf16(O[dt][4 * j + 2] * inv, O[dt][4 * j + 3] * inv));
    }
}

constexpr int kSmallM = 2048;   // up to this many rows the split-contraction kernel is used (it is 1.4x slower at 16384 rows)

// the pre-pass projection of positions n0 .. n0 + Nc - 1 of every batch row of `src` with the split-contraction kernel
// pairs_to: the caller's K (with V): only the pairs are projected and they go straight into the cache rows and their copies
// write_vt = false: the transposed copy of the values is left to vt_from_rows_kernel
static hipError_t small_prepass(const LayerDims &D, const Weights &W, const Scratch &S, const void *src, int n0, int Nc, hipStream_t st,
                                void *pairs_K = nullptr, void *pairs_V = nullptr, bool write_vt = true)
{
    PreOut po = {};
    po.Wq = (const bf16_t *)W.Wq; po.Wk = (const bf16_t *)W.Wk; po.Wv = (const bf16_t *)W.Wv;
    po.g_q = (const bf16_t *)W.g_q; po.g_k = (const bf16_t *)W.g_k;
    po.Q = (bf16_t *)S.Q; po.Kt = (bf16_t *)S.Kt; po.Vt = (bf16_t *)S.Vt; po.Qf = S.Qf; po.Ktf = S.Ktf;
    po.H = D.H; po.Bc = D.B;
    if (pairs_K) {
        po.y0 = D.H;
        po.K = (bf16_t *)pairs_K; po.V = (bf16_t *)pairs_V; po.Klo = S.Klo; po.Kh = S.Kh; po.VT = write_vt ? S.VT : nullptr;
        po.vt_stride = S.vt_stride;
    }
    const int M = D.B * Nc;
    return blk_gemm_launch<PG_PRE>(dim3((unsigned)((M + 63) / 64), (unsigned)((pairs_K ? 2 : 3) * D.H)), st, (const bf16_t *)src, nullptr, M, 3 * D.d,
                                   D.d, Nc, D.N, n0, (const bf16_t *)W.g_attn, D.eps, D.norm_free, D.alpha, nullptr, nullptr,
                                   nullptr, nullptr, po);
}

// h = x + alpha Wo a;  u = gelu(W1 RMS(h));  y = h + alpha W2 u  for positions n0 .. n0 + Nc - 1 of every batch row
static void block_gemms(const LayerDims &D, const Weights &W, const void *x, void *y, bf16_t *a_b, float *h_f, bf16_t *h_b,
                        bf16_t *u_b, float *rinv, int n0, int Nc, hipStream_t st)
{
    const int d = D.d, F = D.F, M = D.B * Nc;
    if (M <= kSmallM && d % 128 == 0 && F % 128 == 0) {   // few rows: the split-contraction kernel
        const unsigned gs = (unsigned)((M + 63) / 64);
        const PreOut none = {};
        (void)blk_gemm_launch<PG_WO>(dim3(gs, (unsigned)(d / 64)), st, a_b, (const bf16_t *)W.Wo, M, d, d, Nc, D.N, n0, nullptr, D.eps,
                                     D.norm_free, D.alpha, (const bf16_t *)x, nullptr, h_f, h_b, none);
        // W1 from 1024 rows on: 128 x 128 tiles (half the operand traffic of the 64 x 64 ones, which then bounds the product;
        // 1024 rows, d = 1024: 121.3 -> 115.0 ms per 512 positions; at 512 rows 71.4 -> 75.4)
        if (M >= 1024)
            hipLaunchKernelGGL(par_gemm_kernel<PG_W1>, dim3((unsigned)((M + 127) / 128), (unsigned)((F + 127) / 128)), dim3(256), 0, st, h_b,
                               (const bf16_t *)W.W1, M, F, d, Nc, D.N, n0, (const bf16_t *)W.g_mlp, D.eps, D.norm_free, D.alpha,
                               (const bf16_t *)nullptr, (const float *)nullptr, (float *)nullptr, u_b);
        else
            (void)blk_gemm_launch<PG_W1>(dim3(gs, (unsigned)(F / 64)), st, h_b, (const bf16_t *)W.W1, M, F, d, Nc, D.N, n0,
                                         (const bf16_t *)W.g_mlp, D.eps, D.norm_free, D.alpha, nullptr, nullptr, nullptr, u_b, none);
        (void)blk_gemm_launch<PG_W2>(dim3(gs, (unsigned)(d / 64)), st, u_b, (const bf16_t *)W.W2, M, d, F, Nc, D.N, n0, nullptr, D.eps,
                                     D.norm_free, D.alpha, nullptr, h_f, nullptr, (bf16_t *)y, none);
        return;
    }
    if (d % 128 == 0 && F % 128 == 0) {   // both operands through LDS
        const unsigned gt = (unsigned)((M + 255) / 256);
        hipLaunchKernelGGL(tiled_gemm_kernel<PG_WO>, dim3(gt, (unsigned)(d / 128)), dim3(256), 0, st, a_b, (const bf16_t *)W.Wo, M, d, d,
                           Nc, D.N, n0, (const bf16_t *)W.g_mlp, (const float *)nullptr, D.norm_free, D.alpha, (const bf16_t *)x,
                           (const float *)nullptr, h_f, h_b);
        if (!D.norm_free)
            hipLaunchKernelGGL(par_rinv_kernel, dim3((unsigned)((M + 3) / 4)), dim3(256), 0, st, h_f, rinv, M, Nc, D.N, n0, d, D.eps);
        hipLaunchKernelGGL(tiled_gemm_kernel<PG_W1>, dim3(gt, (unsigned)(F / 128)), dim3(256), 0, st, h_b, (const bf16_t *)W.W1, M, F, d,
                           Nc, D.N, n0, (const bf16_t *)nullptr, rinv, D.norm_free, D.alpha, (const bf16_t *)nullptr,
                           (const float *)nullptr, (float *)nullptr, u_b);
        hipLaunchKernelGGL(tiled_gemm_kernel<PG_W2>, dim3(gt, (unsigned)(d / 128)), dim3(256), 0, st, u_b, (const bf16_t *)W.W2, M, d, F,
                           Nc, D.N, n0, (const bf16_t *)nullptr, (const float *)nullptr, D.norm_free, D.alpha,
                           (const bf16_t *)nullptr, h_f, (float *)nullptr, (bf16_t *)y);
        return;
    }
    const unsigned gm = (unsigned)((M + 127) / 128);
    hipLaunchKernelGGL(par_gemm_kernel<PG_WO>, dim3(gm, (unsigned)((d + 127) / 128)), dim3(256), 0, st, a_b, (const bf16_t *)W.Wo, M, d,
                       d, Nc, D.N, n0, (const bf16_t *)nullptr, D.eps, D.norm_free, D.alpha, (const bf16_t *)x,
                       (const float *)nullptr, h_f, h_b);
    hipLaunchKernelGGL(par_gemm_kernel<PG_W1>, dim3(gm, (unsigned)((F + 127) / 128)), dim3(256), 0, st, h_b, (const bf16_t *)W.W1, M, F,
                       d, Nc, D.N, n0, (const bf16_t *)W.g_mlp, D.eps, D.norm_free, D.alpha, (const bf16_t *)nullptr,
                       (const float *)nullptr, (float *)nullptr, u_b);
    hipLaunchKernelGGL(par_gemm_kernel<PG_W2>, dim3(gm, (unsigned)((d + 127) / 128)), dim3(256), 0, st, u_b, (const bf16_t *)W.W2, M, d,
                       F, Nc, D.N, n0, (const bf16_t *)nullptr, D.eps, D.norm_free, D.alpha, (const bf16_t *)nullptr, h_f,
                       (float *)nullptr, (bf16_t *)y);
}

// For the backward pass's recompute: the persistent pairs and the temporary values as fp32 rows [N][B H][64] -> the bf16
// head and remainder of the keys, the bf16 values transposed (columns N .. 64 ceil(N / 64) - 1 zero) and the bf16
// temporary values, 64 positions of one (b, h) per workgroup.  grid (B*H, ceil(N / 64)), block 256.
__global__ __launch_bounds__(256) void flash_export_f32_kernel(const float *__restrict__ Kf, const float *__restrict__ Vf,
                                                               const float *__restrict__ Vtf, bf16_t *__restrict__ K,
                                                               bf16_t *__restrict__ Klo, bf16_t *__restrict__ VT,
                                                               bf16_t *__restrict__ VTlo, bf16_t *__restrict__ Vt, int vt_stride,
                                                               int BH, int N)
{
    constexpr int kLd = 72;
    __shared__ __align__(16) bf16_t tile[2 * 64 * kLd];   // head and remainder of the values
    const int tid = threadIdx.x, r = tid >> 2, c = tid & 3, bh = blockIdx.x, t0 = blockIdx.y * 64;
    const int t = t0 + r;
    uint32_t vb[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u}, vl[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
    if (t < N) {
        const size_t off = ((size_t)t * BH + bh) * kHeadDim + 16 * c;
        float kf[16], vf[16], tf[16];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float4 a = *reinterpret_cast<const float4 *>(Kf + off + 4 * j), b = *reinterpret_cast<const float4 *>(Vf + off + 4 * j),
                         e = *reinterpret_cast<const float4 *>(Vtf + off + 4 * j);
            kf[4 * j] = a.x; kf[4 * j + 1] = a.y; kf[4 * j + 2] = a.z; kf[4 * j + 3] = a.w;
            vf[4 * j] = b.x; vf[4 * j + 1] = b.y; vf[4 * j + 2] = b.z; vf[4 * j + 3] = b.w;
            tf[4 * j] = e.x; tf[4 * j + 1] = e.y; tf[4 * j + 2] = e.z; tf[4 * j + 3] = e.w;
        }
        uint32_t kh[8], kl[8], tb[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            kh[j] = pack_bf16(kf[2 * j], kf[2 * j + 1]);
            kl[j] = pack_bf16(kf[2 * j] - __uint_as_float(kh[j] << 16), kf[2 * j + 1] - __uint_as_float(kh[j] & 0xFFFF0000u));
            vb[j] = pack_bf16(vf[2 * j], vf[2 * j + 1]);
            vl[j] = pack_bf16(vf[2 * j] - __uint_as_float(vb[j] << 16), vf[2 * j + 1] - __uint_as_float(vb[j] & 0xFFFF0000u));
            tb[j] = pack_bf16(tf[2 * j], tf[2 * j + 1]);
        }
        *reinterpret_cast<uint4 *>(K + off) = make_uint4(kh[0], kh[1], kh[2], kh[3]);
        *reinterpret_cast<uint4 *>(K + off + 8) = make_uint4(kh[4], kh[5], kh[6], kh[7]);
        *reinterpret_cast<uint4 *>(Klo + off) = make_uint4(kl[0], kl[1], kl[2], kl[3]);
        *reinterpret_cast<uint4 *>(Klo + off + 8) = make_uint4(kl[4], kl[5], kl[6], kl[7]);
        *reinterpret_cast<uint4 *>(Vt + off) = make_uint4(tb[0], tb[1], tb[2], tb[3]);
        *reinterpret_cast<uint4 *>(Vt + off + 8) = make_uint4(tb[4], tb[5], tb[6], tb[7]);
    }
    *reinterpret_cast<uint4 *>(tile + r * kLd + 16 * c) = make_uint4(vb[0], vb[1], vb[2], vb[3]);
    *reinterpret_cast<uint4 *>(tile + r * kLd + 16 * c + 8) = make_uint4(vb[4], vb[5], vb[6], vb[7]);
    *reinterpret_cast<uint4 *>(tile + (64 + r) * kLd + 16 * c) = make_uint4(vl[0], vl[1], vl[2], vl[3]);
    *reinterpret_cast<uint4 *>(tile + (64 + r) * kLd + 16 * c + 8) = make_uint4(vl[4], vl[5], vl[6], vl[7]);
    __syncthreads();
#pragma unroll
    for (int part = 0; part < 2; ++part) {
        const bf16_t *tp = tile + part * 64 * kLd;
        uint32_t w[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
            w[j] = (uint32_t)tp[(16 * c + 2 * j) * kLd + r] | ((uint32_t)tp[(16 * c + 2 * j + 1) * kLd + r] << 16);
        bf16_t *dst = (part == 0 ? VT : VTlo) + ((size_t)bh * kHeadDim + r) * vt_stride + t0 + 16 * c;
        *reinterpret_cast<uint4 *>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
        *reinterpret_cast<uint4 *>(dst + 8) = make_uint4(w[4], w[5], w[6], w[7]);
    }
}

size_t flash_recompute_scratch_bytes(size_t B, size_t N, size_t d, size_t H)
{
    const size_t M = B * N, vt_stride = (N + 63) / 64 * 64;
    auto up = [](size_t v) { return (v + 255) / 256 * 256; };
    return 3 * up(M * d * 2) + 2 * up(B * H * kHeadDim * vt_stride * 2);
}

hipError_t flash_recompute_f32(const LayerDims &D, const float *Qn, const float *Ktn, const float *Vt, const float *Kp, const float *Vp,
                               float *c, float *lse, void *scratch, hipStream_t st)
{
    const int B = D.B, N = D.N, BH = B * D.H;
    const size_t M = (size_t)B * N, vt_stride = ((size_t)N + 63) / 64 * 64;
    auto up = [](size_t v) { return (v + 255) / 256 * 256; };
    char *p = (char *)scratch;
    bf16_t *Kb = (bf16_t *)p; p += up(M * D.d * 2);
    bf16_t *Klo = (bf16_t *)p; p += up(M * D.d * 2);
    bf16_t *Vtb = (bf16_t *)p; p += up(M * D.d * 2);
    bf16_t *VT = (bf16_t *)p; p += up((size_t)BH * kHeadDim * vt_stride * 2);
    bf16_t *VTlo = (bf16_t *)p;
    hipLaunchKernelGGL(flash_export_f32_kernel, dim3(BH, (N + 63) / 64), dim3(256), 0, st, Kp, Vp, Vt, Kb, Klo, VT, VTlo, Vtb,
                       (int)vt_stride, BH, N);
    const int ntiles = (N + 127) / 128;
    const size_t lds = 2 * 4 * (size_t)kKC * kTileLd * 2;   // two buffers of four tiles: keys, V^T, key remainder, V^T remainder
    static bool raised = false;
    if (!raised) {
        hipError_t e = hipFuncSetAttribute((const void *)par_flash_kernel<true, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)par_flash_kernel<false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        raised = true;
    }
    const dim3 grid((unsigned)(ntiles * BH));
    if (D.alibi > 0.f)
        hipLaunchKernelGGL((par_flash_kernel<true, true>), grid, dim3(256), lds, st, Qn, Ktn, Vtb, Kb, Klo, VT, (int)vt_stride,
                           (bf16_t *)nullptr, BH, D.H, N, ntiles, D.scale, D.alibi, c, lse, VTlo, Vt);
    else
        hipLaunchKernelGGL((par_flash_kernel<false, true>), grid, dim3(256), lds, st, Qn, Ktn, Vtb, Kb, Klo, VT, (int)vt_stride,
                           (bf16_t *)nullptr, BH, D.H, N, ntiles, D.scale, D.alibi, c, lse, VTlo, Vt);
    return hipGetLastError();
}

bool parallel_supported(const LayerDims &D, bool mfma_bf16) { return mfma_bf16 && D.d % 64 == 0 && D.F % 64 == 0; }

size_t parallel_scratch_bytes(size_t M, size_t d, size_t F) { return M * d * 2 + M * d * 4 + M * d * 2 + M * F * 2 + 1024; }

// pairs_src: the rows the persistent pairs are projected from (z for the recompute, x for the Transformer layer);
// pairs_gain: the RMS gain that goes with them (g_kv or g_attn).  par: parallel_scratch_bytes(B * N, d, F) bytes.
hipError_t parallel_layer(const LayerDims &D, const Weights &W, const Scratch &S, const void *x, const void *pairs_src,
                          bool pairs_are_temporary, void *y, void *K, void *V, void *par, hipStream_t st)
{
    const int B = D.B, N = D.N, d = D.d, F = D.F, BH = B * D.H, M = B * N;
    char *p = (char *)par;
    auto up = [](size_t v) { return (v + 255) / 256 * 256; };
    bf16_t *a_b = (bf16_t *)p; p += up((size_t)M * d * 2);
    float *h_f = (float *)p; p += up((size_t)M * d * 4);
    bf16_t *h_b = (bf16_t *)p; p += up((size_t)M * d * 2);
    bf16_t *u_b = (bf16_t *)p;

    Weights Wp = W;
    if (!pairs_are_temporary) Wp.g_attn = W.g_kv;
    hipError_t e = Launch<bf16_t>::prepass(D, Wp, S, pairs_src, B, N, true, st);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(par_export_tile_kernel, dim3(BH, (N + 63) / 64), dim3(256), 0, st, (const bf16_t *)S.Kt, S.Ktf,
                       (const bf16_t *)S.Vt, (bf16_t *)K, (bf16_t *)V, S.Klo, S.Kh, S.VT, S.vt_stride, BH, N);
    if (!pairs_are_temporary) {
        e = Launch<bf16_t>::prepass(D, W, S, x, B, N, true, st);
        if (e != hipSuccess) return e;
    }
    {   // attention of all positions: one masked pass over the cache rows plus the temporary pair
        const int ntiles = (N + 127) / 128;
        const size_t lds = 2 * (size_t)cross_tile_lds_bytes<true, true>();   // two tiles per buffer: fp16 keys, V^T
        const dim3 grid((unsigned)(ntiles * BH));
        const bf16_t *Kh = (const bf16_t *)S.Kh;   // 2-byte elements either way; the kernel reads them as fp16
        if (D.alibi > 0.f)
            hipLaunchKernelGGL(par_flash_kernel<true>, grid, dim3(256), lds, st, S.Qf, S.Ktf, (const bf16_t *)S.Vt, (const bf16_t *)K,
                               Kh, S.VT, S.vt_stride, a_b, BH, D.H, N, ntiles, D.scale, D.alibi);
        else
            hipLaunchKernelGGL(par_flash_kernel<false>, grid, dim3(256), lds, st, S.Qf, S.Ktf, (const bf16_t *)S.Vt, (const bf16_t *)K,
                               Kh, S.VT, S.vt_stride, a_b, BH, D.H, N, ntiles, D.scale, D.alibi);
    }
    block_gemms(D, W, x, y, a_b, h_f, h_b, u_b, S.rinv, 0, N, st);
    return hipGetLastError();
}

// Blocked recurrence (Sec. 8, Discussion; the reading is stated at rt_layer_prefill_blocked in rt.h): blocks of Sblk
// positions, a power of two that divides p_min, so that every event of Algorithm 1 falls on a block boundary.  While
// a block is evaluated its rows of K, V hold the TEMPORARY pairs (the direct window of merge_body then reads
// persistent pairs of earlier blocks and temporary pairs of the own block without knowing the difference); after the
// block's outputs are there they are overwritten with the persistent pairs projected from those outputs.
// The transposed copy of the values for positions t_lo + 32 blockIdx.y .. + 31 of head (b, h) = blockIdx.x from the cache rows:
// written position by position it costs a 64-byte write per 2-byte element; here a workgroup turns a 32 x 64 tile through
// LDS and writes 64-byte runs.  t_lo a multiple of 32.  grid (B*H, positions / 32), block 256.
__global__ __launch_bounds__(256) void vt_from_rows_kernel(const bf16_t *__restrict__ V, bf16_t *__restrict__ VT, int vt_stride, int BH,
                                                           int t_lo)
{
    constexpr int kLd = 72;
    __shared__ __align__(16) bf16_t tile[32 * kLd];
    const int tid = threadIdx.x, bh = blockIdx.x, t0 = t_lo + 32 * (int)blockIdx.y;
    {
        const int r = tid >> 3, c = tid & 7;
        *reinterpret_cast<uint4 *>(tile + r * kLd + 8 * c) =
            *reinterpret_cast<const uint4 *>(V + ((size_t)(t0 + r) * BH + bh) * kHeadDim + 8 * c);
    }
    __syncthreads();
    const int dim = tid >> 2, q = tid & 3;
    uint32_t w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        w[j] = (uint32_t)tile[(8 * q + 2 * j) * kLd + dim] | ((uint32_t)tile[(8 * q + 2 * j + 1) * kLd + dim] << 16);
    *reinterpret_cast<uint4 *>(VT + ((size_t)bh * kHeadDim + dim) * vt_stride + t0 + 8 * q) = make_uint4(w[0], w[1], w[2], w[3]);
}

hipError_t blocked_layer(const LayerDims &D, const Weights &W, const Scratch &S, const void *x, int Sblk, void *y, void *K, void *V,
                         void *par, hipStream_t st)
{
    const int B = D.B, N = D.N, d = D.d, F = D.F, BH = B * D.H;
    const size_t Mmax = (size_t)B * N;
    char *p = (char *)par;
    auto up = [](size_t v) { return (v + 255) / 256 * 256; };
    bf16_t *a_b = (bf16_t *)p; p += up(Mmax * d * 2);
    float *h_f = (float *)p; p += up(Mmax * d * 4);
    bf16_t *h_b = (bf16_t *)p; p += up(Mmax * d * 2);
    bf16_t *u_b = (bf16_t *)p;
    (void)F;
    Weights Wp = W;
    Wp.g_attn = W.g_kv;
    hipError_t e = Launch<bf16_t>::prepass(D, W, S, x, B, N, true, st);   // q and temporary pairs of every position
    if (e != hipSuccess) return e;
    // the temporary pairs of ALL positions go into the cache rows at once: a block reads rows below its own end only, and its
    // rows receive the persistent pairs when it is done
    hipLaunchKernelGGL(par_export_tile_kernel, dim3(BH, (N + 63) / 64), dim3(256), 0, st, (const bf16_t *)S.Kt, S.Ktf,
                       (const bf16_t *)S.Vt, (bf16_t *)K, (bf16_t *)V, S.Klo, S.Kh, S.VT, S.vt_stride, BH, N);
    for (int t0 = 0; t0 < N; t0 += Sblk) {
        const int nr = Sblk < N - t0 ? Sblk : N - t0;
        hipLaunchKernelGGL(par_merge_kernel, dim3(BH, nr), dim3(64), 0, st, (const bf16_t *)S.Q, S.Qf, (const bf16_t *)S.Kt, S.Ktf,
                           (const bf16_t *)S.Vt, (const bf16_t *)K, S.Klo, (const bf16_t *)V, S.pm, S.pl, S.po, a_b, BH, D.H, N,
                           D.p_min, D.log2_pmin, S.levels, S.slots, D.scale, D.alibi, t0);
        block_gemms(D, W, x, y, a_b, h_f, h_b, u_b, S.rinv, t0, nr, st);
        // persistent pairs of the block from its outputs (rows t0.. of the pre-pass buffers are free again)
        // the tiles of Algorithm 1 are the only readers of the transposed values: with p_min a multiple of 32 it is written
        // in runs of p_min positions right before the tile that closes them
        const bool lazy_vt = D.p_min % 32 == 0;
        if (B * nr <= kSmallM && d % 128 == 0) {
            e = small_prepass(D, Wp, S, y, t0, nr, st, K, V, !lazy_vt);   // pairs only, written into the cache by the product's epilogue
            if (e != hipSuccess) return e;
            if (lazy_vt && (t0 + nr) % D.p_min == 0)
                hipLaunchKernelGGL(vt_from_rows_kernel, dim3(BH, (unsigned)(D.p_min / 32)), dim3(256), 0, st, (const bf16_t *)V, S.VT,
                                   S.vt_stride, BH, t0 + nr - D.p_min);
        } else {
            e = Launch<bf16_t>::prepass(D, Wp, S, y, B, nr, true, st, (size_t)N * d, t0);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(par_export_kernel, dim3(BH, nr), dim3(64), 0, st, (const bf16_t *)S.Kt, S.Ktf, (const bf16_t *)S.Vt,
                               (bf16_t *)K, (bf16_t *)V, S.Klo, S.Kh, S.VT, S.vt_stride, BH, t0);
        }
        const int t1 = t0 + nr;
        const int P = t1 & -t1;
        if (P >= D.p_min && t1 < N) {
            const int nq = (P < N - t1) ? P : N - t1;
            e = cross_mfma_launch(D, S, K, t1, P, nq, true, st);
            if (e != hipSuccess) return e;
        }
    }
    return hipGetLastError();
}

}  // namespace rt
