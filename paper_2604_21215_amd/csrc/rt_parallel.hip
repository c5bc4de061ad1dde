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
//   every cross-block UpdateTile of Algorithm 1 (all independent now), then one merge launch over all positions
//   (stored partial states + direct window + temporary pair)
//   h = x + alpha Wo a;  u = gelu(W1 RMS(h));  y = h + alpha W2 u   as three GEMMs with fused epilogues.
#include "rt_base_case.h"
#include "rt_mfma_device.h"

namespace rt {

hipError_t cross_mfma_launch(const LayerDims &D, const Scratch &S, const void *K, int t1, int P, int nq, bool hp,
                             hipStream_t st);

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

// K, V of positions t0 .. t0 + gridDim.y - 1 from the pre-pass outputs (rows (t, b, h)): the caller's cache rows, the bf16 remainder
// of the keys and the transposed values for the tiles.  grid (B*H, N), block 64.
__global__ __launch_bounds__(64) void par_export_kernel(const bf16_t *__restrict__ Ks, const float *__restrict__ Kf,
                                                        const bf16_t *__restrict__ Vs, bf16_t *__restrict__ K,
                                                        bf16_t *__restrict__ V, bf16_t *__restrict__ Klo,
                                                        bf16_t *__restrict__ VT, int vt_stride, int BH, int t0)
{
    const int lane = threadIdx.x, bh = blockIdx.x, t = t0 + blockIdx.y;
    const size_t off = ((size_t)t * BH + bh) * kHeadDim + lane;
    const bf16_t k = Ks[off], v = Vs[off];
    K[off] = k;
    V[off] = v;
    Klo[off] = f32_to_bf16(Kf[off] - bf16_to_f32(k));
    VT[((size_t)bh * kHeadDim + lane) * vt_stride + t] = v;
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

// h = x + alpha Wo a;  u = gelu(W1 RMS(h));  y = h + alpha W2 u  for positions n0 .. n0 + Nc - 1 of every batch row
static void block_gemms(const LayerDims &D, const Weights &W, const void *x, void *y, bf16_t *a_b, float *h_f, bf16_t *h_b,
                        bf16_t *u_b, int n0, int Nc, hipStream_t st)
{
    const int d = D.d, F = D.F, M = D.B * Nc;
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
    hipLaunchKernelGGL(par_export_kernel, dim3(BH, N), dim3(64), 0, st, (const bf16_t *)S.Kt, S.Ktf, (const bf16_t *)S.Vt,
                       (bf16_t *)K, (bf16_t *)V, S.Klo, S.VT, S.vt_stride, BH, 0);
    if (!pairs_are_temporary) {
        e = Launch<bf16_t>::prepass(D, W, S, x, B, N, true, st);
        if (e != hipSuccess) return e;
    }
    // Algorithm 1's events; none depends on another here
    for (int t1 = 1; t1 < N; ++t1) {
        const int P = t1 & -t1;
        if (P < D.p_min) continue;
        const int nq = (P < N - t1) ? P : N - t1;
        e = cross_mfma_launch(D, S, K, t1, P, nq, true, st);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(par_merge_kernel, dim3(BH, N), dim3(64), 0, st, (const bf16_t *)S.Q, S.Qf, (const bf16_t *)S.Kt, S.Ktf,
                       (const bf16_t *)S.Vt, (const bf16_t *)K, S.Klo, (const bf16_t *)V, S.pm, S.pl, S.po, a_b, BH, D.H, N, D.p_min,
                       D.log2_pmin, S.levels, S.slots, D.scale, D.alibi, 0);
    block_gemms(D, W, x, y, a_b, h_f, h_b, u_b, 0, N, st);
    return hipGetLastError();
}

// Blocked recurrence (Sec. 8, Discussion; the reading is stated at rt_layer_prefill_blocked in rt.h): blocks of Sblk
// positions, a power of two that divides p_min, so that every event of Algorithm 1 falls on a block boundary.  While
// a block is evaluated its rows of K, V hold the TEMPORARY pairs (the direct window of merge_body then reads
// persistent pairs of earlier blocks and temporary pairs of the own block without knowing the difference); after the
// block's outputs are there they are overwritten with the persistent pairs projected from those outputs.
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
    for (int t0 = 0; t0 < N; t0 += Sblk) {
        const int nr = Sblk < N - t0 ? Sblk : N - t0;
        hipLaunchKernelGGL(par_export_kernel, dim3(BH, nr), dim3(64), 0, st, (const bf16_t *)S.Kt, S.Ktf, (const bf16_t *)S.Vt,
                           (bf16_t *)K, (bf16_t *)V, S.Klo, S.VT, S.vt_stride, BH, t0);
        hipLaunchKernelGGL(par_merge_kernel, dim3(BH, nr), dim3(64), 0, st, (const bf16_t *)S.Q, S.Qf, (const bf16_t *)S.Kt, S.Ktf,
                           (const bf16_t *)S.Vt, (const bf16_t *)K, S.Klo, (const bf16_t *)V, S.pm, S.pl, S.po, a_b, BH, D.H, N,
                           D.p_min, D.log2_pmin, S.levels, S.slots, D.scale, D.alibi, t0);
        block_gemms(D, W, x, y, a_b, h_f, h_b, u_b, t0, nr, st);
        // persistent pairs of the block from its outputs (rows t0.. of the pre-pass buffers are free again)
        e = Launch<bf16_t>::prepass(D, Wp, S, y, B, nr, true, st, (size_t)N * d, t0);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(par_export_kernel, dim3(BH, nr), dim3(64), 0, st, (const bf16_t *)S.Kt, S.Ktf, (const bf16_t *)S.Vt,
                           (bf16_t *)K, (bf16_t *)V, S.Klo, S.VT, S.vt_stride, BH, t0);
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
