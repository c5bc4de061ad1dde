// Plain-ALU kernels of the RT layer: one launch per phase of a position.
//
// These cover every storage dtype (fp32 and bf16, fp32 arithmetic throughout) and any sequence
// length.  They are the per-position engine ("stepwise"), the decode step, and the fp32 path of the
// cross-block update.  The MFMA kernels live in rt_mfma.hip, the single-launch engine in
// rt_persistent.hip.
#include "rt_base_case.h"
#include "rt_ll.h"

namespace rt {

// =============================================================================================
// Cross-block update, plain-ALU form: queries [t1, t1+nq) against keys [t1-P, t1) of every (b, h);
// the partial state (m, l, o) is written once into the slot of (level log2 P, query).
// grid (nq, B*H), block 64.
// =============================================================================================
template <typename T>
__global__ __launch_bounds__(64) void cross_generic_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                           const T *__restrict__ V, float *__restrict__ pm,
                                                           float *__restrict__ pl, float *__restrict__ po, int BH, int t1,
                                                           int P, int level, int level_rel, int slots, float scale,
                                                           float alibi, int H)
{
    const int lane = threadIdx.x;
    const int i0 = t1 + blockIdx.x;
    const int bh = blockIdx.y;
    const size_t rs = (size_t)BH * kHeadDim;
    const float q = to_f32(Q[(size_t)i0 * rs + (size_t)bh * kHeadDim + lane]);
    float m = -INFINITY, l = 0.f, o = 0.f;
    attend_keys<T>(q, K + (size_t)(t1 - P) * rs + (size_t)bh * kHeadDim, V + (size_t)(t1 - P) * rs + (size_t)bh * kHeadDim,
                   rs, P, scale, m, l, o, nullptr, alibi_slope(alibi, bh % H, H), i0 - (t1 - P));
    const size_t idx = partial_index(level_rel, partial_slot(level, i0), slots, BH, bh);
    if (lane == 0) { pm[idx] = m; pl[idx] = l; }
    po[idx * kHeadDim + lane] = o;
}

// Decode: keys [split*chunk, min(t, (split+1)*chunk)) of the cache against the single query row 0.
// grid (nsplit, B*H), block 64; the partial goes to slot `split` of relative level 0.
template <typename T>
__global__ __launch_bounds__(64) void decode_split_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                          const T *__restrict__ V, float *__restrict__ pm,
                                                          float *__restrict__ pl, float *__restrict__ po, int BH, int t,
                                                          int chunk, int slots, float scale, float alibi, int H)
{
    const int lane = threadIdx.x;
    const int split = blockIdx.x, bh = blockIdx.y;
    const size_t rs = (size_t)BH * kHeadDim;
    const int k_lo = split * chunk, k_hi = min(t, k_lo + chunk);
    const float q = to_f32(Q[(size_t)bh * kHeadDim + lane]);
    float m = -INFINITY, l = 0.f, o = 0.f;
    attend_keys<T>(q, K + (size_t)k_lo * rs + (size_t)bh * kHeadDim, V + (size_t)k_lo * rs + (size_t)bh * kHeadDim, rs,
                   k_hi - k_lo, scale, m, l, o, nullptr, alibi_slope(alibi, bh % H, H), t - k_lo);
    const size_t idx = partial_index(0, split, slots, BH, bh);
    if (lane == 0) { pm[idx] = m; pl[idx] = l; }
    po[idx * kHeadDim + lane] = o;
}

// The same for bf16 caches and splits of 64 keys with every load of the split issued at once (the generic kernel
// walks the value rows eight at a time behind the softmax: nine dependent round trips; here the split's 8 KB of keys and
// 8 KB of values are requested before anything is computed).  Keys and values alike: piece i of a lane is row
// 8 i + lane / 8, columns 8 (lane % 8) .. + 7 (eight lanes cover one 128-byte row); the logits are summed over the
// eight lanes of a row and stay there (the value rows have the same layout), and the eight lanes that share columns
// are summed at the end.  Rows past the split's end are read from its last row with weight zero.
// One split per wavefront: grid (ceil(nsplit / 4), B*H), block 256.
__global__ __launch_bounds__(256) void decode_split64_bf16_kernel(const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K,
                                                                 const bf16_t *__restrict__ V, float *__restrict__ pm,
                                                                 float *__restrict__ pl, float *__restrict__ po, int BH, int t,
                                                                 int slots, float scale, float alibi, int H)
{
    const int lane = threadIdx.x & 63;
    const int split = blockIdx.x * 4 + (threadIdx.x >> 6), bh = blockIdx.y;   // one split per wavefront
    const size_t rs = (size_t)BH * kHeadDim;
    const int k_lo = split * 64, cnt = min(t - k_lo, 64);
    if (cnt <= 0) return;   // no barriers in this kernel
    uint4 kr[8], vr[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const size_t off = (size_t)(k_lo + min(8 * i + (lane >> 3), cnt - 1)) * rs + (size_t)bh * kHeadDim + (lane & 7) * 8;
        kr[i] = *reinterpret_cast<const uint4 *>(K + off);
        vr[i] = *reinterpret_cast<const uint4 *>(V + off);
    }
    const float qv = bf16_to_f32(Q[(size_t)bh * kHeadDim + lane]);
    float q8[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) q8[e] = __shfl(qv, (lane & 7) * 8 + e, 64);
    // the dot product of row 8 i + lane / 8 over this lane's eight columns, summed over the eight lanes of the row inside
    // the lanes' row of sixteen (no LDS crossbar): every lane of a row holds its logit, and its weight is computed there
    const float slope = alibi_slope(alibi, bh % H, H);
    const int r8 = lane >> 3;
    float sc[8];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t w[4] = {kr[i].x, kr[i].y, kr[i].z, kr[i].w};
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            d = fmaf(q8[2 * e], __uint_as_float(w[e] << 16), d);
            d = fmaf(q8[2 * e + 1], __uint_as_float(w[e] & 0xFFFF0000u), d);
        }
        d += dpp_f(d, 0);
        d += dpp_f(d, 1);
        d += dpp_f(d, 2);
        const int j = 8 * i + r8;
        sc[i] = j < cnt ? fmaf(-slope, (float)(t - k_lo - j), d * scale) : -INFINITY;
        mx = fmaxf(mx, sc[i]);
    }
    const float m = fast_max(mx);
    float psum = 0.f;
    float o8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float pr = __expf(sc[i] - m);   // exp(-inf) = 0 for rows past the end
        psum += pr;
        const uint32_t w[4] = {vr[i].x, vr[i].y, vr[i].z, vr[i].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            o8[2 * e] = fmaf(pr, __uint_as_float(w[e] << 16), o8[2 * e]);
            o8[2 * e + 1] = fmaf(pr, __uint_as_float(w[e] & 0xFFFF0000u), o8[2 * e + 1]);
        }
    }
    const float l = fast_sum(psum) * 0.125f;   // every weight was counted by the eight lanes of its row
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        o8[e] += __shfl_xor(o8[e], 8, 64);
        o8[e] += __shfl_xor(o8[e], 16, 64);
        o8[e] += __shfl_xor(o8[e], 32, 64);
    }
    const size_t idx = partial_index(0, split, slots, BH, bh);
    if (lane == 0) { pm[idx] = m; pl[idx] = l; }
    if (lane < 8) {
        float *dst = po + idx * kHeadDim + lane * 8;
        *reinterpret_cast<float4 *>(dst) = make_float4(o8[0], o8[1], o8[2], o8[3]);
        *reinterpret_cast<float4 *>(dst + 4) = make_float4(o8[4], o8[5], o8[6], o8[7]);
    }
}

// =============================================================================================
// Base case, part 1: finish the attention output of position t (merge_body).  grid B*H, block 64.
// =============================================================================================
template <typename T>
__global__ __launch_bounds__(64) void merge_kernel(const T *__restrict__ Q, const T *__restrict__ Kt,
                                                   const T *__restrict__ Vt, const T *__restrict__ K,
                                                   const T *__restrict__ V, const float *__restrict__ pm,
                                                   const float *__restrict__ pl, const float *__restrict__ po,
                                                   float *__restrict__ attn_cat, int BH, int H, int t, int q_row,
                                                   int p_min, int log2_pmin, int levels, int slots, int n_splits,
                                                   float scale, float alibi, bf16_t *__restrict__ op_a)
{
    merge_body<T, false>(Q, nullptr, Kt, nullptr, Vt, K, nullptr, V, pm, pl, po, attn_cat, BH, H, blockIdx.x, t, q_row, p_min,
                         log2_pmin, levels, slots, n_splits, scale, -1, 0, op_a, alibi);
}

// =============================================================================================
// Small-M matrix products of the base case (gemv_body) for one layer: rows o < n_first come from Wa,
// n_first <= o < 2 n_first from Wb, the rest from Wc; one gain vector.
// =============================================================================================
template <typename T> struct ThreeMatrices {
    const T *Wa, *Wb, *Wc, *g;
    int n_first, n_in;
    __device__ __forceinline__ const T *row(int o) const
    {
        const int which = o / n_first;
        return (which == 0 ? Wa : (which == 1 ? Wb : Wc)) + (size_t)(o - which * n_first) * n_in;
    }
    __device__ __forceinline__ const T *gain() const { return g; }
};

template <typename T, typename IN_T, int EPI, int KS>
__global__ __launch_bounds__(256) void gemv_kernel(const T *__restrict__ Wa, const T *__restrict__ Wb,
                                                   const T *__restrict__ Wc, int n_first, int n_out, int n_in,
                                                   const IN_T *__restrict__ in, size_t in_stride, int Bn,
                                                   const T *__restrict__ gain, float eps, int do_norm, float alpha,
                                                   const T *__restrict__ res_T, size_t res_stride,
                                                   const float *__restrict__ res_f, float *__restrict__ out_f,
                                                   T *__restrict__ out_T, size_t out_T_stride)
{
    __shared__ float part[4][kGemvPart];
    const ThreeMatrices<T> rows{Wa, Wb, Wc, gain, n_first, n_in};
    gemv_body<T, IN_T, EPI, KS>(rows, blockIdx.x, n_out, n_in, in, in_stride, Bn, eps, do_norm, alpha, res_T, res_stride, res_f,
                                out_f, out_T, out_T_stride, part);
}

// Decoding step, after the raw [q | k_tmp | v_tmp] product of one position: qkRMS of q and k_tmp per head and the
// rows of Q, Kt, Vt (row index b: one position).  grid B*H, block 64.
template <typename T>
__global__ __launch_bounds__(64) void finalize_qkv_kernel(const float *__restrict__ raw, const T *__restrict__ g_q,
                                                          const T *__restrict__ g_k, T *__restrict__ Q, T *__restrict__ Kt,
                                                          T *__restrict__ Vt, int H, int d, float eps, int norm_free)
{
    const int lane = threadIdx.x, bh = blockIdx.x;
    const int b = bh / H, h = bh % H;
    const float *r = raw + (size_t)b * 3 * d + h * kHeadDim + lane;
    float q = r[0], k = r[d];
    const float v = r[2 * d];
    if (!norm_free) {
        q = q * rsqrtf(wave_sum(q * q) / (float)kHeadDim + eps) * (g_q ? to_f32(g_q[h * kHeadDim + lane]) : 1.f);
        k = k * rsqrtf(wave_sum(k * k) / (float)kHeadDim + eps) * (g_k ? to_f32(g_k[h * kHeadDim + lane]) : 1.f);
    }
    const size_t off = (size_t)b * d + h * kHeadDim + lane;
    Q[off] = from_f32<T>(q);
    Kt[off] = from_f32<T>(k);
    Vt[off] = from_f32<T>(v);
}

// =============================================================================================
// Base case, last part: qkRMS of the new key, store the persistent pair of position t (and the
// transposed bf16 copy of v used by the MFMA cross-block kernel).  grid B*H, block 64.
// =============================================================================================
template <typename T>
__global__ __launch_bounds__(64) void finalize_kv_kernel(const float *__restrict__ kv_raw, const T *__restrict__ g_k,
                                                         T *__restrict__ K, T *__restrict__ V, bf16_t *__restrict__ VT,
                                                         int vt_stride, int BH, int H, int d, int t, float eps,
                                                         int norm_free)
{
    const int lane = threadIdx.x, bh = blockIdx.x;
    const int b = bh / H, h = bh % H;
    float k = kv_raw[(size_t)b * 2 * d + h * kHeadDim + lane];
    const float v = kv_raw[(size_t)b * 2 * d + d + h * kHeadDim + lane];
    if (!norm_free) {
        const float ss = wave_sum(k * k);
        k = k * rsqrtf(ss / (float)kHeadDim + eps) * (g_k ? to_f32(g_k[h * kHeadDim + lane]) : 1.f);
    }
    const size_t off = ((size_t)t * BH + bh) * kHeadDim + lane;
    K[off] = from_f32<T>(k);
    V[off] = from_f32<T>(v);
    if (VT) VT[((size_t)bh * kHeadDim + lane) * vt_stride + t] = f32_to_bf16(v);
}

// =============================================================================================
// Pre-pass, plain-ALU form.  rinv[m] = 1/sqrt(mean(x_m^2)+eps); then for every row m = (b, n):
//   [q | k_tmp | v_tmp] = (x_m * rinv * g_attn) [Wq | Wk | Wv]^T,  qkRMS on q and k_tmp per head.
// Tile 64 rows x 64 columns (one head of one of the three outputs), 256 threads, 4x4 per thread.
// =============================================================================================
template <typename T>
__global__ __launch_bounds__(256) void row_rinv_kernel(const T *__restrict__ x, float *__restrict__ rinv, int M, int Nc,
                                                       size_t x_bstride, int n0, int d, float eps, int norm_free)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = blockIdx.x * 4 + wave;
    if (m >= M) return;
    const T *xr = x + (size_t)(m / Nc) * x_bstride + (size_t)(n0 + m % Nc) * d;
    float ss = 0.f;
    for (int k = lane; k < d; k += 64) { const float v = to_f32(xr[k]); ss = fmaf(v, v, ss); }
    ss = wave_sum(ss);
    if (lane == 0) rinv[m] = norm_free ? 1.f : rsqrtf(ss / (float)d + eps);
}

template <typename T>
__global__ __launch_bounds__(256) void prepass_generic_kernel(const T *__restrict__ x, const float *__restrict__ rinv,
                                                              const T *__restrict__ Wq, const T *__restrict__ Wk,
                                                              const T *__restrict__ Wv, const T *__restrict__ g_attn,
                                                              const T *__restrict__ g_q, const T *__restrict__ g_k,
                                                              T *__restrict__ Q, T *__restrict__ Kt, T *__restrict__ Vt,
                                                              int Bc, int Nc, size_t x_bstride, int n0, int d, int H,
                                                              float eps, int norm_free)
{
    __shared__ float As[16][64 + 1];
    __shared__ float Bs[16][64 + 1];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int M = Bc * Nc;
    const int m0 = blockIdx.x * 64;
    const int which = blockIdx.y / H, h = blockIdx.y % H;  // 0 = q, 1 = k_tmp, 2 = v_tmp
    const T *W = which == 0 ? Wq : (which == 1 ? Wk : Wv);
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    for (int k0 = 0; k0 < d; k0 += 16) {
        __syncthreads();
        for (int idx = tid; idx < 64 * 16; idx += 256) {
            const int r = idx >> 4, kk = idx & 15;
            const int m = min(m0 + r, M - 1);
            const int k = k0 + kk;
            float a = 0.f, bv = 0.f;
            if (k < d) {
                a = to_f32(x[(size_t)(m / Nc) * x_bstride + (size_t)(n0 + m % Nc) * d + k]);
                if (!norm_free) a *= rinv[m] * (g_attn ? to_f32(g_attn[k]) : 1.f);
                bv = to_f32(W[(size_t)(h * kHeadDim + r) * d + k]);
            }
            As[kk][r] = a;
            Bs[kk][r] = bv;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], bb[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; bb[i] = Bs[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], bb[j], acc[i][j]);
        }
    }
    const T *g = which == 0 ? g_q : g_k;
    T *dst = which == 0 ? Q : (which == 1 ? Kt : Vt);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float sc = 1.f;
        if (which < 2 && !norm_free) {
            float ss = acc[i][0] * acc[i][0] + acc[i][1] * acc[i][1] + acc[i][2] * acc[i][2] + acc[i][3] * acc[i][3];
#pragma unroll
            for (int o = 8; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);  // the 16 threads of a row are adjacent lanes
            sc = rsqrtf(ss / (float)kHeadDim + eps);
        }
        const int m = m0 + ty * 4 + i;
        if (m < M) {
            const int b = m / Nc, n = n0 + m % Nc;
            T *o = dst + ((size_t)n * Bc + b) * d + h * kHeadDim + tx * 4;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float v = acc[i][j] * sc;
                if (which < 2 && !norm_free && g) v *= to_f32(g[h * kHeadDim + tx * 4 + j]);
                o[j] = from_f32<T>(v);
            }
        }
    }
}

// =============================================================================================
// Launchers
// =============================================================================================
hipError_t prepass_mfma_launch(const LayerDims &D, const Weights &W, const Scratch &S, const void *x, int Bc, int Nc,
                               size_t x_bstride, int n0, hipStream_t st);
hipError_t cross_mfma_launch(const LayerDims &D, const Scratch &S, const void *K, int t1, int P, int nq, bool hp,
                             hipStream_t st);

template <typename T>
hipError_t Launch<T>::prepass(const LayerDims &D, const Weights &W, const Scratch &S, const void *x, int Bc, int Nc,
                              bool mfma, hipStream_t st, size_t x_bstride, int n0)
{
    const int M = Bc * Nc;
    if (x_bstride == 0) x_bstride = (size_t)Nc * D.d;
    hipLaunchKernelGGL(row_rinv_kernel<T>, dim3((M + 3) / 4), dim3(256), 0, st, (const T *)x, S.rinv, M, Nc, x_bstride, n0,
                       D.d, D.eps, D.norm_free);
    if (mfma && sizeof(T) == 2) return prepass_mfma_launch(D, W, S, x, Bc, Nc, x_bstride, n0, st);
    hipLaunchKernelGGL(prepass_generic_kernel<T>, dim3((M + 63) / 64, 3 * D.H), dim3(256), 0, st, (const T *)x, S.rinv,
                       (const T *)W.Wq, (const T *)W.Wk, (const T *)W.Wv, (const T *)W.g_attn, (const T *)W.g_q,
                       (const T *)W.g_k, (T *)S.Q, (T *)S.Kt, (T *)S.Vt, Bc, Nc, x_bstride, n0, D.d, D.H, D.eps,
                       D.norm_free);
    return hipGetLastError();
}

template <typename T>
hipError_t Launch<T>::merge(const LayerDims &D, const Scratch &S, const void *K, const void *V, int t, int q_row,
                            int n_decode_splits, hipStream_t st, bool split_out)
{
    hipLaunchKernelGGL(merge_kernel<T>, dim3(D.B * D.H), dim3(64), 0, st, (const T *)S.Q, (const T *)S.Kt,
                       (const T *)S.Vt, (const T *)K, (const T *)V, S.pm, S.pl, S.po, S.attn_cat, D.B * D.H, D.H, t, q_row,
                       D.p_min, D.log2_pmin, S.levels, S.slots, n_decode_splits, D.scale, D.alibi,
                       split_out ? S.op_a : (bf16_t *)nullptr);
    return hipGetLastError();
}

// Batch rows beyond one tile of 8 are handled by further launches of the same kernel.
template <typename T, typename IN_T, int EPI>
static hipError_t gemv_launch(const T *Wa, const T *Wb, const T *Wc, int n_first, int n_out, int n_in, const IN_T *in,
                              size_t in_stride, int B, const T *gain, float eps, int do_norm, float alpha, const T *res_T,
                              size_t res_stride, const float *res_f, float *out_f, T *out_T, size_t out_T_stride,
                              hipStream_t st)
{
    for (int b0 = 0; b0 < B; b0 += kBatchTile) {
        const int Bn = (B - b0 < kBatchTile) ? B - b0 : kBatchTile;
        if (n_in <= 1024)
            hipLaunchKernelGGL((gemv_kernel<T, IN_T, EPI, 2>), dim3((n_out + 2 * kGemvRows - 1) / (2 * kGemvRows)), dim3(256), 0, st,
                               Wa, Wb, Wc, n_first, n_out, n_in, in + (size_t)b0 * in_stride, in_stride, Bn, gain, eps, do_norm,
                               alpha, res_T ? res_T + (size_t)b0 * res_stride : res_T, res_stride,
                               res_f ? res_f + (size_t)b0 * n_out : res_f, out_f + (size_t)b0 * n_out,
                               out_T ? out_T + (size_t)b0 * out_T_stride : out_T, out_T_stride);
        else
            hipLaunchKernelGGL((gemv_kernel<T, IN_T, EPI, 4>), dim3((n_out + kGemvRows - 1) / kGemvRows), dim3(256), 0, st, Wa, Wb,
                               Wc, n_first, n_out, n_in, in + (size_t)b0 * in_stride, in_stride, Bn, gain, eps, do_norm, alpha,
                               res_T ? res_T + (size_t)b0 * res_stride : res_T, res_stride,
                               res_f ? res_f + (size_t)b0 * n_out : res_f, out_f + (size_t)b0 * n_out,
                               out_T ? out_T + (size_t)b0 * out_T_stride : out_T, out_T_stride);
    }
    return hipGetLastError();
}

// One position's [q | k_tmp | v_tmp] (a decoding step): the three products as one small-M launch, then the per-head
// normalisation.  x_t rows are B apart by x_stride elements.
template <typename T>
hipError_t Launch<T>::prepass_one(const LayerDims &D, const Weights &W, const Scratch &S, const void *x_t, size_t x_stride,
                                  hipStream_t st, bool matrix_cores)
{
    hipError_t e = matrix_cores ? step_qkv_mm(D, W, S, x_t, x_stride, st) : gemv_launch<T, T, EPI_KV>((const T *)W.Wq, (const T *)W.Wk, (const T *)W.Wv, D.d, 3 * D.d, D.d,
                                             (const T *)x_t, x_stride, D.B, (const T *)W.g_attn, D.eps, D.norm_free ? 0 : 1,
                                             D.alpha, (const T *)nullptr, (size_t)0, (const float *)nullptr, S.qkv_raw,
                                             (T *)nullptr, (size_t)0, st);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(finalize_qkv_kernel<T>, dim3(D.B * D.H), dim3(64), 0, st, S.qkv_raw, (const T *)W.g_q, (const T *)W.g_k,
                       (T *)S.Q, (T *)S.Kt, (T *)S.Vt, D.H, D.d, D.eps, D.norm_free);
    return hipGetLastError();
}

template <typename T>
hipError_t Launch<T>::gemv_wo(const LayerDims &D, const Weights &W, const Scratch &S, const void *x_t, size_t x_stride_b,
                              hipStream_t st)
{
    return gemv_launch<T, float, EPI_WO>((const T *)W.Wo, (const T *)W.Wo, (const T *)W.Wo, D.d, D.d, D.d, S.attn_cat, (size_t)D.d, D.B, (const T *)nullptr,
                                  D.eps, 0, D.alpha, (const T *)x_t, x_stride_b, (const float *)nullptr, S.h, (T *)nullptr,
                                  (size_t)0, st);
}

template <typename T> hipError_t Launch<T>::gemv_w1(const LayerDims &D, const Weights &W, const Scratch &S, hipStream_t st)
{
    return gemv_launch<T, float, EPI_W1>((const T *)W.W1, (const T *)W.W1, (const T *)W.W1, D.F, D.F, D.d, S.h, (size_t)D.d, D.B, (const T *)W.g_mlp, D.eps,
                                  D.norm_free ? 0 : 1, D.alpha, (const T *)nullptr, (size_t)0, (const float *)nullptr, S.u,
                                  (T *)nullptr, (size_t)0, st);
}

template <typename T>
hipError_t Launch<T>::gemv_w2(const LayerDims &D, const Weights &W, const Scratch &S, void *y_t, size_t y_stride_b,
                              hipStream_t st)
{
    return gemv_launch<T, float, EPI_W2>((const T *)W.W2, (const T *)W.W2, (const T *)W.W2, D.d, D.d, D.F, S.u, (size_t)D.F, D.B, (const T *)nullptr, D.eps, 0,
                                  D.alpha, (const T *)nullptr, (size_t)0, S.h, S.z, (T *)y_t, y_stride_b, st);
}

template <typename T> hipError_t Launch<T>::gemv_kv(const LayerDims &D, const Weights &W, const Scratch &S, hipStream_t st)
{
    const T *g = (const T *)(W.g_kv ? W.g_kv : W.g_attn);
    return gemv_launch<T, float, EPI_KV>((const T *)W.Wk, (const T *)W.Wv, (const T *)W.Wv, D.d, 2 * D.d, D.d, S.z, (size_t)D.d, D.B, g, D.eps,
                                  D.norm_free ? 0 : 1, D.alpha, (const T *)nullptr, (size_t)0, (const float *)nullptr,
                                  S.kv_raw, (T *)nullptr, (size_t)0, st);
}

template <typename T>
hipError_t Launch<T>::finalize_kv(const LayerDims &D, const Weights &W, const Scratch &S, void *K, void *V, int t,
                                  bool write_vt, hipStream_t st)
{
    hipLaunchKernelGGL(finalize_kv_kernel<T>, dim3(D.B * D.H), dim3(64), 0, st, S.kv_raw, (const T *)W.g_k, (T *)K, (T *)V,
                       write_vt ? S.VT : (bf16_t *)nullptr, S.vt_stride, D.B * D.H, D.H, D.d, t, D.eps, D.norm_free);
    return hipGetLastError();
}

template <typename T>
hipError_t Launch<T>::cross(const LayerDims &D, const Scratch &S, const void *K, const void *V, int t1, int P, int nq,
                            bool mfma, hipStream_t st)
{
    int level = 0;
    while ((1 << level) < P) ++level;
    if (mfma && sizeof(T) == 2) return cross_mfma_launch(D, S, K, t1, P, nq, false, st);
    hipLaunchKernelGGL(cross_generic_kernel<T>, dim3(nq, D.B * D.H), dim3(64), 0, st, (const T *)S.Q, (const T *)K,
                       (const T *)V, S.pm, S.pl, S.po, D.B * D.H, t1, P, level, level - D.log2_pmin, S.slots, D.scale, D.alibi,
                       D.H);
    return hipGetLastError();
}

template <typename T>
hipError_t Launch<T>::decode_split(const LayerDims &D, const Scratch &S, const void *K, const void *V, int t, int chunk,
                                   int nsplit, hipStream_t st)
{
    if (sizeof(T) == 2 && chunk == 64)
        hipLaunchKernelGGL(decode_split64_bf16_kernel, dim3((nsplit + 3) / 4, D.B * D.H), dim3(256), 0, st, (const bf16_t *)S.Q,
                           (const bf16_t *)K, (const bf16_t *)V, S.pm, S.pl, S.po, D.B * D.H, t, S.slots, D.scale, D.alibi, D.H);
    else
        hipLaunchKernelGGL(decode_split_kernel<T>, dim3(nsplit, D.B * D.H), dim3(64), 0, st, (const T *)S.Q, (const T *)K,
                           (const T *)V, S.pm, S.pl, S.po, D.B * D.H, t, chunk, S.slots, D.scale, D.alibi, D.H);
    return hipGetLastError();
}

// Attention output of EVERY position when all key-value pairs are known (loop-free layers): one wavefront per (b, h, i);
// the state starts from the temporary pair of i and runs over the cache rows j < i.  a_out: fp32 rows [B][N][d].
// grid (B*H, positions), block 64: positions t0 .. t0 + gridDim.y - 1.
template <typename T>
__global__ __launch_bounds__(64) void attend_all_kernel(const T *__restrict__ Q, const T *__restrict__ Kt, const T *__restrict__ Vt,
                                                        const T *__restrict__ K, const T *__restrict__ V, float *__restrict__ a_out,
                                                        int BH, int H, int N, float scale, float alibi, int t0)
{
    const int lane = threadIdx.x, bh = blockIdx.x, i = t0 + blockIdx.y;
    const size_t rs = (size_t)BH * kHeadDim;
    const size_t qo = (size_t)i * rs + (size_t)bh * kHeadDim + lane;
    const float q = to_f32(Q[qo]);
    float m = wave_sum(q * to_f32(Kt[qo])) * scale, l = 1.f, o = to_f32(Vt[qo]);   // distance 0: no positional bias
    if (i > 0)
        attend_keys<T>(q, K + (size_t)bh * kHeadDim, V + (size_t)bh * kHeadDim, rs, i, scale, m, l, o, nullptr,
                       alibi_slope(alibi, bh % H, H), i);
    const int b = bh / H, h = bh % H;
    a_out[((size_t)b * N + i) * ((size_t)H * kHeadDim) + h * kHeadDim + lane] = o / l;
}

template <typename T>
hipError_t Launch<T>::loop_free(const LayerDims &D, const Weights &W, const Scratch &S, const void *x, const void *pairs_src,
                                bool pairs_are_temporary, void *y, void *K, void *V, void *par, hipStream_t st)
{
    const int B = D.B, N = D.N, d = D.d, F = D.F, M = B * N;
    float *a_f = (float *)par, *h_f = a_f + (size_t)M * d, *z_f = h_f + (size_t)M * d, *u_f = z_f + (size_t)M * d;
    Weights Wp = W;
    if (!pairs_are_temporary) Wp.g_attn = W.g_kv;
    hipError_t e = prepass(D, Wp, S, pairs_src, B, N, false, st);
    if (e != hipSuccess) return e;
    // the pre-pass rows (position, b, h) are laid out like the cache rows
    const size_t kv_bytes = (size_t)N * B * d * sizeof(T);
    if ((e = hipMemcpyAsync(K, S.Kt, kv_bytes, hipMemcpyDeviceToDevice, st)) != hipSuccess) return e;
    if ((e = hipMemcpyAsync(V, S.Vt, kv_bytes, hipMemcpyDeviceToDevice, st)) != hipSuccess) return e;
    if (!pairs_are_temporary && (e = prepass(D, W, S, x, B, N, false, st)) != hipSuccess) return e;
    hipLaunchKernelGGL(attend_all_kernel<T>, dim3(B * D.H, N), dim3(64), 0, st, (const T *)S.Q, (const T *)S.Kt, (const T *)S.Vt,
                       (const T *)K, (const T *)V, a_f, B * D.H, D.H, N, D.scale, D.alibi, 0);
    e = gemv_launch<T, float, EPI_WO>((const T *)W.Wo, (const T *)W.Wo, (const T *)W.Wo, d, d, d, a_f, (size_t)d, M, (const T *)nullptr,
                                      D.eps, 0, D.alpha, (const T *)x, (size_t)d, (const float *)nullptr, h_f, (T *)nullptr, (size_t)0, st);
    if (e != hipSuccess) return e;
    e = gemv_launch<T, float, EPI_W1>((const T *)W.W1, (const T *)W.W1, (const T *)W.W1, F, F, d, h_f, (size_t)d, M, (const T *)W.g_mlp,
                                      D.eps, D.norm_free ? 0 : 1, D.alpha, (const T *)nullptr, (size_t)0, (const float *)nullptr, u_f,
                                      (T *)nullptr, (size_t)0, st);
    if (e != hipSuccess) return e;
    return gemv_launch<T, float, EPI_W2>((const T *)W.W2, (const T *)W.W2, (const T *)W.W2, d, d, F, u_f, (size_t)F, M, (const T *)nullptr,
                                         D.eps, 0, D.alpha, (const T *)nullptr, (size_t)0, h_f, z_f, (T *)y, (size_t)d, st);
}

template <typename T>
hipError_t Launch<T>::blocked_generic(const LayerDims &D, const Weights &W, const Scratch &S, const void *x, int Sblk, void *y,
                                      void *K, void *V, void *par, hipStream_t st)
{
    const int B = D.B, N = D.N, d = D.d, F = D.F, M = B * N;
    float *a_f = (float *)par, *h_f = a_f + (size_t)M * d, *z_f = h_f + (size_t)M * d, *u_f = z_f + (size_t)M * d;
    Weights Wp = W;
    Wp.g_attn = W.g_kv;
    hipError_t e = prepass(D, W, S, x, B, N, false, st);   // q and temporary pairs of every position
    if (e != hipSuccess) return e;
    const size_t row_bytes = (size_t)B * d * sizeof(T);    // one position of the pre-pass buffers and of the cache alike
    for (int t0 = 0; t0 < N; t0 += Sblk) {
        const int nr = Sblk < N - t0 ? Sblk : N - t0;
        // while the block is evaluated its cache rows hold its temporary pairs
        if ((e = hipMemcpyAsync((char *)K + t0 * row_bytes, (const char *)S.Kt + t0 * row_bytes, nr * row_bytes,
                                hipMemcpyDeviceToDevice, st)) != hipSuccess) return e;
        if ((e = hipMemcpyAsync((char *)V + t0 * row_bytes, (const char *)S.Vt + t0 * row_bytes, nr * row_bytes,
                                hipMemcpyDeviceToDevice, st)) != hipSuccess) return e;
        hipLaunchKernelGGL(attend_all_kernel<T>, dim3(B * D.H, nr), dim3(64), 0, st, (const T *)S.Q, (const T *)S.Kt, (const T *)S.Vt,
                           (const T *)K, (const T *)V, a_f, B * D.H, D.H, N, D.scale, D.alibi, t0);
        for (int b = 0; b < B; ++b) {   // the block's rows of one batch row are contiguous
            const size_t r0 = (size_t)b * N + t0;
            e = gemv_launch<T, float, EPI_WO>((const T *)W.Wo, (const T *)W.Wo, (const T *)W.Wo, d, d, d, a_f + r0 * d, (size_t)d, nr,
                                              (const T *)nullptr, D.eps, 0, D.alpha, (const T *)x + r0 * d, (size_t)d,
                                              (const float *)nullptr, h_f + r0 * d, (T *)nullptr, (size_t)0, st);
            if (e != hipSuccess) return e;
            e = gemv_launch<T, float, EPI_W1>((const T *)W.W1, (const T *)W.W1, (const T *)W.W1, F, F, d, h_f + r0 * d, (size_t)d, nr,
                                              (const T *)W.g_mlp, D.eps, D.norm_free ? 0 : 1, D.alpha, (const T *)nullptr, (size_t)0,
                                              (const float *)nullptr, u_f + r0 * F, (T *)nullptr, (size_t)0, st);
            if (e != hipSuccess) return e;
            e = gemv_launch<T, float, EPI_W2>((const T *)W.W2, (const T *)W.W2, (const T *)W.W2, d, d, F, u_f + r0 * F, (size_t)F, nr,
                                              (const T *)nullptr, D.eps, 0, D.alpha, (const T *)nullptr, (size_t)0, h_f + r0 * d,
                                              z_f + r0 * d, (T *)y + r0 * d, (size_t)d, st);
            if (e != hipSuccess) return e;
        }
        // persistent pairs of the block from its outputs, over the temporary ones
        if ((e = prepass(D, Wp, S, y, B, nr, false, st, (size_t)N * d, t0)) != hipSuccess) return e;
        if ((e = hipMemcpyAsync((char *)K + t0 * row_bytes, (const char *)S.Kt + t0 * row_bytes, nr * row_bytes,
                                hipMemcpyDeviceToDevice, st)) != hipSuccess) return e;
        if ((e = hipMemcpyAsync((char *)V + t0 * row_bytes, (const char *)S.Vt + t0 * row_bytes, nr * row_bytes,
                                hipMemcpyDeviceToDevice, st)) != hipSuccess) return e;
    }
    return hipSuccess;
}

template struct Launch<float>;
template struct Launch<bf16_t>;

}  // namespace rt
