// Layer-wavefront engine for a stack of RT layers.
//
// Every layer has its own key-value memory and a layer's queries depend only on its own input
// (Sec. 2.2; Sec. 5: the two conditions under which the exact tiled schedule applies hold per layer),
// so different layers can work on different positions at the same time.  The dependent chain shrinks
// from L * N positions to N + (L - 1) * C, and every launch carries the work of all active layers:
// the small-M products of the base case then move L times the weight bytes per launch, which is what
// they need to come near the memory rate.
//
// Schedule.  Layer l runs C positions (one "chunk", a power of two) behind layer l - 1: at step s it
// works on position t = s - l * C.  When it enters a chunk, the layer below has finished that chunk, so
//   * the chunk's queries and temporary pairs come from one GEMM over its C input rows (the pre-pass of
//     Algorithm 1 applied to the rows that are known), and
//   * all keys before the chunk are folded into the chunk's queries by one UpdateTile (Appendix C,
//     Algorithm 2): one "far" partial state per query.
// Inside the chunk the schedule is Algorithm 1 as it stands (blocks P = 2^nu2(t) < C against the next P
// queries, which lie in the same chunk; blocks below p_min attended directly).  Blocks of C keys and more
// cannot be served the way Algorithm 1 does it - their queries are not known yet - and the far tile takes
// their place: exact, with attention traffic N^2 / C instead of N log N, which at C = 128 is still two
// orders of magnitude below the weight traffic of the base case.
//
// One step = six launches over the active layers (grid.y = layer), the per-position engine's phases:
// merge, Wo, W1, W2, [Wk; Wv], finalize; plus, at the steps where a block closes, one launch for the
// cross-block tiles of all layers (all layers are at the same offset inside their chunks).
// Logit inputs are kept unrounded on the bf16 path (fp32 q and k_tmp, keys as bf16 head + bf16
// remainder), as in the single-launch engine.
#include "rt_base_case.h"
#include "rt_cross_tile.h"

namespace rt {

constexpr int kFarLevel = 30;   // partial_slot(kFarLevel, i) == i: the far partial of query i sits in slot i

// position of layer l at a step whose layer-0 position is t0
__device__ __forceinline__ int layer_pos(int t0, int l, int chunk) { return t0 - l * chunk; }

template <typename T, bool HP>
__global__ __launch_bounds__(64) void wf_merge_kernel(const WaveLayer *__restrict__ layers, int l_first, int s, int chunk,
                                                      int log2_chunk, int BH, int H, int p_min, int log2_pmin, float scale)
{
    const int l = l_first + blockIdx.y, t = layer_pos(s, l, chunk);
    const WaveLayer &Y = layers[l];
    const int tree_levels = log2_chunk - log2_pmin;
    merge_body<T, HP>((const T *)Y.S.Q, Y.S.Qf, (const T *)Y.S.Kt, Y.S.Ktf, (const T *)Y.S.Vt, (const T *)Y.K, Y.S.Klo,
                      (const T *)Y.V, Y.S.pm, Y.S.pl, Y.S.po, Y.S.attn_cat, BH, H, blockIdx.x, t, t, p_min, log2_pmin, tree_levels,
                      Y.S.slots, -1, scale, tree_levels, log2_chunk);
}

template <typename T> struct StackedRows {   // rows o < n_first from Wa, the rest from Wb
    const T *Wa, *Wb, *g;
    int n_first, n_in;
    __device__ __forceinline__ const T *row(int o) const
    {
        return o < n_first ? Wa + (size_t)o * n_in : Wb + (size_t)(o - n_first) * n_in;
    }
    __device__ __forceinline__ const T *gain() const { return g; }
};

// grid (row blocks, layers, batch tiles of 8)
template <typename T, int EPI, int KS>
__global__ __launch_bounds__(256) void wf_gemv_kernel(const WaveLayer *__restrict__ layers, int l_first, int s, int chunk, int B,
                                                      int N, int d, int F, float eps, int norm_free, float alpha)
{
    __shared__ float part[4][kGemvPart];
    const int l = l_first + blockIdx.y, t = layer_pos(s, l, chunk);
    const WaveLayer &Y = layers[l];
    const int b0 = blockIdx.z * kBatchTile;
    const int Bn = min(kBatchTile, B - b0);
    const size_t row_t = (size_t)b0 * N * d + (size_t)t * d;   // element offset of row (b0, t) in a [B, N, d] tensor
    if (EPI == EPI_WO) {
        const StackedRows<T> rows{(const T *)Y.W.Wo, (const T *)Y.W.Wo, nullptr, d, d};
        gemv_body<T, float, EPI, KS>(rows, blockIdx.x, d, d, Y.S.attn_cat + (size_t)b0 * d, (size_t)d, Bn, eps, 0, alpha,
                                     (const T *)Y.x + row_t, (size_t)N * d, nullptr, Y.S.h + (size_t)b0 * d, nullptr, 0, part);
    } else if (EPI == EPI_W1) {
        const StackedRows<T> rows{(const T *)Y.W.W1, (const T *)Y.W.W1, (const T *)Y.W.g_mlp, F, d};
        gemv_body<T, float, EPI, KS>(rows, blockIdx.x, F, d, Y.S.h + (size_t)b0 * d, (size_t)d, Bn, eps, norm_free ? 0 : 1, alpha,
                                     nullptr, 0, nullptr, Y.S.u + (size_t)b0 * F, nullptr, 0, part);
    } else if (EPI == EPI_W2) {
        const StackedRows<T> rows{(const T *)Y.W.W2, (const T *)Y.W.W2, nullptr, d, F};
        gemv_body<T, float, EPI, KS>(rows, blockIdx.x, d, F, Y.S.u + (size_t)b0 * F, (size_t)F, Bn, eps, 0, alpha, nullptr, 0,
                                     Y.S.h + (size_t)b0 * d, Y.S.z + (size_t)b0 * d, (T *)Y.y + row_t, (size_t)N * d, part);
    } else {
        const StackedRows<T> rows{(const T *)Y.W.Wk, (const T *)Y.W.Wv, (const T *)Y.W.g_kv, d, d};
        gemv_body<T, float, EPI, KS>(rows, blockIdx.x, 2 * d, d, Y.S.z + (size_t)b0 * d, (size_t)d, Bn, eps, norm_free ? 0 : 1,
                                     alpha, nullptr, 0, nullptr, Y.S.kv_raw + (size_t)b0 * 2 * d, nullptr, 0, part);
    }
}

// grid (B*H, layers), block 64: qkRMS of the new key, persistent pair of (l, t) and its copies for the tiles.
template <typename T, bool HP>
__global__ __launch_bounds__(64) void wf_finalize_kernel(const WaveLayer *__restrict__ layers, int l_first, int s, int chunk,
                                                         int B, int H, int d, float eps, int norm_free)
{
    const int lane = threadIdx.x, bh = blockIdx.x;
    const int l = l_first + blockIdx.y, t = layer_pos(s, l, chunk);
    const WaveLayer &Y = layers[l];
    const int BH = B * H, b = bh / H, h = bh % H;
    const float *r = Y.S.kv_raw + (size_t)b * 2 * d + h * kHeadDim + lane;
    const float k = head_rms<T>(r[0], (const T *)Y.W.g_k, h, eps, norm_free);
    const float v = r[d];
    const size_t off = ((size_t)t * BH + bh) * kHeadDim + lane;
    const T kr = from_f32<T>(k);
    ((T *)Y.K)[off] = kr;
    ((T *)Y.V)[off] = from_f32<T>(v);
    if (HP) Y.S.Klo[off] = f32_to_bf16(k - to_f32(kr));
    if (Y.S.VT) Y.S.VT[((size_t)bh * kHeadDim + lane) * Y.S.vt_stride + t] = f32_to_bf16(v);
}

// ---------------------------------------------------------------------------------------------
// Cross-block tiles of all active layers in one launch.  Layer l's block: keys [t1 - P, t1) against queries
// [t1, t1 + nq) with t1 = t1_0 - l * chunk; far = 1: P = t1 (every key before the chunk), the partial goes to
// slot (far_rel, query); else P is the same for all layers.  Layers with t1 <= 0 or t1 >= N have nothing to do.
// ---------------------------------------------------------------------------------------------
struct CrossJob { int t1, P, nq, level, level_rel; bool any; };
__device__ __forceinline__ CrossJob cross_job(int t1_0, int l, int chunk, int N, int far, int P_tree, int far_rel,
                                              int log2_pmin)
{
    CrossJob j;
    j.t1 = t1_0 - l * chunk;
    j.any = j.t1 > 0 && j.t1 < N;
    if (far) {
        j.P = j.t1; j.nq = min(chunk, N - j.t1); j.level = kFarLevel; j.level_rel = far_rel;
    } else {
        j.P = P_tree; j.nq = min(P_tree, N - j.t1);
        j.level = 31 - __builtin_clz((unsigned)P_tree); j.level_rel = j.level - log2_pmin;
    }
    return j;
}

// blocks of 64 keys and more, LDS-staged; grid (8 * ceil(BH/8) * nqb, layers), block 256
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void wf_cross_tile_kernel(
    const WaveLayer *__restrict__ layers, int l_first, int t1_0, int chunk, int N, int far, int P_tree, int far_rel,
    int log2_pmin, int BH, int nqb, float scale)
{
    __shared__ __align__(16) unsigned char lds[2 * cross_tile_lds_bytes<true>()];
    const int l = l_first + blockIdx.y;
    const CrossJob J = cross_job(t1_0, l, chunk, N, far, P_tree, far_rel, log2_pmin);
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int bh = (j / nqb) * 8 + xcd, qb = j % nqb;
    if (!J.any || bh >= BH || qb * 128 >= J.nq) return;   // the whole workgroup leaves together
    const WaveLayer &Y = layers[l];
    cross_tile_wg<true, 4, 2>(nullptr, Y.S.Qf, (const bf16_t *)Y.K, Y.S.Klo, Y.S.VT, Y.S.vt_stride, Y.S.pm, Y.S.pl, Y.S.po, BH, bh,
                              J.t1, 0, J.t1 - J.P, J.P, qb * 128 + (int)(threadIdx.x >> 6) * 32, J.nq, J.level, J.level_rel,
                              Y.S.slots, scale, lds, (int)threadIdx.x);
}

// blocks of 32 keys (any multiple of 32); grid (ceil(nq/128), B*H, layers), block 256, no barriers
__global__ __launch_bounds__(256) void wf_cross_wave_kernel(const WaveLayer *__restrict__ layers, int l_first, int t1_0, int chunk,
                                                            int N, int far, int P_tree, int far_rel, int log2_pmin, int BH,
                                                            float scale)
{
    const int l = l_first + blockIdx.z;
    const CrossJob J = cross_job(t1_0, l, chunk, N, far, P_tree, far_rel, log2_pmin);
    const int q0 = blockIdx.x * 128 + (int)(threadIdx.x >> 6) * 32;
    if (!J.any || q0 >= J.nq) return;
    const WaveLayer &Y = layers[l];
    cross_mfma_wave<true>(nullptr, Y.S.Qf, (const bf16_t *)Y.K, Y.S.Klo, Y.S.VT, Y.S.vt_stride, Y.S.pm, Y.S.pl, Y.S.po, BH,
                          blockIdx.y, J.t1, 0, J.t1 - J.P, J.P, q0, J.nq, J.level, J.level_rel, Y.S.slots, scale);
}

// plain-ALU form (fp32 storage, or bf16 without the MFMA kernels); grid (max nq, B*H, layers), block 64
template <typename T>
__global__ __launch_bounds__(64) void wf_cross_generic_kernel(const WaveLayer *__restrict__ layers, int l_first, int t1_0,
                                                              int chunk, int N, int far, int P_tree, int far_rel, int log2_pmin,
                                                              int BH, float scale)
{
    const int lane = threadIdx.x, bh = blockIdx.y;
    const int l = l_first + blockIdx.z;
    const CrossJob J = cross_job(t1_0, l, chunk, N, far, P_tree, far_rel, log2_pmin);
    if (!J.any || (int)blockIdx.x >= J.nq) return;
    const WaveLayer &Y = layers[l];
    const int i0 = J.t1 + blockIdx.x;
    const size_t rs = (size_t)BH * kHeadDim;
    const float q = to_f32(((const T *)Y.S.Q)[(size_t)i0 * rs + (size_t)bh * kHeadDim + lane]);
    float m = -INFINITY, lsum = 0.f, o = 0.f;
    const size_t kb = (size_t)(J.t1 - J.P) * rs + (size_t)bh * kHeadDim;
    attend_keys<T>(q, (const T *)Y.K + kb, (const T *)Y.V + kb, rs, J.P, scale, m, lsum, o);
    const size_t idx = partial_index(J.level_rel, partial_slot(J.level, i0), Y.S.slots, BH, bh);
    if (lane == 0) { Y.S.pm[idx] = m; Y.S.pl[idx] = lsum; }
    Y.S.po[idx * kHeadDim + lane] = o;
}

template <typename T, bool HP>
static hipError_t wf_cross_launch(const LayerDims &D, const WaveLayer *dev_layers, int l0, int nl, int t1_0, int chunk, int far,
                                  int P_tree, int far_rel, hipStream_t st)
{
    const int BH = D.B * D.H;
    const int max_nq = far ? chunk : P_tree;
    if (HP) {
        // far tiles cover a multiple of the chunk (>= 64 keys); tree blocks of 64 keys and more use the same kernel
        if (far || P_tree >= kKC) {
            const int nqb = (max_nq + 127) / 128, bh8 = (BH + 7) / 8 * 8;
            hipLaunchKernelGGL(wf_cross_tile_kernel, dim3(bh8 * nqb, nl), dim3(256), 0, st, dev_layers, l0, t1_0, chunk, D.N, far,
                               P_tree, far_rel, D.log2_pmin, BH, nqb, D.scale);
        } else {
            hipLaunchKernelGGL(wf_cross_wave_kernel, dim3((max_nq + 127) / 128, BH, nl), dim3(256), 0, st, dev_layers, l0, t1_0,
                               chunk, D.N, far, P_tree, far_rel, D.log2_pmin, BH, D.scale);
        }
    } else {
        hipLaunchKernelGGL(wf_cross_generic_kernel<T>, dim3(max_nq, BH, nl), dim3(64), 0, st, dev_layers, l0, t1_0, chunk, D.N,
                           far, P_tree, far_rel, D.log2_pmin, BH, D.scale);
    }
    return hipGetLastError();
}

template <typename T, bool HP, int KSd, int KSF>
static hipError_t wavefront_steps(const LayerDims &D, const WaveLayer *dev_layers, const WaveLayer *host_layers, int L, int chunk,
                                  bool mfma, hipStream_t st)
{
    const int B = D.B, N = D.N, d = D.d, F = D.F, BH = D.B * D.H;
    int log2_chunk = 0;
    while ((1 << log2_chunk) < chunk) ++log2_chunk;
    const int far_rel = log2_chunk - D.log2_pmin;
    const unsigned bt = (unsigned)((B + kBatchTile - 1) / kBatchTile);
    constexpr int rows_d = (4 / KSd) * kGemvRows, rows_F = (4 / KSF) * kGemvRows;   // output rows per workgroup
    const int n_steps = N + (L - 1) * chunk;
    for (int s = 0; s < n_steps; ++s) {
        // active layers: 0 <= s - l * chunk < N
        const int l1 = s / chunk < L - 1 ? s / chunk : L - 1;
        int l0 = s - (N - 1) > 0 ? (s - (N - 1) + chunk - 1) / chunk : 0;
        if (l0 > l1) continue;   // between the last position of one layer and the first of the next (N not a multiple of the chunk)
        const unsigned nl = (unsigned)(l1 - l0 + 1);
        hipError_t e;
        if (s % chunk == 0) {
            // the active layers enter a chunk: queries and temporary pairs of its rows, then the far tile
            for (int l = l0 > 1 ? l0 : 1; l <= l1; ++l) {
                const int t = s - l * chunk;
                const int Nc = chunk < N - t ? chunk : N - t;
                e = Launch<T>::prepass(D, host_layers[l].W, host_layers[l].S, host_layers[l].x, B, Nc, mfma, st, (size_t)N * d, t);
                if (e != hipSuccess) return e;
            }
            if (s - l0 * chunk > 0) {
                e = wf_cross_launch<T, HP>(D, dev_layers, l0, (int)nl, s, chunk, 1, 0, far_rel, st);
                if (e != hipSuccess) return e;
            }
        }
        hipLaunchKernelGGL((wf_merge_kernel<T, HP>), dim3(BH, nl), dim3(64), 0, st, dev_layers, l0, s, chunk, log2_chunk, BH, D.H,
                           D.p_min, D.log2_pmin, D.scale);
        hipLaunchKernelGGL((wf_gemv_kernel<T, EPI_WO, KSd>), dim3((d + rows_d - 1) / rows_d, nl, bt), dim3(256), 0, st, dev_layers,
                           l0, s, chunk, B, N, d, F, D.eps, D.norm_free, D.alpha);
        hipLaunchKernelGGL((wf_gemv_kernel<T, EPI_W1, KSd>), dim3((F + rows_d - 1) / rows_d, nl, bt), dim3(256), 0, st, dev_layers,
                           l0, s, chunk, B, N, d, F, D.eps, D.norm_free, D.alpha);
        hipLaunchKernelGGL((wf_gemv_kernel<T, EPI_W2, KSF>), dim3((d + rows_F - 1) / rows_F, nl, bt), dim3(256), 0, st, dev_layers,
                           l0, s, chunk, B, N, d, F, D.eps, D.norm_free, D.alpha);
        hipLaunchKernelGGL((wf_gemv_kernel<T, EPI_KV, KSd>), dim3((2 * d + rows_d - 1) / rows_d, nl, bt), dim3(256), 0, st,
                           dev_layers, l0, s, chunk, B, N, d, F, D.eps, D.norm_free, D.alpha);
        hipLaunchKernelGGL((wf_finalize_kernel<T, HP>), dim3(BH, nl), dim3(64), 0, st, dev_layers, l0, s, chunk, B, D.H, d, D.eps,
                           D.norm_free);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        // a block inside the chunk closes: s + 1 positions of layer 0 are finished, every layer is at the same offset
        const int t1 = s + 1;
        const int P = t1 & -t1;
        if (P >= D.p_min && P < chunk) {
            e = wf_cross_launch<T, HP>(D, dev_layers, l0, (int)nl, t1, chunk, 0, P, far_rel, st);
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

template <typename T>
hipError_t wavefront_prefill(const LayerDims &D, const WaveLayer *dev_layers, const WaveLayer *host_layers, int L, int chunk,
                             bool mfma, hipStream_t st)
{
    // layer 0: its input is known in full, all queries and temporary pairs at once
    hipError_t e = Launch<T>::prepass(D, host_layers[0].W, host_layers[0].S, host_layers[0].x, D.B, D.N, mfma, st);
    if (e != hipSuccess) return e;
    const bool hp = mfma && sizeof(T) == 2;
    const bool ks2_d = D.d <= 1024, ks2_F = D.F <= 1024;   // one 512-column slice per wavefront up to 1024 columns
#define RT_WF_GO(HPv, KD, KF) return wavefront_steps<T, HPv, KD, KF>(D, dev_layers, host_layers, L, chunk, mfma, st)
    if (hp) {
        if (ks2_d && ks2_F) RT_WF_GO(true, 2, 2);
        if (ks2_d) RT_WF_GO(true, 2, 4);
        RT_WF_GO(true, 4, 4);
    }
    if (ks2_d && ks2_F) RT_WF_GO(false, 2, 2);
    if (ks2_d) RT_WF_GO(false, 2, 4);
    RT_WF_GO(false, 4, 4);
#undef RT_WF_GO
}

template hipError_t wavefront_prefill<float>(const LayerDims &, const WaveLayer *, const WaveLayer *, int, int, bool, hipStream_t);
template hipError_t wavefront_prefill<bf16_t>(const LayerDims &, const WaveLayer *, const WaveLayer *, int, int, bool, hipStream_t);

}  // namespace rt
