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
#include "rt_prepass_device.h"

namespace rt {

constexpr int kFarLevel = 30;   // partial_slot(kFarLevel, i) == i: the far partial of query i sits in slot i

// position of layer l at a step whose layer-0 position is t0
__device__ __forceinline__ int layer_pos(int t0, int l, int chunk) { return t0 - l * chunk; }

template <typename T, bool HP>
__global__ __launch_bounds__(64) void wf_merge_kernel(const WaveLayer *__restrict__ layers, int l_first, int s, int chunk,
                                                      int log2_chunk, int BH, int H, int p_min, int log2_pmin, float scale,
                                                      float alibi)
{
    const int l = l_first + blockIdx.y, t = layer_pos(s, l, chunk);
    const WaveLayer &Y = layers[l];
    const int tree_levels = log2_chunk - log2_pmin;
    if (HP && p_min == 32 && tree_levels <= kFastLevels) {
        const int bh = blockIdx.x, lane = threadIdx.x;
        const float a = merge_window32_hp(Y.S.Qf, Y.S.Ktf, (const bf16_t *)Y.S.Vt, (const bf16_t *)Y.K, Y.S.Klo, Y.S.VT, Y.S.vt_stride,
                                          Y.S.pm, Y.S.pl, Y.S.po, BH, H, bh, t, tree_levels, Y.S.slots, scale, tree_levels, log2_chunk,
                                          alibi);
        const int b = bh / H, h = bh % H;
        const size_t d = (size_t)H * kHeadDim;
        Y.S.attn_cat[(size_t)b * d + h * kHeadDim + lane] = a;
        const bf16_t hi = f32_to_bf16(a);
        Y.S.op_a[(size_t)(2 * b) * d + h * kHeadDim + lane] = hi;
        Y.S.op_a[(size_t)(2 * b + 1) * d + h * kHeadDim + lane] = f32_to_bf16(a - bf16_to_f32(hi));
        return;
    }
    merge_body<T, HP>((const T *)Y.S.Q, Y.S.Qf, (const T *)Y.S.Kt, Y.S.Ktf, (const T *)Y.S.Vt, (const T *)Y.K, Y.S.Klo,
                      (const T *)Y.V, Y.S.pm, Y.S.pl, Y.S.po, Y.S.attn_cat, BH, H, blockIdx.x, t, t, p_min, log2_pmin, tree_levels,
                      Y.S.slots, -1, scale, tree_levels, log2_chunk, HP ? Y.S.op_a : nullptr, alibi);
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

// ---------------------------------------------------------------------------------------------
// The same four products on the matrix cores (bf16 storage).  With at most 16 batch rows the products are
// bound by the weight bytes, and the plain-ALU form spends more instructions on the cross-lane sums than
// on the multiply-adds; v_mfma_f32_16x16x32_bf16 does that reduction for free:
//     D[16 weight rows][16 batch columns] += W[16 rows][32 k] * X^T[32 k][16 columns]
// A fragments come straight from the row-major weights (lane: row lane%16, 16 bytes), and so that a lane's
// two consecutive loads cover 32 contiguous bytes (the four lanes of a row one 128-byte line per pair of
// steps) the contraction index of step pair p is assigned as k = 64 p + 16 g + (0..7 | 8..15), g = lane/16.
// The input vector is not rounded: it comes as a bf16 head row plus a bf16 remainder row (written by the
// producing kernel's epilogue with the consumer's RMS gain applied) and each weight fragment feeds two
// instructions.  The RMS scale is applied to the finished sums (the product is linear in its input); its
// sum of squares comes as one partial per 16 elements from the producer and is added in a fixed order.
// KS wavefronts of a workgroup share 16 rows and split the contraction; their partial tiles meet in LDS.
// grid (n_out / (16 * 4 / KS), layers, batch tiles of 16), block 256.
// ---------------------------------------------------------------------------------------------
constexpr int kMmBatch = 16;

__device__ __forceinline__ void split_store4(bf16_t *__restrict__ op, size_t hi_off, size_t lo_off, const float *v)
{
    uint32_t h01 = pack_bf16(v[0], v[1]), h23 = pack_bf16(v[2], v[3]);
    const float r0 = v[0] - __uint_as_float(h01 << 16), r1 = v[1] - __uint_as_float(h01 & 0xFFFF0000u);
    const float r2 = v[2] - __uint_as_float(h23 << 16), r3 = v[3] - __uint_as_float(h23 & 0xFFFF0000u);
    *reinterpret_cast<uint2 *>(op + hi_off) = make_uint2(h01, h23);
    *reinterpret_cast<uint2 *>(op + lo_off) = make_uint2(pack_bf16(r0, r1), pack_bf16(r2, r3));
}

// 1 / rms of batch row `col` from the producer's partial sums of squares (ng of them); all four lanes that share
// a column end up with the same value.
__device__ __forceinline__ float rms_scale_from_parts(const float *__restrict__ ssq, int col, int g, int ng, int K, float eps)
{
    float tot = 0.f;
    const int per = (ng + 3) / 4;
    for (int j = g * per; j < min(ng, (g + 1) * per); ++j) tot += ssq[(size_t)col * ng + j];
    tot += __shfl_xor(tot, 16, 64);
    tot += __shfl_xor(tot, 32, 64);
    return rsqrtf(tot / (float)K + eps);
}

// NW wavefronts per workgroup, KS of them share 16 rows: 16 * NW / KS rows per workgroup.  XL: the operand rows of
// the batch tile are staged in LDS once per workgroup (row stride K + 8 elements: the rows of a 16-lane group
// then sit in different banks) instead of being fetched through the vector cache by every wavefront.
// Weight fragments are fetched one block of 256 contraction indices ahead of the instructions that use them.
// EPI_KV needs NW / KS = 4: a workgroup is then one head of k or of v, and the epilogue finishes the position
// (qkRMS of the key, persistent pair of (l, t) in place, remainder keys and transposed values for the tiles).
// Dynamic LDS: NW KB of partial tiles, 256 B of per-head sums, then the operand rows.
// PACKED: the weights come in fragment order (Scratch::wp_*); else row-major as the caller holds them (a lane's two
// fragments of a step pair are then 64 bytes apart in its row: half a cache line per row and instruction).
// EPI_QKV: the raw [q | k_tmp | v_tmp] of one position from [Wq; Wk; Wv] and the operand rows op_x (a decoding step).
// Y: the layer; t: its position (row t of x / y / K / V / V^T); block_x: row block; batch_tile: which 16 batch rows.
constexpr int EPI_QKV = 4;
template <int EPI, int KS, int NW, bool XL, bool PACKED>
__device__ __forceinline__ void mm_body(const WaveLayer &Y, int t, int block_x, int batch_tile, int B, int N, int d, int F, int H,
                                        float eps, int norm_free, float alpha, unsigned char *wf_mm_smem)
{
    float(*part)[16 * 16] = reinterpret_cast<float(*)[16 * 16]>(wf_mm_smem);
    float *hss = reinterpret_cast<float *>(wf_mm_smem + NW * 1024);
    bf16_t *xs = reinterpret_cast<bf16_t *>(wf_mm_smem + NW * 1024 + 256);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, g = lane >> 4;
    constexpr int RG = NW / KS;
    const int rg = wave / KS, kw = wave % KS;
    const int row0 = (block_x * RG + rg) * 16;
    const int b0 = batch_tile * kMmBatch;
    const int Bn = min(kMmBatch, B - b0);
    const int K = EPI == EPI_W2 ? F : d;
    const bf16_t *Wp;       // the matrix in fragment order (Scratch::wp_*), PACKED only
    const bf16_t *Wr;       // this wavefront's first row in the caller's row-major matrix, !PACKED only
    const bf16_t *X;        // operand rows [2B][K]
    if (EPI == EPI_WO) { Wp = Y.S.wp_o; Wr = (const bf16_t *)Y.W.Wo + (size_t)row0 * K; X = Y.S.op_a; }
    else if (EPI == EPI_W1) { Wp = Y.S.wp_1; Wr = (const bf16_t *)Y.W.W1 + (size_t)row0 * K; X = Y.S.op_h; }
    else if (EPI == EPI_W2) { Wp = Y.S.wp_2; Wr = (const bf16_t *)Y.W.W2 + (size_t)row0 * K; X = Y.S.op_u; }
    else if (EPI == EPI_KV) {
        Wp = Y.S.wp_kv; X = Y.S.op_z;
        Wr = row0 < d ? (const bf16_t *)Y.W.Wk + (size_t)row0 * K : (const bf16_t *)Y.W.Wv + (size_t)(row0 - d) * K;
    } else {
        Wp = nullptr; X = Y.S.op_x;
        Wr = (const bf16_t *)(row0 < d ? Y.W.Wq : (row0 < 2 * d ? Y.W.Wk : Y.W.Wv)) + (size_t)(row0 % d) * K;
    }
    const int klen = K / KS, kbeg = kw * klen;
    // step pair p (contraction indices 64p .. 64p+63) of this wavefront's 16 rows: two fragments, the first covering
    // k = 64p + 8g + (0..7), the second 32 further; PACKED: fragments 2p and 2p + 1 of the row group, 1 KB each
    const bf16_t *wr = PACKED ? Wp + ((size_t)(row0 / 16) * (K / 64) + kbeg / 64) * 1024 + lane * 8
                              : Wr + (size_t)col * K + kbeg + 8 * g;
    constexpr int kPairStride = PACKED ? 1024 : 64, kFragStride = PACKED ? 512 : 32;
    const int cb = min(col, Bn - 1);   // columns beyond Bn repeat the last batch row (their results are dropped)
    const int xld = XL ? K + 8 : K;
    const bf16_t *xh = (XL ? xs + (size_t)(2 * cb) * xld : X + (size_t)(2 * (b0 + cb)) * K) + kbeg + 8 * g;
    const bf16_t *xl = xh + xld;

    uint4 wa[8], wb[8];
#define RT_WF_LOADW(buf, kk)                                                                   \
    _Pragma("unroll") for (int j = 0; j < 4; ++j)                                              \
    {                                                                                          \
        buf[2 * j] = global_load16(wr + ((kk) / 64 + j) * kPairStride);                \
        buf[2 * j + 1] = global_load16(wr + ((kk) / 64 + j) * kPairStride + kFragStride); \
    }
#define RT_WF_PAIR(a0v, a1v, kk)                                                               \
    {                                                                                          \
        Frag a0, a1, h0, h1, l0, l1;                                                           \
        a0.u = a0v; a1.u = a1v;                                                                \
        h0.u = *reinterpret_cast<const uint4 *>(xh + (kk));                                    \
        h1.u = *reinterpret_cast<const uint4 *>(xh + (kk) + 32);                               \
        l0.u = *reinterpret_cast<const uint4 *>(xl + (kk));                                    \
        l1.u = *reinterpret_cast<const uint4 *>(xl + (kk) + 32);                               \
        acc = mfma16(a0, l0, acc);                                                             \
        acc = mfma16(a1, l1, acc);                                                             \
        acc = mfma16(a0, h0, acc);                                                             \
        acc = mfma16(a1, h1, acc);                                                             \
    }
#define RT_WF_COMPUTE(buf, kk) \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) RT_WF_PAIR(buf[2 * j], buf[2 * j + 1], (kk) + 64 * j)

    const int nfull = klen / 256;
    if (nfull > 0) { RT_WF_LOADW(wa, 0) }
    const bool do_norm = !norm_free && (EPI == EPI_W1 || EPI == EPI_KV || EPI == EPI_QKV);
    float rscale = 1.f;
    if (do_norm && !(XL && EPI == EPI_QKV))
        rscale = rms_scale_from_parts((EPI == EPI_W1 ? Y.S.ssq_h : (EPI == EPI_KV ? Y.S.ssq_z : Y.S.ssq_x)) + (size_t)b0 * (d / 16),
                                      cb, g, d / 16, d, eps);
    if (XL && EPI == EPI_QKV) {
        // a decoding step's input rows x_t [B][d] (Y.x, rows d apart) become the operand rows right here: head + remainder of
        // x * g_attn, and the 1/rms of x from sums that meet in LDS (no separate preparation launch)
        if (tid < 16) hss[tid] = 0.f;
        __syncthreads();
        const bf16_t *xin = (const bf16_t *)Y.x;
        const bf16_t *ga = (const bf16_t *)Y.W.g_attn;
        const int ppr = K / 4;   // 4-element pieces per row
        for (int p = tid; p < Bn * ppr; p += 64 * NW) {
            const int r = p / ppr, e0 = (p - r * ppr) * 4;
            const uint2 xr = *reinterpret_cast<const uint2 *>(xin + (size_t)(b0 + r) * d + e0);
            float v[4] = {__uint_as_float(xr.x << 16), __uint_as_float(xr.x & 0xFFFF0000u), __uint_as_float(xr.y << 16),
                          __uint_as_float(xr.y & 0xFFFF0000u)};
            atomicAdd(&hss[r], (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]));
            if (ga && !norm_free) {
                const uint2 gr = *reinterpret_cast<const uint2 *>(ga + e0);
                v[0] *= __uint_as_float(gr.x << 16); v[1] *= __uint_as_float(gr.x & 0xFFFF0000u);
                v[2] *= __uint_as_float(gr.y << 16); v[3] *= __uint_as_float(gr.y & 0xFFFF0000u);
            }
            split_store4(xs, (size_t)(2 * r) * xld + e0, (size_t)(2 * r + 1) * xld + e0, v);
        }
        __syncthreads();
        if (do_norm) rscale = rsqrtf(hss[cb] / (float)d + eps);
    } else if (XL) {
        const int ppr = K / 8;   // 16-byte pieces per operand row
        for (int p = tid; p < 2 * Bn * ppr; p += 64 * NW) {
            const int r = p / ppr, c = p - r * ppr;
            *reinterpret_cast<uint4 *>(xs + (size_t)r * xld + c * 8) =
                *reinterpret_cast<const uint4 *>(X + (size_t)(2 * b0 + r) * K + c * 8);
        }
        __syncthreads();
    }
    f32x4_t acc = f32x4_t{0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < nfull; i += 2) {
        if (i + 1 < nfull) { RT_WF_LOADW(wb, (i + 1) * 256) }
        RT_WF_COMPUTE(wa, i * 256)
        if (i + 1 < nfull) {
            if (i + 2 < nfull) { RT_WF_LOADW(wa, (i + 2) * 256) }
            RT_WF_COMPUTE(wb, (i + 1) * 256)
        }
    }
    for (int k = nfull * 256; k < klen; k += 64)
        RT_WF_PAIR(global_load16(wr + (k / 64) * kPairStride), global_load16(wr + (k / 64) * kPairStride + kFragStride), k)
#undef RT_WF_LOADW
#undef RT_WF_PAIR
#undef RT_WF_COMPUTE
    if (KS > 1) {
#pragma unroll
        for (int r = 0; r < 4; ++r) part[wave][(4 * g + r) * 16 + col] = acc[r];
        __syncthreads();
        if (kw == 0) {
#pragma unroll
            for (int j = 1; j < KS; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[r] += part[wave + j][(4 * g + r) * 16 + col];
        }
    }
    // wavefronts with kw == 0 hold the tile: lane = outputs (rows row0 + 4g .. + 3, batch row b0 + col)
    const bool live = col < Bn && kw == 0;
    const int b = b0 + cb, o = row0 + 4 * g;
    float v[4] = {acc[0] * rscale, acc[1] * rscale, acc[2] * rscale, acc[3] * rscale};
    if (EPI == EPI_WO || EPI == EPI_W2) {
        if (kw != 0) return;   // no barrier below on this path
        float gn[4] = {1.f, 1.f, 1.f, 1.f}, ss = 0.f;
        const bf16_t *gp = (const bf16_t *)(EPI == EPI_WO ? Y.W.g_mlp : Y.W.g_kv);
        if (gp && !norm_free) {
            const uint2 gg = *reinterpret_cast<const uint2 *>(gp + o);
            gn[0] = __uint_as_float(gg.x << 16); gn[1] = __uint_as_float(gg.x & 0xFFFF0000u);
            gn[2] = __uint_as_float(gg.y << 16); gn[3] = __uint_as_float(gg.y & 0xFFFF0000u);
        }
        float res[4];
        if (EPI == EPI_WO) {
            const uint2 xr = *reinterpret_cast<const uint2 *>((const bf16_t *)Y.x + ((size_t)b * N + t) * d + o);
            res[0] = __uint_as_float(xr.x << 16); res[1] = __uint_as_float(xr.x & 0xFFFF0000u);
            res[2] = __uint_as_float(xr.y << 16); res[3] = __uint_as_float(xr.y & 0xFFFF0000u);
        } else {
            const float4 hr = *reinterpret_cast<const float4 *>(Y.S.h + (size_t)b * d + o);
            res[0] = hr.x; res[1] = hr.y; res[2] = hr.z; res[3] = hr.w;
        }
        float gv[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) { v[r] = res[r] + alpha * v[r]; ss = fmaf(v[r], v[r], ss); gv[r] = v[r] * gn[r]; }
        if (!live) ss = 0.f;
        ss += __shfl_xor(ss, 16, 64);
        ss += __shfl_xor(ss, 32, 64);
        if (live) {
            if (EPI == EPI_WO) {
                *reinterpret_cast<float4 *>(Y.S.h + (size_t)b * d + o) = make_float4(v[0], v[1], v[2], v[3]);
                split_store4(Y.S.op_h, (size_t)(2 * b) * d + o, (size_t)(2 * b + 1) * d + o, gv);
                if (g == 0) Y.S.ssq_h[(size_t)b * (d / 16) + row0 / 16] = ss;
            } else {
                *reinterpret_cast<uint2 *>((bf16_t *)Y.y + ((size_t)b * N + t) * d + o) =
                    make_uint2(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]));
                split_store4(Y.S.op_z, (size_t)(2 * b) * d + o, (size_t)(2 * b + 1) * d + o, gv);
                if (g == 0) Y.S.ssq_z[(size_t)b * (d / 16) + row0 / 16] = ss;
            }
        }
    } else if (EPI == EPI_W1) {
        if (live) {
            float u[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) u[r] = gelu_erf(v[r]);
            split_store4(Y.S.op_u, (size_t)(2 * b) * F + o, (size_t)(2 * b + 1) * F + o, u);
        }
    } else if (EPI == EPI_QKV) {
        if (live) *reinterpret_cast<float4 *>(Y.S.qkv_raw + (size_t)b * 3 * d + o) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
        // the workgroup is head hh of [k heads | v heads]; this wavefront holds head dimensions 16 rg + 4g .. + 3
        const int hh = block_x;
        const bool is_k = hh < H;
        if (is_k && !norm_free) {
            float ss = live ? (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]) : 0.f;
            ss += __shfl_xor(ss, 16, 64);
            ss += __shfl_xor(ss, 32, 64);
            if (kw == 0 && g == 0) hss[rg * 16 + col] = ss;
            __syncthreads();   // is_k is uniform over the workgroup
            const float tot = (hss[col] + hss[16 + col]) + (hss[32 + col] + hss[48 + col]);
            const float sc = rsqrtf(tot / (float)kHeadDim + eps);
            const bf16_t *gk = (const bf16_t *)Y.W.g_k;
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] *= sc * (gk ? bf16_to_f32(gk[hh * kHeadDim + 16 * rg + 4 * g + r]) : 1.f);
        }
        if (live) {
            const int h = is_k ? hh : hh - H, bh = b * H + h, BH = B * H;
            const size_t off = ((size_t)t * BH + bh) * kHeadDim + 16 * rg + 4 * g;
            const uint32_t p01 = pack_bf16(v[0], v[1]), p23 = pack_bf16(v[2], v[3]);
            if (is_k) {
                *reinterpret_cast<uint2 *>((bf16_t *)Y.K + off) = make_uint2(p01, p23);
                const float r0 = v[0] - __uint_as_float(p01 << 16), r1 = v[1] - __uint_as_float(p01 & 0xFFFF0000u);
                const float r2 = v[2] - __uint_as_float(p23 << 16), r3 = v[3] - __uint_as_float(p23 & 0xFFFF0000u);
                if (Y.S.Klo) *reinterpret_cast<uint2 *>(Y.S.Klo + off) = make_uint2(pack_bf16(r0, r1), pack_bf16(r2, r3));
                if (Y.S.Kh) *reinterpret_cast<uint2 *>(Y.S.Kh + off) = make_uint2(pack_f16(v[0], v[1]), pack_f16(v[2], v[3]));
            } else {
                *reinterpret_cast<uint2 *>((bf16_t *)Y.V + off) = make_uint2(p01, p23);
                if (Y.S.VT) {
                    bf16_t *vt = Y.S.VT + ((size_t)bh * kHeadDim + 16 * rg + 4 * g) * Y.S.vt_stride + t;
                    vt[0] = (bf16_t)(p01 & 0xFFFFu);
                    vt[(size_t)Y.S.vt_stride] = (bf16_t)(p01 >> 16);
                    vt[2 * (size_t)Y.S.vt_stride] = (bf16_t)(p23 & 0xFFFFu);
                    vt[3 * (size_t)Y.S.vt_stride] = (bf16_t)(p23 >> 16);
                }
            }
        }
    }
}

// the body over the active layers of a stack (layer-wavefront engine): grid (row blocks, layers, batch tiles of 16)
template <int EPI, int KS, int NW, bool XL>
__global__ __launch_bounds__(64 * NW) void wf_mm_kernel(const WaveLayer *__restrict__ layers, int l_first, int s, int chunk, int B,
                                                        int N, int d, int F, int H, float eps, int norm_free, float alpha)
{
    extern __shared__ __align__(16) unsigned char wf_mm_smem[];
    const int l = l_first + blockIdx.y;
    mm_body<EPI, KS, NW, XL, true>(layers[l], layer_pos(s, l, chunk), (int)blockIdx.x, (int)blockIdx.z, B, N, d, F, H, eps, norm_free,
                                   alpha, wf_mm_smem);
}

// the body for one layer and one position whose rows the descriptor's pointers already address (a decoding step:
// x, y [B][d], K / V / Klo pointing at the cache row to write, V^T at its column), weights as the caller holds them:
// grid (row blocks, 1, batch tiles of 16)
template <int EPI, int KS, int NW, bool XL>
__global__ __launch_bounds__(64 * NW) void step_mm_kernel(const WaveLayer Y, int B, int d, int F, int H, float eps, int norm_free,
                                                          float alpha)
{
    extern __shared__ __align__(16) unsigned char wf_mm_smem[];
    mm_body<EPI, KS, NW, XL, false>(Y, 0, (int)blockIdx.x, (int)blockIdx.z, B, 1, d, F, H, eps, norm_free, alpha, wf_mm_smem);
}

// A decoding step's input rows x_t [B][d] as operand rows: head + remainder of x * g_attn, and the sums of squares of
// x per 16 elements.  grid (ceil(d / 1024), B), block 256: a thread takes 4 elements, 4 adjacent threads one group.
__global__ __launch_bounds__(256) void step_prep_kernel(const bf16_t *__restrict__ x, size_t x_stride, const bf16_t *__restrict__ g,
                                                        bf16_t *__restrict__ op_x, float *__restrict__ ssq_x, int d, int norm_free)
{
    const int b = blockIdx.y, e0 = ((int)blockIdx.x * 256 + (int)threadIdx.x) * 4;
    const bool in = e0 < d;   // d is a multiple of 64: a group of 16 is all in or all out
    float v[4] = {0.f, 0.f, 0.f, 0.f}, gv[4];
    if (in) {
        const uint2 xr = *reinterpret_cast<const uint2 *>(x + (size_t)b * x_stride + e0);
        v[0] = __uint_as_float(xr.x << 16); v[1] = __uint_as_float(xr.x & 0xFFFF0000u);
        v[2] = __uint_as_float(xr.y << 16); v[3] = __uint_as_float(xr.y & 0xFFFF0000u);
    }
    float ss = (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]);
    ss += __shfl_xor(ss, 1, 64);
    ss += __shfl_xor(ss, 2, 64);
#pragma unroll
    for (int r = 0; r < 4; ++r) gv[r] = v[r] * ((g && !norm_free && in) ? bf16_to_f32(g[e0 + r]) : 1.f);
    if (in) {
        split_store4(op_x, (size_t)(2 * b) * d + e0, (size_t)(2 * b + 1) * d + e0, gv);
        if ((threadIdx.x & 3) == 0) ssq_x[(size_t)b * (d / 16) + e0 / 16] = ss;
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
    if (HP) Y.S.Kh[off] = f32_to_f16_bits(k);
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
template <bool ALIBI>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void wf_cross_tile_kernel(
    const WaveLayer *__restrict__ layers, int l_first, int t1_0, int chunk, int N, int far, int P_tree, int far_rel,
    int log2_pmin, int BH, int nqb, float scale, float alibi, int H)
{
    __shared__ __align__(16) unsigned char lds[2 * cross_tile_lds_bytes<true>()];
    const int l = l_first + blockIdx.y;
    const CrossJob J = cross_job(t1_0, l, chunk, N, far, P_tree, far_rel, log2_pmin);
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int bh = (j / nqb) * 8 + xcd, qb = j % nqb;
    if (!J.any || bh >= BH || qb * 128 >= J.nq) return;   // the whole workgroup leaves together
    const WaveLayer &Y = layers[l];
    cross_tile_wg<true, 4, 2, ALIBI>(nullptr, Y.S.Qf, (const bf16_t *)Y.K, reinterpret_cast<const bf16_t *>(Y.S.Kh), Y.S.VT, Y.S.vt_stride, Y.S.pm, Y.S.pl, Y.S.po,
                                     BH, bh, J.t1, 0, J.t1 - J.P, J.P, qb * 128 + (int)(threadIdx.x >> 6) * 32, J.nq, J.level,
                                     J.level_rel, Y.S.slots, scale, lds, (int)threadIdx.x,
                                     ALIBI ? alibi_slope(alibi, bh % H, H) : 0.f);
}

// blocks of 32 keys (any multiple of 32); grid (ceil(nq/128), B*H, layers), block 256, no barriers
template <bool ALIBI>
__global__ __launch_bounds__(256) void wf_cross_wave_kernel(const WaveLayer *__restrict__ layers, int l_first, int t1_0, int chunk,
                                                            int N, int far, int P_tree, int far_rel, int log2_pmin, int BH,
                                                            float scale, float alibi, int H)
{
    const int l = l_first + blockIdx.z;
    const CrossJob J = cross_job(t1_0, l, chunk, N, far, P_tree, far_rel, log2_pmin);
    const int q0 = blockIdx.x * 128 + (int)(threadIdx.x >> 6) * 32;
    if (!J.any || q0 >= J.nq) return;
    const WaveLayer &Y = layers[l];
    cross_mfma_wave<true, ALIBI>(nullptr, Y.S.Qf, (const bf16_t *)Y.K, Y.S.Klo, Y.S.VT, Y.S.vt_stride, Y.S.pm, Y.S.pl, Y.S.po, BH,
                                 blockIdx.y, J.t1, 0, J.t1 - J.P, J.P, q0, J.nq, J.level, J.level_rel, Y.S.slots, scale,
                                 ALIBI ? alibi_slope(alibi, (int)blockIdx.y % H, H) : 0.f);
}

// plain-ALU form (fp32 storage, or bf16 without the MFMA kernels); grid (max nq, B*H, layers), block 64
template <typename T>
__global__ __launch_bounds__(64) void wf_cross_generic_kernel(const WaveLayer *__restrict__ layers, int l_first, int t1_0,
                                                              int chunk, int N, int far, int P_tree, int far_rel, int log2_pmin,
                                                              int BH, float scale, float alibi, int H)
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
    attend_keys<T>(q, (const T *)Y.K + kb, (const T *)Y.V + kb, rs, J.P, scale, m, lsum, o, nullptr,
                   alibi_slope(alibi, bh % H, H), i0 - (J.t1 - J.P));
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
            if (D.alibi > 0.f)
                hipLaunchKernelGGL(wf_cross_tile_kernel<true>, dim3(bh8 * nqb, nl), dim3(256), 0, st, dev_layers, l0, t1_0, chunk,
                                   D.N, far, P_tree, far_rel, D.log2_pmin, BH, nqb, D.scale, D.alibi, D.H);
            else
                hipLaunchKernelGGL(wf_cross_tile_kernel<false>, dim3(bh8 * nqb, nl), dim3(256), 0, st, dev_layers, l0, t1_0, chunk,
                                   D.N, far, P_tree, far_rel, D.log2_pmin, BH, nqb, D.scale, D.alibi, D.H);
        } else {
            if (D.alibi > 0.f)
                hipLaunchKernelGGL(wf_cross_wave_kernel<true>, dim3((max_nq + 127) / 128, BH, nl), dim3(256), 0, st, dev_layers, l0,
                                   t1_0, chunk, D.N, far, P_tree, far_rel, D.log2_pmin, BH, D.scale, D.alibi, D.H);
            else
                hipLaunchKernelGGL(wf_cross_wave_kernel<false>, dim3((max_nq + 127) / 128, BH, nl), dim3(256), 0, st, dev_layers,
                                   l0, t1_0, chunk, D.N, far, P_tree, far_rel, D.log2_pmin, BH, D.scale, D.alibi, D.H);
        }
    } else {
        hipLaunchKernelGGL(wf_cross_generic_kernel<T>, dim3(max_nq, BH, nl), dim3(64), 0, st, dev_layers, l0, t1_0, chunk, D.N,
                           far, P_tree, far_rel, D.log2_pmin, BH, D.scale, D.alibi, D.H);
    }
    return hipGetLastError();
}

// Queries and temporary pairs of the chunks that layers l_first .. enter at this step, one launch: the pre-pass GEMM
// over the chunk's rows of each layer's input, 1/rms of the rows formed on the way.
// grid (ceil(B * chunk / 128), ceil(3H / 2), layers), block 256.
__global__ __launch_bounds__(256) void wf_prepass_kernel(const WaveLayer *__restrict__ layers, int l_first, int s, int chunk, int B,
                                                         int N, int d, int H, float eps, int norm_free)
{
    const int l = l_first + blockIdx.z, t = layer_pos(s, l, chunk);
    const WaveLayer &Y = layers[l];
    const int Nc = min(chunk, N - t);
    prepass_mfma_body<true>((const bf16_t *)Y.x, nullptr, (const bf16_t *)Y.W.Wq, (const bf16_t *)Y.W.Wk, (const bf16_t *)Y.W.Wv,
                            (const bf16_t *)Y.W.g_attn, (const bf16_t *)Y.W.g_q, (const bf16_t *)Y.W.g_k, (bf16_t *)Y.S.Q,
                            (bf16_t *)Y.S.Kt, (bf16_t *)Y.S.Vt, Y.S.Qf, Y.S.Ktf, B, Nc, (size_t)N * d, t, d, H, eps, norm_free,
                            blockIdx.x, blockIdx.y);
}

// Re-lays n_rows x K row-major weights in fragment order (Scratch::wp_*): one thread per 16-byte piece of the output.
__global__ __launch_bounds__(256) void wf_pack_kernel(const bf16_t *__restrict__ W, bf16_t *__restrict__ Wp, int n_rows, int K)
{
    const size_t q = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (q >= (size_t)n_rows * K / 8) return;
    const int lane = (int)(q & 63), f = (int)((q >> 6) & 1);
    const size_t pr = q >> 7;                       // (row group, step pair)
    const int p = (int)(pr % (size_t)(K / 64)), R = (int)(pr / (size_t)(K / 64));
    const int col = lane & 15, g = lane >> 4;
    *reinterpret_cast<uint4 *>(Wp + q * 8) = *reinterpret_cast<const uint4 *>(W + (size_t)(R * 16 + col) * K + 64 * p + 32 * f + 8 * g);
}
static void pack_launch(const void *W, bf16_t *Wp, int n_rows, int K, hipStream_t st)
{
    const size_t pieces = (size_t)n_rows * K / 8;
    hipLaunchKernelGGL(wf_pack_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st, (const bf16_t *)W, Wp, n_rows, K);
}

bool wavefront_uses_matrix_cores(int d, int F, bool mfma_bf16)
{   // every wavefront's share of a contraction must be a multiple of 64 (d and F multiples of 256)
    return mfma_bf16 && d % 256 == 0 && F % 256 == 0;
}

// Launches one of the four matrix-core products.  Shapes (measured best at d = 1024, F = 4096, 12 layers): WO and W2
// split the contraction in four with eight wavefronts (32 rows per workgroup), W1 does not split it (64 rows), [Wk; Wv]
// splits it in two with eight wavefronts (64 rows = one head).  The operand rows go through LDS when they fit.
constexpr size_t kMmMaxLds = 96 * 1024;
template <int EPI, int KS, int NW>
static hipError_t mm_launch(int n_out, unsigned nl, hipStream_t st, const WaveLayer *dev_layers, int l0, int s, int chunk,
                            const LayerDims &D)
{
    const int K = EPI == EPI_W2 ? D.F : D.d;
    const unsigned bt = (unsigned)((D.B + kMmBatch - 1) / kMmBatch);
    const int Bt = D.B < kMmBatch ? D.B : kMmBatch;
    const size_t base = (size_t)NW * 1024 + 256, xbytes = (size_t)2 * Bt * (K + 8) * 2;
    const dim3 grid((unsigned)(n_out / (16 * NW / KS)), nl, bt);
    if (base + xbytes <= kMmMaxLds) {
        static bool raised = false;   // more than the default 64 KB of dynamic LDS needs the attribute once
        if (!raised) {
            hipError_t e = hipFuncSetAttribute((const void *)wf_mm_kernel<EPI, KS, NW, true>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMmMaxLds);
            if (e != hipSuccess) return e;
            raised = true;
        }
        hipLaunchKernelGGL((wf_mm_kernel<EPI, KS, NW, true>), grid, dim3(64 * NW), base + xbytes, st, dev_layers, l0, s, chunk,
                           D.B, D.N, D.d, D.F, D.H, D.eps, D.norm_free, D.alpha);
    } else {
        hipLaunchKernelGGL((wf_mm_kernel<EPI, KS, NW, false>), grid, dim3(64 * NW), base, st, dev_layers, l0, s, chunk, D.B, D.N,
                           D.d, D.F, D.H, D.eps, D.norm_free, D.alpha);
    }
    return hipSuccess;
}

// The steps of one prefill.  The layers are dealt to W.n groups of consecutive layers, each group enqueued on its own
// stream: a step is a chain of dependent launches, each with a serial start-up and tail, and the chains of different
// groups fill each other's gaps.  A group's first layer enters a chunk only after the group below has finished it:
// one event per group, recorded after every chunk's last step, awaited before the next group's chunk entry.
template <typename T, bool HP, int KSd, int KSF>
static hipError_t wavefront_steps(const LayerDims &D, const WaveLayer *dev_layers, const WaveLayer *host_layers, int L, int chunk,
                                  bool mfma, const WaveStreams &W)
{
    const int B = D.B, N = D.N, d = D.d, F = D.F, BH = D.B * D.H;
    int log2_chunk = 0;
    while ((1 << log2_chunk) < chunk) ++log2_chunk;
    const int far_rel = log2_chunk - D.log2_pmin;
    const unsigned bt = (unsigned)((B + kBatchTile - 1) / kBatchTile);
    constexpr int rows_d = (4 / KSd) * kGemvRows, rows_F = (4 / KSF) * kGemvRows;   // output rows per workgroup
    const bool use_mm = HP && wavefront_uses_matrix_cores(d, F, true);
    const int G = W.n < L ? W.n : L;
    const int per = (L + G - 1) / G;   // layers per group
    hipError_t e;
    // the other streams start after everything enqueued on the caller's stream so far (inputs, layer 0's pre-pass)
    if (G > 1) {
        if ((e = hipEventRecord(W.ev[0], W.st[0])) != hipSuccess) return e;
        for (int g = 1; g < G; ++g)
            if ((e = hipStreamWaitEvent(W.st[g], W.ev[0], 0)) != hipSuccess) return e;
    }
    const int n_steps = N + (L - 1) * chunk;
    for (int s = 0; s < n_steps; ++s) {
        // active layers: 0 <= s - l * chunk < N
        const int a1 = s / chunk < L - 1 ? s / chunk : L - 1;
        const int a0 = s - (N - 1) > 0 ? (s - (N - 1) + chunk - 1) / chunk : 0;
        for (int g = 0; g < G; ++g) {
            const int l0 = a0 > g * per ? a0 : g * per;
            const int l1 = a1 < (g + 1) * per - 1 ? a1 : (g + 1) * per - 1;
            if (l0 > l1) continue;
            hipStream_t st = W.st[g];
            const unsigned nl = (unsigned)(l1 - l0 + 1);
            if (s % chunk == 0) {
                // the active layers enter a chunk: the group below has finished it
                if (g > 0 && (e = hipStreamWaitEvent(st, W.ev[g - 1], 0)) != hipSuccess) return e;
                // queries and temporary pairs of the chunk's rows, then the far tile
                const int lp = l0 > 1 ? l0 : 1;
                if (HP && lp <= l1) {
                    hipLaunchKernelGGL(wf_prepass_kernel, dim3((unsigned)((B * chunk + 127) / 128), (unsigned)((3 * D.H + 1) / 2),
                                                               (unsigned)(l1 - lp + 1)),
                                       dim3(256), 0, st, dev_layers, lp, s, chunk, B, N, d, D.H, D.eps, D.norm_free);
                }
                for (int l = lp; l <= l1 && !HP; ++l) {
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
            hipLaunchKernelGGL((wf_merge_kernel<T, HP>), dim3(BH, nl), dim3(64), 0, st, dev_layers, l0, s, chunk, log2_chunk, BH,
                               D.H, D.p_min, D.log2_pmin, D.scale, D.alibi);
            if (HP && use_mm) {
                if ((e = mm_launch<EPI_WO, 4, 8>(d, nl, st, dev_layers, l0, s, chunk, D)) != hipSuccess) return e;
                if ((e = mm_launch<EPI_W1, 1, 4>(F, nl, st, dev_layers, l0, s, chunk, D)) != hipSuccess) return e;
                if ((e = mm_launch<EPI_W2, 4, 8>(d, nl, st, dev_layers, l0, s, chunk, D)) != hipSuccess) return e;
                // the epilogue of this one also finishes the position (persistent pair and its copies)
                if ((e = mm_launch<EPI_KV, 2, 8>(2 * d, nl, st, dev_layers, l0, s, chunk, D)) != hipSuccess) return e;
            } else {
                hipLaunchKernelGGL((wf_gemv_kernel<T, EPI_WO, KSd>), dim3((d + rows_d - 1) / rows_d, nl, bt), dim3(256), 0, st,
                                   dev_layers, l0, s, chunk, B, N, d, F, D.eps, D.norm_free, D.alpha);
                hipLaunchKernelGGL((wf_gemv_kernel<T, EPI_W1, KSd>), dim3((F + rows_d - 1) / rows_d, nl, bt), dim3(256), 0, st,
                                   dev_layers, l0, s, chunk, B, N, d, F, D.eps, D.norm_free, D.alpha);
                hipLaunchKernelGGL((wf_gemv_kernel<T, EPI_W2, KSF>), dim3((d + rows_F - 1) / rows_F, nl, bt), dim3(256), 0, st,
                                   dev_layers, l0, s, chunk, B, N, d, F, D.eps, D.norm_free, D.alpha);
                hipLaunchKernelGGL((wf_gemv_kernel<T, EPI_KV, KSd>), dim3((2 * d + rows_d - 1) / rows_d, nl, bt), dim3(256), 0, st,
                                   dev_layers, l0, s, chunk, B, N, d, F, D.eps, D.norm_free, D.alpha);
                hipLaunchKernelGGL((wf_finalize_kernel<T, HP>), dim3(BH, nl), dim3(64), 0, st, dev_layers, l0, s, chunk, B, D.H, d,
                                   D.eps, D.norm_free);
            }
            if ((e = hipGetLastError()) != hipSuccess) return e;
            // a block inside the chunk closes: s + 1 positions of layer 0 are finished, every layer is at the same offset
            const int t1 = s + 1;
            const int P = t1 & -t1;
            if (P >= D.p_min && P < chunk) {
                e = wf_cross_launch<T, HP>(D, dev_layers, l0, (int)nl, t1, chunk, 0, P, far_rel, st);
                if (e != hipSuccess) return e;
            }
            // last step of a chunk (or of the sequence): the group above may enter it
            if (g + 1 < G && ((s + 1) % chunk == 0 || s - l1 * chunk == N - 1))
                if ((e = hipEventRecord(W.ev[g], st)) != hipSuccess) return e;
        }
    }
    // the caller's stream continues after every group
    for (int g = 1; g < G; ++g) {
        if ((e = hipEventRecord(W.ev[g], W.st[g])) != hipSuccess) return e;
        if ((e = hipStreamWaitEvent(W.st[0], W.ev[g], 0)) != hipSuccess) return e;
    }
    return hipSuccess;
}

template <typename T>
hipError_t wavefront_prefill(const LayerDims &D, const WaveLayer *dev_layers, const WaveLayer *host_layers, int L, int chunk,
                             bool mfma, const WaveStreams &W)
{
    hipStream_t st = W.st[0];
    // layer 0: its input is known in full, all queries and temporary pairs at once
    hipError_t e = Launch<T>::prepass(D, host_layers[0].W, host_layers[0].S, host_layers[0].x, D.B, D.N, mfma, st);
    if (e != hipSuccess) return e;
    const bool hp = mfma && sizeof(T) == 2;
    if (wavefront_uses_matrix_cores(D.d, D.F, hp)) {
        // the weights in fragment order, once per call (they are the caller's and may have changed since the last one)
        for (int l = 0; l < L; ++l) {
            const WaveLayer &Y = host_layers[l];
            pack_launch(Y.W.Wo, Y.S.wp_o, D.d, D.d, st);
            pack_launch(Y.W.W1, Y.S.wp_1, D.F, D.d, st);
            pack_launch(Y.W.W2, Y.S.wp_2, D.d, D.F, st);
            pack_launch(Y.W.Wk, Y.S.wp_kv, D.d, D.d, st);
            pack_launch(Y.W.Wv, Y.S.wp_kv + (size_t)D.d * D.d, D.d, D.d, st);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    const bool ks2_d = D.d <= 1024, ks2_F = D.F <= 1024;   // one 512-column slice per wavefront up to 1024 columns
#define RT_WF_GO(HPv, KD, KF) return wavefront_steps<T, HPv, KD, KF>(D, dev_layers, host_layers, L, chunk, mfma, W)
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

template hipError_t wavefront_prefill<float>(const LayerDims &, const WaveLayer *, const WaveLayer *, int, int, bool,
                                             const WaveStreams &);
template hipError_t wavefront_prefill<bf16_t>(const LayerDims &, const WaveLayer *, const WaveLayer *, int, int, bool,
                                              const WaveStreams &);

// ---------------------------------------------------------------------------------------------
// One position of one layer with the matrix-core products (rt_decode_step on the bf16 path): the caller's
// row-major weights, one launch per product, smaller workgroups than in the stack engine (one layer has to
// fill the chip by itself).
// ---------------------------------------------------------------------------------------------
bool step_mm_supported(const LayerDims &D, bool mfma_bf16) { return wavefront_uses_matrix_cores(D.d, D.F, mfma_bf16); }

// whether step_mm_launch<EPI, ., NW> stages the operand rows in LDS for these dimensions
template <int EPI, int NW> static bool step_mm_stages(const LayerDims &D)
{
    const int K = EPI == EPI_W2 ? D.F : D.d;
    const int Bt = D.B < kMmBatch ? D.B : kMmBatch;
    return (size_t)NW * 1024 + 256 + (size_t)2 * Bt * (K + 8) * 2 <= (size_t)144 * 1024;
}

template <int EPI, int KS, int NW>
static hipError_t step_mm_launch(const WaveLayer &Y, int n_out, const LayerDims &D, hipStream_t st)
{
    const int K = EPI == EPI_W2 ? D.F : D.d;
    const unsigned bt = (unsigned)((D.B + kMmBatch - 1) / kMmBatch);
    const int Bt = D.B < kMmBatch ? D.B : kMmBatch;
    const size_t base = (size_t)NW * 1024 + 256, xbytes = (size_t)2 * Bt * (K + 8) * 2;
    const dim3 grid((unsigned)(n_out / (16 * NW / KS)), 1, bt);
    constexpr size_t kStepMaxLds = 144 * 1024;   // one layer never has more than one workgroup per compute unit here
    if (base + xbytes <= kStepMaxLds) {
        static bool raised = false;
        if (!raised) {
            hipError_t e = hipFuncSetAttribute((const void *)step_mm_kernel<EPI, KS, NW, true>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kStepMaxLds);
            if (e != hipSuccess) return e;
            raised = true;
        }
        hipLaunchKernelGGL((step_mm_kernel<EPI, KS, NW, true>), grid, dim3(64 * NW), base + xbytes, st, Y, D.B, D.d, D.F, D.H, D.eps,
                           D.norm_free, D.alpha);
    } else {
        hipLaunchKernelGGL((step_mm_kernel<EPI, KS, NW, false>), grid, dim3(64 * NW), base, st, Y, D.B, D.d, D.F, D.H, D.eps,
                           D.norm_free, D.alpha);
    }
    return hipSuccess;
}

static WaveLayer step_layer(const Weights &W, const Scratch &S, const void *x_t, void *y_t, void *K_row, void *V_row)
{
    WaveLayer Y;
    Y.W = W;
    Y.S = S;
    Y.S.Klo = nullptr;   // a decoding step writes the caller's cache rows only
    Y.S.Kh = nullptr;
    Y.S.VT = nullptr;
    Y.x = x_t; Y.y = y_t; Y.K = K_row; Y.V = V_row;
    return Y;
}

// raw [q | k_tmp | v_tmp] of the rows x_t [B][d] into S.qkv_raw
hipError_t step_qkv_mm(const LayerDims &D, const Weights &W, const Scratch &S, const void *x_t, size_t x_stride, hipStream_t st)
{
    if (x_stride != (size_t)D.d) return hipErrorInvalidValue;   // the products address the rows of x_t d apart
    // operand rows that fit LDS: the product's workgroups prepare their operand rows themselves
    if (!step_mm_stages<EPI_QKV, 4>(D))
        hipLaunchKernelGGL(step_prep_kernel, dim3((unsigned)((D.d + 1023) / 1024), (unsigned)D.B), dim3(256), 0, st, (const bf16_t *)x_t,
                           x_stride, (const bf16_t *)W.g_attn, S.op_x, S.ssq_x, D.d, D.norm_free);
    const WaveLayer Y = step_layer(W, S, x_t, nullptr, nullptr, nullptr);
    return step_mm_launch<EPI_QKV, 4, 4>(Y, 3 * D.d, D, st);
}

// h = x_t + alpha Wo a (a as operand rows in S.op_a), MLP, y_t, and the persistent pair into K_row, V_row ([B][H][64])
hipError_t step_base_case_mm(const LayerDims &D, const Weights &W, const Scratch &S, const void *x_t, void *y_t, void *K_row,
                             void *V_row, hipStream_t st)
{
    const WaveLayer Y = step_layer(W, S, x_t, y_t, K_row, V_row);
    hipError_t e;
    // Wo and W2 have d / 16 row groups only: eight wavefronts share each group's contraction (shorter dependent chains)
    // when every wavefront still gets whole 64-index step pairs
    e = D.d % 512 == 0 ? step_mm_launch<EPI_WO, 8, 8>(Y, D.d, D, st) : step_mm_launch<EPI_WO, 4, 4>(Y, D.d, D, st);
    if (e != hipSuccess) return e;
    if ((e = step_mm_launch<EPI_W1, 4, 4>(Y, D.F, D, st)) != hipSuccess) return e;
    e = D.F % 512 == 0 ? step_mm_launch<EPI_W2, 8, 8>(Y, D.d, D, st) : step_mm_launch<EPI_W2, 4, 4>(Y, D.d, D, st);
    if (e != hipSuccess) return e;
    if ((e = step_mm_launch<EPI_KV, 2, 8>(Y, 2 * D.d, D, st)) != hipSuccess) return e;
    return hipGetLastError();
}

}  // namespace rt
