// Shared device helpers and the internal launch interface of the RT layer library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rt {

constexpr int kHeadDim = 64;   // one head = one 64-lane wavefront
constexpr int kBatchTile = 8;  // batch rows one small-M kernel instance handles

typedef uint16_t bf16_t;  // raw bits

// ---------------------------------------------------------------- storage conversions
__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{  // round to nearest, ties to even (inputs are finite on this path)
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
__device__ __forceinline__ uint16_t f32_to_f16_bits(float f)
{   // round to nearest, ties to even
    const _Float16 h = (_Float16)f;
    return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ uint32_t pack_f16(float lo, float hi)
{
    return (uint32_t)f32_to_f16_bits(lo) | ((uint32_t)f32_to_f16_bits(hi) << 16);
}
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return bf16_to_f32(v); }
template <typename T> __device__ __forceinline__ T from_f32(float f);
template <> __device__ __forceinline__ float from_f32<float>(float f) { return f; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float f) { return f32_to_bf16(f); }

// 8 consecutive elements -> 8 floats (16-byte aligned for bf16, 32-byte for f32)
__device__ __forceinline__ void load8(const float *p, float *o)
{
    const float4 a = *reinterpret_cast<const float4 *>(p);
    const float4 b = *reinterpret_cast<const float4 *>(p + 4);
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t *p, float *o)
{
    const uint4 a = *reinterpret_cast<const uint4 *>(p);
    o[0] = __uint_as_float(a.x << 16); o[1] = __uint_as_float(a.x & 0xFFFF0000u);
    o[2] = __uint_as_float(a.y << 16); o[3] = __uint_as_float(a.y & 0xFFFF0000u);
    o[4] = __uint_as_float(a.z << 16); o[5] = __uint_as_float(a.z & 0xFFFF0000u);
    o[6] = __uint_as_float(a.w << 16); o[7] = __uint_as_float(a.w & 0xFFFF0000u);
}

// ---------------------------------------------------------------- wavefront (64 lanes) reductions
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float lane_bcast(float v, int lane)
{  // value of a wave-uniform lane index, read without going through LDS
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// 16 bytes from an address known to be global memory (a pointer that was itself loaded from memory is a generic address
// to the compiler, and accesses through it become flat instructions that also count on the LDS counter, so that every
// wait for an LDS operand waits for them as well; this load stays on the vector-memory counter alone)
typedef unsigned rt_v4u_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 global_load16(const void *p)
{
    const rt_v4u_t v = *(const __attribute__((address_space(1))) rt_v4u_t *)(uintptr_t)p;
    return make_uint4(v[0], v[1], v[2], v[3]);
}

__device__ __forceinline__ float gelu_erf(float u) { return 0.5f * u * (1.0f + erff(u * 0.70710678118654752440f)); }
// erf by the rational form 1 - (1 + a1 x + ... + a6 x^6)^-16 (Abramowitz and Stegun 7.1.28, |error| < 3e-7 before
// rounding, about 2e-6 evaluated in fp32): for outputs that are rounded to bf16 (2^-9 relative) right afterwards.
__device__ __forceinline__ float erf_rational(float x)
{
    const float ax = fabsf(x);
    float p = fmaf(ax, 0.0000430638f, 0.0002765672f);
    p = fmaf(ax, p, 0.0001520143f);
    p = fmaf(ax, p, 0.0092705272f);
    p = fmaf(ax, p, 0.0422820123f);
    p = fmaf(ax, p, 0.0705230784f);
    p = fmaf(ax, p, 1.0f);
    p *= p; p *= p; p *= p; p *= p;
    return copysignf(1.0f - __frcp_rn(p), x);
}
__device__ __forceinline__ float gelu_bf16_out(float u) { return 0.5f * u * (1.0f + erf_rational(u * 0.70710678118654752440f)); }

// =============================================================================================
// One query against a run of KV rows, online softmax (Appendix C, Algorithm 2, for one query row).
// A wavefront owns one (query, batch row, head): lane c holds q[c] and o[c]; within a chunk of
// 64 keys lane j owns key j.  m, l are wave-uniform.
// =============================================================================================
// With HP the keys are Kb + Klo_b (bf16 head plus bf16 remainder, same row layout).
// Linear positional bias (ALiBi): key j of the run is dist_first - j positions before the query and its logit is
// lowered by slope times that distance (slope = 0: no bias).
template <typename T, bool HP = false>
__device__ __forceinline__ void attend_keys(float q, const T *__restrict__ Kb, const T *__restrict__ Vb,
                                            size_t row_stride, int nkeys, float scale, float &m, float &l, float &o,
                                            const bf16_t *__restrict__ Klo_b = nullptr, float slope = 0.f,
                                            int dist_first = 0)
{
    const int lane = threadIdx.x & 63;
    for (int k0 = 0; k0 < nkeys; k0 += 64) {
        const int j = k0 + lane;
        const bool valid = j < nkeys;
        const T *krow = Kb + (size_t)(valid ? j : nkeys - 1) * row_stride;
        float acc = 0.f;
#pragma unroll
        for (int c8 = 0; c8 < 8; ++c8) {
            float kk[8];
            load8(krow + c8 * 8, kk);
            if (HP) {
                float kl[8];
                load8(Klo_b + (size_t)(valid ? j : nkeys - 1) * row_stride + c8 * 8, kl);
#pragma unroll
                for (int e = 0; e < 8; ++e) kk[e] += kl[e];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) acc = fmaf(lane_bcast(q, c8 * 8 + e), kk[e], acc);
        }
        const float logit = valid ? fmaf(-slope, (float)(dist_first - j), acc * scale) : -INFINITY;
        const float m_new = fmaxf(m, wave_max(logit));
        const float resc = expf(m - m_new);  // exp(-inf) = 0 on the first chunk
        const float p = valid ? expf(logit - m_new) : 0.f;
        l = l * resc + wave_sum(p);
        float on = o * resc;
        const int cnt = min(64, nkeys - k0);
        for (int j0 = 0; j0 < cnt; j0 += 8) {  // eight value rows in flight at a time
            float vv[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) vv[e] = to_f32(Vb[(size_t)(k0 + min(j0 + e, cnt - 1)) * row_stride + lane]);
#pragma unroll
            for (int e = 0; e < 8; ++e) on = fmaf(j0 + e < cnt ? lane_bcast(p, min(j0 + e, 63)) : 0.f, vv[e], on);
        }
        o = on;
        m = m_new;
    }
}

// ---------------------------------------------------------------- launch parameters
struct LayerDims {
    int B, N, d, H, F;
    int kv_cap;
    int p_min, log2_pmin;
    float alpha, scale, eps;
    int norm_free;
    float alibi;   // maximum ALiBi bias beta (head slopes 2^(-beta (h+1)/H)); 0 = no positional bias
};

// ALiBi slope of head h (Press et al.: a geometric sequence over the heads)
__host__ __device__ __forceinline__ float alibi_slope(float beta, int h, int H)
{
    return beta > 0.f ? exp2f(-beta * (float)(h + 1) / (float)H) : 0.f;
}

struct Weights {
    const void *Wq, *Wk, *Wv, *Wo, *W1, *W2;
    const void *g_attn, *g_mlp, *g_kv, *g_q, *g_k;
};

// Scratch owned by a context.  Partial softmax states are stored once per (level, query):
//   pm, pl : [levels][slots][B*H]        po : [levels][slots][B*H][64]     (fp32)
struct Scratch {
    void *Q, *Kt, *Vt;   // [N][B][H][64] storage dtype: queries and temporary pairs
    float *Qf, *Ktf;     // [N][B][H][64] unrounded q and k_tmp (persistent engine's high-precision logits), or null
    bf16_t *Klo;         // [N][B][H][64] bf16 remainder k - bf16(k) of the persistent keys, or null
    uint16_t *Kh;        // [N][B][H][64] the persistent keys rounded once to fp16 (11 significant bits): what the LDS-staged
                         // cross-block tiles multiply with the fp16 queries; written wherever Klo is
    bf16_t *VT;          // [B*H][64][vt_stride] transposed copy of the persistent values (bf16 MFMA path)
    int vt_stride;
    float *pm, *pl, *po;
    int levels, slots;
    float *rinv;         // [B*N] 1/rms of the input rows
    float *attn_cat;     // [B][d] concatenated head outputs of the current position
    float *h;            // [B][d]
    float *u;            // [B][F]
    float *z;            // [B][d]
    float *kv_raw;       // [B][2d]
    float *qkv_raw;      // [B][3d] raw q, k_tmp, v_tmp of a decoding step
    // layer-wavefront engine, bf16: inputs of the base-case products as bf16 head + remainder rows (row 2b: head of
    // batch row b, row 2b + 1: remainder), gains already applied; sums of squares per group of 16 elements
    bf16_t *op_a, *op_h, *op_z;   // [2B][d]
    bf16_t *op_u;                 // [2B][F]
    float *ssq_h, *ssq_z;         // [B][d/16]
    bf16_t *op_x;                 // [2B][d] the same for a decoding step's input row (gain g_attn applied)
    float *ssq_x;                 // [B][d/16]
    // the layer's Wo, W1, W2 and [Wk; Wv] re-laid in matrix-core fragment order (or null): for rows 16R .. 16R+15 and
    // contraction indices 64p .. 64p+63, two fragments of 64 lanes x 16 bytes, lane (col, g) of fragment f holding
    // W[16R + col][64p + 32f + 8g .. + 7]; a wavefront's weight stream is then one contiguous run
    bf16_t *wp_o, *wp_1, *wp_2, *wp_kv;
    bf16_t *wg_qkv;      // [3d][d] [Wq; Wk; Wv] with the columns multiplied by the attention RMS gain (tiled pre-pass), MFMA path only
};

__host__ __device__ __forceinline__ size_t partial_index(int level_rel, int slot, int slots, int BH, int bh)
{
    return ((size_t)level_rel * slots + slot) * BH + bh;
}
// compact slot of 0-based query i0 at absolute level l (bit l of i0 must be set)
__host__ __device__ __forceinline__ int partial_slot(int l, int i0) { return ((i0 >> (l + 1)) << l) | (i0 & ((1 << l) - 1)); }

// ---------------------------------------------------------------- launchers (one per kernel family)
template <typename T> struct Launch {
    // rows n0 .. n0+Nc-1 of every batch row of x (batch rows x_bstride elements apart; 0 = Nc * d, a dense
    // [Bc][Nc][d] tensor) -> Q, Kt, Vt rows ((n0 + n)*Bc + b)
    static hipError_t prepass(const LayerDims &D, const Weights &W, const Scratch &S, const void *x, int Bc, int Nc,
                              bool mfma, hipStream_t st, size_t x_bstride = 0, int n0 = 0);
    // one position's q, k_tmp, v_tmp (decoding step): rows b of Q, Kt, Vt
    static hipError_t prepass_one(const LayerDims &D, const Weights &W, const Scratch &S, const void *x_t, size_t x_stride,
                                  hipStream_t st, bool matrix_cores = false);
    // split_out: a is also written as operand rows (bf16 head + remainder) into S.op_a
    static hipError_t merge(const LayerDims &D, const Scratch &S, const void *K, const void *V, int t, int q_row,
                            int n_decode_splits, hipStream_t st, bool split_out = false);
    static hipError_t gemv_wo(const LayerDims &D, const Weights &W, const Scratch &S, const void *x_t, size_t x_stride_b,
                              hipStream_t st);
    static hipError_t gemv_w1(const LayerDims &D, const Weights &W, const Scratch &S, hipStream_t st);
    static hipError_t gemv_w2(const LayerDims &D, const Weights &W, const Scratch &S, void *y_t, size_t y_stride_b,
                              hipStream_t st);
    static hipError_t gemv_kv(const LayerDims &D, const Weights &W, const Scratch &S, hipStream_t st);
    static hipError_t finalize_kv(const LayerDims &D, const Weights &W, const Scratch &S, void *K, void *V, int t,
                                  bool write_vt, hipStream_t st);
    static hipError_t cross(const LayerDims &D, const Scratch &S, const void *K, const void *V, int t1, int P, int nq,
                            bool mfma, hipStream_t st);
    static hipError_t decode_split(const LayerDims &D, const Scratch &S, const void *K, const void *V, int t, int chunk,
                                   int nsplit, hipStream_t st);
    // The layer without its sequential loop (recompute from a given output, Sec. 6.1; Transformer layer, Sec. 2.1) on the
    // plain-ALU kernels, any storage type: pre-pass over pairs_src -> K, V rows; pre-pass over x unless the pairs are the
    // temporary ones; one wavefront per (b, h, position) for the attention; the three products in tiles of eight rows.
    // par: loop_free_scratch_bytes(B * N, d, F) bytes.
    static hipError_t loop_free(const LayerDims &D, const Weights &W, const Scratch &S, const void *x, const void *pairs_src,
                                bool pairs_are_temporary, void *y, void *K, void *V, void *par, hipStream_t st);
    static size_t loop_free_scratch_bytes(size_t M, size_t d, size_t F) { return M * (3 * d + F) * 4 + 1024; }
    // The blocked recurrence (blocks of Sblk positions: persistent pairs across blocks, temporary pairs inside a block) on
    // the same plain-ALU kernels; same scratch.
    static hipError_t blocked_generic(const LayerDims &D, const Weights &W, const Scratch &S, const void *x, int Sblk, void *y,
                                      void *K, void *V, void *par, hipStream_t st);
};

// One layer of a stack as the layer-wavefront engine's kernels see it (an array of these lives in device memory).
struct WaveLayer {
    Weights W;
    Scratch S;        // this layer's own queries, temporary pairs, partial states and base-case vectors
    const void *x;    // [B][N][d] input (the output of the layer below)
    void *y;          // [B][N][d] output
    void *K, *V;      // [kv_cap][B][H][64]
};

// Streams of the layer-wavefront engine: st[0] is the caller's, the others belong to the context (default
// priority); ev[g] orders group g + 1 after group g (ev[0] also starts the other streams, ev[g >= 1] joins them).
constexpr int kMaxWaveStreams = 4;
struct WaveStreams {
    int n;
    hipStream_t st[kMaxWaveStreams];
    hipEvent_t ev[kMaxWaveStreams];
};

// All layers of a stack, layer l running `chunk` positions behind layer l - 1 (rt_wavefront.hip).
template <typename T>
hipError_t wavefront_prefill(const LayerDims &D, const WaveLayer *dev_layers, const WaveLayer *host_layers, int L, int chunk,
                             bool mfma, const WaveStreams &W);
// whether the engine's matrix-core products cover this shape (they need the packed weight copies in the scratch)
// one cross-block UpdateTile on the matrix cores (bf16), queries t1+1 .. t1+nq against keys t1-P+1 .. t1 (1-based);
// hp: high-precision logits from the unrounded queries (S.Qf) and the key remainders (S.Klo)
hipError_t cross_mfma_launch(const LayerDims &D, const Scratch &S, const void *K, int t1, int P, int nq, bool hp, hipStream_t st);
bool wavefront_uses_matrix_cores(int d, int F, bool mfma_bf16);
// One position of one layer with the same products from the caller's row-major weights (decoding, bf16): x_t, y_t
// rows d apart ([B][d]); K_row, V_row the cache rows to write ([B][H][64]).
bool step_mm_supported(const LayerDims &D, bool mfma_bf16);
hipError_t step_qkv_mm(const LayerDims &D, const Weights &W, const Scratch &S, const void *x_t, size_t x_stride, hipStream_t st);
hipError_t step_base_case_mm(const LayerDims &D, const Weights &W, const Scratch &S, const void *x_t, void *y_t, void *K_row,
                             void *V_row, hipStream_t st);

// Whole-sequence evaluation when every key-value pair is known in advance (rt_parallel.hip): the recompute of a
// layer from its input and output (Sec. 6.1) and the standard Transformer layer (Sec. 2.1).  bf16 + matrix cores.
bool parallel_supported(const LayerDims &D, bool mfma_bf16);
size_t parallel_scratch_bytes(size_t M, size_t d, size_t F);
hipError_t parallel_layer(const LayerDims &D, const Weights &W, const Scratch &S, const void *x, const void *pairs_src,
                          bool pairs_are_temporary, void *y, void *K, void *V, void *par, hipStream_t st);
// blocked recurrence over blocks of Sblk positions (a power of two dividing p_min); same scratch
hipError_t blocked_layer(const LayerDims &D, const Weights &W, const Scratch &S, const void *x, int Sblk, void *y, void *K, void *V,
                         void *par, hipStream_t st);

// The attention of every position from fp32 rows (the backward pass's recompute, Sec. 6.1) as the same masked pass on the
// matrix cores: Qn, Ktn, Vt, Kp, Vp [N][B H][64] fp32 (queries, temporary pairs, persistent pairs) -> c [N][B H][64] and the
// log-sum-exp of every query's logits lse [N][B H].  Keys enter as bf16 head + remainder, values as bf16.
size_t flash_recompute_scratch_bytes(size_t B, size_t N, size_t d, size_t H);
hipError_t flash_recompute_f32(const LayerDims &D, const float *Qn, const float *Ktn, const float *Vt, const float *Kp, const float *Vp,
                               float *c, float *lse, void *scratch, hipStream_t st);

// embedding lookup and final-norm + output projection of a layer stack (rt_stack.hip)
template <typename T>
hipError_t embed_rows_launch(const void *table, const int32_t *ids, void *x, int B, int N, int d, int vocab,
                             long long ids_stride, int first, hipStream_t st);
template <typename T>
hipError_t lm_head_launch(const void *W, const void *g, const void *z, long long z_stride, float *logits, int B, int d,
                          int vocab, float eps, int norm_free, hipStream_t st);

}  // namespace rt
