// Single-launch ("persistent") engine of the sequential loop, bf16 storage.
//
// One cooperative grid of 256 workgroups (one per compute unit) x 512 threads runs all N positions.
// The five matrices of the loop (Wo, W1, W2, Wk, Wv) are split over the workgroups and held in LDS
// for the whole call (weight-stationary: 11 d^2 bf16 elements over 256 x 160 KB of LDS), so a position
// costs no weight traffic at all.  Wo, W1, [Wk; Wv] are split by output rows; W2 in two dimensions
// (64 row blocks x 4 contraction blocks) so that no workgroup has to pull the 4d-wide hidden vector.
// The RMS gains g_mlp, g_kv are folded into the stationary W1, Wk, Wv (W diag(g), rounded once), and
// each RMS scale is applied after its product (the products are linear in their input), so the
// exchanged vectors carry neither gain nor norm and no phase waits for a statistic.
//
// What remains on the critical path is the exchange of small vectors between the phases of a position:
//
//   M    per (b, h) wavefront: poll the raw k, v of position t-1 and the partial sums of z^2; finish
//        that persistent pair (RMS scale of z, qkRMS of k; store K, V, the transposed value copy and
//        the LDS window row); fold it as the newest key into the pre-merged softmax state   -> a
//   O    h = x_t + alpha Wo a                                                                -> bf16(h)
//   1    u = gelu(W1' h / rms(h)),  1/rms(h) from the received values themselves             -> u
//   2a   partial W2 u over one quarter of the hidden dimension                               -> 4 partial sums
//   2b   z = h + alpha (sum of partials), same rows as O                      -> y, bf16(z), partial sums of z^2
//   KV   [Wk'; Wv'] z  (scale 1/rms(z) applied in M)                                         -> raw k, v
// The pre-merge of position t+1 (temporary pair, stored partial states of the bits of c = t at or above
// p_min, direct window out of LDS: everything but the newest key) is kept off this chain.  At a position
// without a cross-block event a helper wavefront of the owning workgroup issues its global loads during
// phase M, parks them in LDS, combines them with the window during phase 2b (it is idle in both phases)
// and leaves q, m, l, o in LDS for the owner.  At an event position the stored states only arrive behind
// phase M: there the helper fetches during phase 2b and the owner combines after the product of phase KV.
//
// Logits are formed from unrounded operands: fp32 q and temporary k from the pre-pass, fp32 keys in the
// LDS window, and for the cross-block tiles the persistent key as bf16 head + bf16 remainder (three MFMA
// terms).  The K the caller receives is the bf16 head.
//
// Exchange format: every value crosses the chip inside a self-validating 64-bit word
// [tag:32 | payload:32] (payload = two bf16 or one fp32), written with one 8-byte agent-scope atomic
// store.  Consumers poll the data itself until every tag equals the tag of (call, position): a hop
// costs one store-to-load trip through the memory side.  Measured on MI355X with 256 workgroups: a
// fenced grid barrier (release, counter, acquire) 7.5-11 us, the fences alone 3.6-7.9 us, a counter
// barrier without fences 4.2 us, a flag-in-data all-to-all hop 2.7-3.3 us; waiting for separate
// "producer done" words before the bulk loads was slower than polling the data (39.8 vs 34.3 us per
// position, so that variant is gone).  Bulk loads are pulled thread-linearly with 16-byte
// agent-scope buffer loads and staged in LDS (see wg_gemv_ll).  Buffers alternate with the parity of t;
// a writer of position t+2 has always (transitively) gathered the partial sums of z^2 of position t+1
// from all workgroups, which each of them stored after it had finished reading position t.
//
// K, V, the transposed value copy and the partial softmax states live in ordinary cached memory.
// The per-position window only re-reads rows that the same wavefront wrote (kept in LDS when
// p_min <= 64).  Cross-workgroup use happens at the cross-block events (every p_min positions): those
// run inline on all wavefronts, bracketed by two fenced grid barriers (release / acquire, agent scope).
//
// Relative to the per-position engine the block decomposition is shifted by one: query t takes its
// newest key t-1 directly (the wavefront that merges has just finished that key), keys [0, t-1) are
// split by the bits of c = t-1 into stored partials (blocks >= p_min) and the direct window.  The
// UpdateTile of the block ending at key e-1 therefore has a whole position of slack.
//
// Every wait is bounded: a poll loop that exceeds spin_limit raises the abort word, every workgroup
// leaves the kernel at its next wait, and the host reports it (rt_device_wait_expired).
#include "rt_persistent.h"
#include "rt_ll.h"
#include <cstring>
#include "rt_cross_tile.h"

#include <cstdlib>

namespace rt {

constexpr int kGlobalP = 256;           // cross-block events of at least this many keys are spread over all workgroups
constexpr int kMaxLevels = 16;         // stored-partial levels a query can take (p_min 32 .. sequence 2^20)

struct PersistArgs {
    int B, N, d, H, F, BH;
    int p_min, log2_pmin;
    float alpha, scale, eps;
    int norm_free;
    int G;
    int R_o, R_1, R_kv;   // rows per workgroup of Wo (and of the z rows it finishes), W1, [Wk; Wv] (all even)
    int R_2;              // rows of a W2 row block = d/64; workgroup (rb, jb) = (wg/4, wg%4) holds W2[rb block][jb*d .. +d)
    int ldw_d, ldw_F;     // LDS row strides in elements
    const bf16_t *Wo, *W1, *W2, *Wk, *Wv, *g_mlp, *g_kv, *g_k;
    const bf16_t *x;
    bf16_t *y, *K, *V;
    const bf16_t *Q, *Kt, *Vt;
    const float *Qf, *Ktf;      // unrounded q, k_tmp
    bf16_t *Klo;                // remainder k - bf16(k) of the persistent keys
    uint16_t *Kh;               // the persistent keys in fp16 (operands of the LDS-staged cross-block tiles)
    bf16_t *VT;
    int vt_stride;
    float *pm, *pl, *po;
    int levels, slots;
    // exchange buffers, each [2 parities][kBMax][...] words
    ll_t *a_ll, *h_ll, *z_ll;   // [..][d/2]   two bf16 per word
    ll_t *u_ll;                 // [..][F/2]
    ll_t *kv_ll;                // [..][2d]    one fp32 per word
    ll_t *zss_ll;               // [..][G]     one fp32 per word
    ll_t *zp_ll;                // [2][4][kBMax][d] one fp32 per word: partial W2 products of the four contraction blocks
    int win_rows;               // p_min when the direct window is kept in LDS, else 0 (window re-read from K, V)
    int upw;                    // merge units per workgroup = ceil(BH_max / G)
    int max_batch;              // rows of the LDS staging area
    unsigned tag_base;          // (call nonce) << 20
    unsigned long long *bar;    // [0] fenced-barrier counter, [8] abort word
    unsigned long long *trace;  // optional: [2][trace_rows][16] wall-clock stamps of workgroup 0 and of workgroup trace_wg
    int trace_wg, trace_rows;
    int pre_sleep;              // units of 4 x 64 clocks a bulk pull waits before its first poll
    int ps_o, ps_1, ps_2a, ps_kv;   // the same per phase
    int early_premerge;         // the helper wavefront also combines the pre-merge (phase 2b) at positions without an event
    long long spin_limit;
    float alibi;                // maximum ALiBi bias (kernels instantiated with ALIBI only)
};

// Direct window out of LDS: query (lane c holds q[c]) against nkeys <= 64 rows kept by this wavefront.
// ALIBI: key j of the window is dist_first - j positions before the query, its logit lowered by slope times that.
template <bool ALIBI>
__device__ __forceinline__ void attend_lds(float q, const float *ks, const bf16_t *vs, int nkeys, float scale, float &m,
                                           float &l, float &o, float slope, int dist_first)
{
    const int lane = threadIdx.x & 63;
    const bool valid = lane < nkeys;
    const float *krow = ks + (size_t)(valid ? lane : 0) * (kHeadDim + 4);   // rows padded against bank conflicts
    float acc = 0.f;
#pragma unroll
    for (int c8 = 0; c8 < 8; ++c8) {
        float kk[8];
        load8(krow + c8 * 8, kk);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc = fmaf(lane_bcast(q, c8 * 8 + e), kk[e], acc);
    }
    const float logit = valid ? (ALIBI ? fmaf(-slope, (float)(dist_first - lane), acc * scale) : acc * scale) : -INFINITY;
    const float m_new = fmaxf(m, fast_max(logit));
    const float resc = __expf(m - m_new);
    const float p = valid ? __expf(logit - m_new) : 0.f;
    l = l * resc + fast_sum(p);
    float on = o * resc;
    // eight value rows are requested before their products (one dependent LDS read per key cost about a microsecond for a full
    // window); rows past the end are read from the last row with weight zero
#pragma unroll
    for (int j0 = 0; j0 < 64; j0 += 8) {
        if (j0 >= nkeys) break;   // wavefront-uniform
        float vv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) vv[e] = bf16_to_f32(vs[(size_t)min(j0 + e, nkeys - 1) * kHeadDim + lane]);
#pragma unroll
        for (int e = 0; e < 8; ++e) on = fmaf(lane_bcast(p, j0 + e), vv[e], on);
    }
    o = on;
    m = m_new;
}

#define RT_STAMP(k)                                                                         \
    do {                                                                                    \
        if (A.trace && tid == 0 && (wg == 0 || wg == A.trace_wg))                            \
            A.trace[((size_t)(wg == 0 ? 0 : A.trace_rows) + t) * 16 + (k)] = wall_clock64(); \
    } while (0)

// Workgroup barrier that also makes every wavefront leave when any of them has given up waiting: the wavefront that gave
// up raises an LDS flag before the barrier, everybody reads it behind the barrier (the flag is never lowered again, so all
// wavefronts take the same branch).  One barrier and one LDS read: a workgroup-wide reduction of the predicate costs two
// barriers and LDS atomics, six times per position.
#define RT_ABORT_IF(cond)                                                                                  \
    do {                                                                                                   \
        if (cond) flag_s[1] = 1;                                                                           \
        __syncthreads();                                                                                   \
        if (flag_s[1] != 0) {                                                                              \
            if (threadIdx.x == 0) __hip_atomic_store(A.bar + 8, 1ULL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); \
            return;                                                                                        \
        }                                                                                                  \
    } while (0)

// Part of the merge of a position that does not need its newest key: the temporary pair, the stored
// partial states (bits of c = t-1 at or above p_min) and the direct window.  The loads are issued ahead
// (pre_issue) and combined later (pre_finish) by the wavefronts named in the file header, so that phase M
// only waits for the raw k, v of the newest key.
struct PreLoad {
    float q, kt, vt;
    float pm[kMaxLevels], pl[kMaxLevels], po[kMaxLevels];
};

__device__ __forceinline__ void pre_issue(const PersistArgs &A, int t, int u, PreLoad &L)
{
    const int lane = threadIdx.x & 63;
    const size_t rs = (size_t)A.BH * kHeadDim;
    const size_t qoff = (size_t)t * rs + (size_t)u * kHeadDim + lane;
    L.q = A.Qf[qoff];
    L.kt = A.Ktf[qoff];
    L.vt = bf16_to_f32(A.Vt[qoff]);
    const int c = t - 1;
#pragma unroll
    for (int lr = 0; lr < kMaxLevels; ++lr) {
        const int lv = lr + A.log2_pmin;
        const bool on = t >= 2 && lr < A.levels && ((c >> lv) & 1);
        const size_t idx = on ? partial_index(lr, partial_slot(lv, c), A.slots, A.BH, u) : 0;
        L.pm[lr] = on ? A.pm[idx] : -INFINITY;
        L.pl[lr] = on ? A.pl[idx] : 0.f;
        L.po[lr] = on ? A.po[idx * kHeadDim + lane] : 0.f;
    }
}

// PreLoad <-> LDS (layout: q, kt, vt rows of 64, then pm[], pl[] as broadcast scalars, then po[][64])
constexpr int kPreFloats = 3 * 64 + 2 * kMaxLevels + kMaxLevels * 64;
__device__ __forceinline__ void pre_to_lds(const PreLoad &L, float *s)
{
    const int lane = threadIdx.x & 63;
    s[lane] = L.q; s[64 + lane] = L.kt; s[128 + lane] = L.vt;
#pragma unroll
    for (int lr = 0; lr < kMaxLevels; ++lr) {
        if (lane == 0) { s[192 + lr] = L.pm[lr]; s[192 + kMaxLevels + lr] = L.pl[lr]; }
        s[192 + 2 * kMaxLevels + lr * 64 + lane] = L.po[lr];
    }
}
__device__ __forceinline__ void pre_from_lds(const float *s, PreLoad &L)
{
    const int lane = threadIdx.x & 63;
    L.q = s[lane]; L.kt = s[64 + lane]; L.vt = s[128 + lane];
#pragma unroll
    for (int lr = 0; lr < kMaxLevels; ++lr) {
        L.pm[lr] = s[192 + lr];
        L.pl[lr] = s[192 + kMaxLevels + lr];
        L.po[lr] = s[192 + 2 * kMaxLevels + lr * 64 + lane];
    }
}

// ALIBI: the stored partial states are already in this query's frame; the window key c - w + j is w + 1 - j
// positions before query t = c + 1.
template <bool ALIBI>
__device__ __forceinline__ void pre_finish(const PersistArgs &A, int t, int u, const PreLoad &L, const float *wk,
                                           const bf16_t *wv, float &q, float &m, float &l, float &o)
{
    q = L.q;
    m = A.scale * fast_sum(L.q * L.kt);
    l = 1.f;
    o = L.vt;
    if (t < 2) return;
    float mx = m;
#pragma unroll
    for (int lr = 0; lr < kMaxLevels; ++lr) mx = fmaxf(mx, L.pm[lr]);
    const float e0 = __expf(m - mx);
    l *= e0;
    o *= e0;
#pragma unroll
    for (int lr = 0; lr < kMaxLevels; ++lr) {
        const float f = __expf(L.pm[lr] - mx);   // exp(-inf) = 0 for absent levels
        l = fmaf(L.pl[lr], f, l);
        o = fmaf(L.po[lr], f, o);
    }
    m = mx;
    const int c = t - 1;
    const int w = c & (A.p_min - 1);
    if (w > 0) {
        const float slope = ALIBI ? alibi_slope(A.alibi, u % A.H, A.H) : 0.f;
        if (A.win_rows) {
            attend_lds<ALIBI>(q, wk, wv, w, A.scale, m, l, o, slope, w + 1);
        } else {
            const size_t rs = (size_t)A.BH * kHeadDim;
            const size_t base = (size_t)(c - w) * rs + (size_t)u * kHeadDim;
            if (ALIBI) attend_keys<bf16_t>(q, A.K + base, A.V + base, rs, w, A.scale, m, l, o, nullptr, slope, w + 1);
            else attend_keys<bf16_t>(q, A.K + base, A.V + base, rs, w, A.scale, m, l, o);
        }
    }
}

// One cross-block item of the whole workgroup.
template <bool ALIBI>
__device__ __forceinline__ void cross_tile_item(const PersistArgs &A, int bh, int t, int P, int q0, int nq, int level,
                                             unsigned char *lds)
{
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));   // opaque: keeps the tile's lane-derived addresses out of the registers of the per-position phases
    if (ALIBI)
        cross_tile_wg<true, kPW, 1, true>(A.Q, A.Qf, A.K, reinterpret_cast<const bf16_t *>(A.Kh), A.VT, A.vt_stride, A.pm, A.pl, A.po, A.BH, bh, t, 1, t - P, P, q0,
                                          nq, level, level - A.log2_pmin, A.slots, A.scale, lds, tid,
                                          alibi_slope(A.alibi, bh % A.H, A.H));
    else
        cross_tile_wg<true, kPW, 1>(A.Q, A.Qf, A.K, reinterpret_cast<const bf16_t *>(A.Kh), A.VT, A.vt_stride, A.pm, A.pl, A.po, A.BH, bh, t, 1, t - P, P, q0, nq,
                                    level, level - A.log2_pmin, A.slots, A.scale, lds, tid);
}

// KSD = d / 256, KSF = F / 256: contraction steps per wavefront, fixed at compile time so that all
// exchange loads of a phase are in flight at once without spilling.
// ALIBI: linear positional bias (PersistArgs::alibi); a separate instantiation, the plain kernel is unchanged.
template <int KSD, int KSF, bool ALIBI = false>
__global__ __launch_bounds__(kPThreads) void persistent_kernel(PersistArgs A)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wg = blockIdx.x, G = A.G;
    const int d = A.d, F = A.F, B = A.B, BH = A.BH;
    // rows per workgroup of Wo (and of the z rows it finishes), W1 and [Wk; Wv] for d = 256 KSD over 256 workgroups
    // (the host computes the same numbers into A.R_o, A.R_1, A.R_kv)
    constexpr int RO = 2 * ((KSD + 1) / 2), R1 = 4 * KSD, RKV = 2 * KSD;

    // ---- LDS carve-up
    bf16_t *wo_s = reinterpret_cast<bf16_t *>(smem);
    bf16_t *w1_s = wo_s + (size_t)A.R_o * A.ldw_d;
    bf16_t *w2_s = w1_s + (size_t)A.R_1 * A.ldw_d;
    bf16_t *wkv_s = w2_s + (size_t)A.R_2 * A.ldw_d;
    float *red = reinterpret_cast<float *>(wkv_s + (size_t)A.R_kv * A.ldw_d);  // [kPW][kRMax][kBMax]
    float *h_loc = red + kPW * kRMax * kBMax;                                  // [kRMax][kBMax]
    float *sq = h_loc + kRMax * kBMax;                                         // [32][kBMax]
    float *rinv_s = sq + 32 * kBMax;                                           // [kBMax]
    int *flag_s = reinterpret_cast<int *>(rinv_s + kBMax);
    float *win_k = reinterpret_cast<float *>(flag_s + 4);                      // [upw][win_rows][64 + 4] unrounded keys
    bf16_t *win_v = reinterpret_cast<bf16_t *>(win_k + (size_t)A.upw * A.win_rows * (kHeadDim + 4));   // [upw][win_rows][64]
    bf16_t *act_s = win_v + (size_t)A.upw * A.win_rows * kHeadDim;             // [max_batch][ldw_d] staged activations
    float *pre_s = reinterpret_cast<float *>(act_s + (size_t)A.max_batch * A.ldw_d);   // [upw][kPreFloats] pre-fetched merge inputs

    // ---- this workgroup's rows
    const int o_lo = min(wg * A.R_o, d), o_n = min(d, o_lo + A.R_o) - o_lo;          // Wo, W2
    const int f_lo = min(wg * A.R_1, F), f_n = min(F, f_lo + A.R_1) - f_lo;          // W1
    const int kv_lo = min(wg * A.R_kv, 2 * d), kv_n = min(2 * d, kv_lo + A.R_kv) - kv_lo;  // [Wk; Wv]

    // W2 is split in two dimensions: row block rb (RB = d/64 rows) x contraction block jb (d columns of F = 4d)
    const int rb = wg >> 2, jb = wg & 3, RB = A.R_2;
    copy_rows_to_lds(wo_s, A.ldw_d, A.Wo, d, 0, d, o_lo, o_n);
    const bf16_t *gm = A.norm_free ? nullptr : A.g_mlp, *gkv = A.norm_free ? nullptr : A.g_kv;
    copy_rows_to_lds(w1_s, A.ldw_d, A.W1, d, 0, d, f_lo, f_n, gm);
    copy_rows_to_lds(w2_s, A.ldw_d, A.W2, F, jb * d, d, rb * RB, RB);
    {   // [Wk; Wv] rows, one at a time (a row block may straddle the two matrices)
        for (int r = 0; r < kv_n; ++r) {
            const int o = kv_lo + r;
            if (o < d) copy_rows_to_lds(wkv_s + (size_t)r * A.ldw_d, A.ldw_d, A.Wk, d, 0, d, o, 1, gkv);
            else copy_rows_to_lds(wkv_s + (size_t)r * A.ldw_d, A.ldw_d, A.Wv, d, 0, d, o - d, 1, gkv);
        }
    }
    if (tid == 0) flag_s[1] = 0;   // "a wavefront of this workgroup gave up waiting"
    __syncthreads();

    const size_t rs = (size_t)BH * kHeadDim;
    unsigned long long nbar = 0;
    const int erow = tid >> 4, eb = tid & 15;  // epilogue thread -> (row, batch) for tid < 256
    const size_t half_d = (size_t)kBMax * (d / 2), half_F = (size_t)kBMax * (F / 2);
    const size_t sz_kv = (size_t)kBMax * 2 * d, sz_ss = (size_t)kBMax * G;

    // this wavefront's merge unit (at most one: B*H <= G*kPW), and its pre-merged state for the next position
    const int my_u = wg + G * wave;
    const bool has_u = my_u < BH;
    // gain of the key normalisation for this wavefront's head: fetched once, phase M is on the critical path of every position
    const float my_gk = (has_u && A.g_k) ? bf16_to_f32(A.g_k[(my_u % A.H) * kHeadDim + lane]) : 1.f;
    const float *my_wk = win_k + (size_t)wave * A.win_rows * (kHeadDim + 4);
    const bf16_t *my_wv = win_v + (size_t)wave * A.win_rows * kHeadDim;
    float cq = 0.f, cm = 0.f, cl = 1.f, co = 0.f;
    // The loads of a pre-merge are made by an otherwise idle helper wavefront (wave 4 + slot) and handed over
    // through LDS, so that no wavefront carries them in registers across a phase.
    const int help_slot = wave - 4;
    const int help_u = wg + G * help_slot;
    const bool is_helper = help_slot >= 0 && help_slot < A.upw && help_u < BH;
    const float *help_wk = win_k + (size_t)(is_helper ? help_slot : 0) * A.win_rows * (kHeadDim + 4);
    const bf16_t *help_wv = win_v + (size_t)(is_helper ? help_slot : 0) * A.win_rows * kHeadDim;
    if (is_helper) {
        PreLoad L;
        pre_issue(A, 0, help_u, L);
        pre_to_lds(L, pre_s + (size_t)help_slot * kPreFloats);
    }
    __syncthreads();
    if (has_u) {
        PreLoad L;
        pre_from_lds(pre_s + (size_t)wave * kPreFloats, L);
        pre_finish<ALIBI>(A, 0, my_u, L, my_wk, my_wv, cq, cm, cl, co);
    }

    for (int t = 0; t <= A.N; ++t) {
        const int par = t & 1, ppar = par ^ 1;
        const unsigned tag = A.tag_base | (unsigned)(t + 1);   // words produced at position t
        const unsigned ptag = A.tag_base | (unsigned)t;        // words produced at position t-1
        int fail = 0;
        if (t < A.N) RT_STAMP(0);
        // The residual input of this workgroup's rows is fetched ahead of phase O - by wavefront 1, into LDS (sq is free until
        // phase 1): the rows' epilogue threads sit in wavefront 0, which is the merging wavefront, and a wavefront gets its
        // loads back in issue order: this read of x comes from HBM and would hold up phase M's polls behind it.
        if (t < A.N && wave == 1) {
            const int xr = lane >> 4, xb = lane & 15;
            if (xr < o_n && xb < B) sq[xr * kBMax + xb] = bf16_to_f32(A.x[((size_t)xb * A.N + t) * d + o_lo + xr]);
        }
        // At a position without a cross-block event the stored states that the next position's pre-merge reads are complete
        // already, so the helper wavefront fetches them during phase M (it is idle there), combines them with the window in
        // phase 2b (idle again) and leaves the finished state in LDS: the owning wavefront then has nothing to do behind the
        // product of phase KV, which is on the critical path of every position.  At an event position the states arrive
        // after phase M: there the helper fetches in phase 2b and the owner combines behind phase KV.
        const bool early = A.early_premerge && !(t >= A.p_min && (t & -t) >= A.p_min) && t + 1 < A.N;
        if (early && is_helper) {
            PreLoad L;
            pre_issue(A, t + 1, help_u, L);
            pre_to_lds(L, pre_s + (size_t)help_slot * kPreFloats);
        }
        // ================================================================ phase M
        if (has_u) {
            const int u = my_u;
            const int b = u / A.H, h = u - b * A.H;
            float q = cq, m = cm, l = cl, o = co;   // pre-merged one phase ahead
            // (2) the newest key: position t-1's raw k, v arrive from phase KV, are finished and stored here
            float kr = 0.f;
            bf16_t kb = 0, vb = 0;
            if (t >= 1) {
                const ll_t *p[6];
                bool act[6];
                ll_t w6[6];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    act[i] = i * 64 + lane < G;
                    p[i] = A.zss_ll + ppar * sz_ss + (size_t)(act[i] ? i * 64 + lane : 0) * kBMax + b;
                }
                p[4] = A.kv_ll + ppar * sz_kv + single_word<RKV>(h * kHeadDim + lane, b);
                p[5] = A.kv_ll + ppar * sz_kv + single_word<RKV>(d + h * kHeadDim + lane, b);
                act[4] = act[5] = true;
                ll_wait_n<6>(p, act, ptag, A, w6, fail);
                float ss = 0.f;
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (act[i]) ss += __uint_as_float((unsigned)w6[i]);
                // |z|^2, |k|^2 and q . (g k) of the raw key are three independent reductions (one after the other they are three
                // dependent chains on the critical path of every position); the scales multiply the finished sums
                const float k0 = __uint_as_float((unsigned)w6[4]);
                const float kg = A.norm_free ? k0 : k0 * my_gk;
                const float Sz = fast_sum(ss), Sk = fast_sum(k0 * k0), Sq = fast_sum(q * kg);
                const float rz = A.norm_free ? 1.f : rsqrtf(Sz / (float)d + A.eps);
                const float kscale = A.norm_free ? 1.f : rz * rsqrtf(rz * rz * Sk / (float)kHeadDim + A.eps);
                kr = kg * kscale;
                const float vr = __uint_as_float((unsigned)w6[5]) * rz;
                kb = f32_to_bf16(kr);
                vb = f32_to_bf16(vr);
                if (t < A.N) {
                    // the newest key is one position before the query
                    const float sn = ALIBI ? A.scale * (Sq * kscale) - alibi_slope(A.alibi, h, A.H) : A.scale * (Sq * kscale);
                    const float m_new = fmaxf(m, sn);
                    const float e1 = __expf(m - m_new), e2 = __expf(sn - m_new);
                    l = l * e1 + e2;
                    o = o * e1 + bf16_to_f32(vb) * e2;
                    m = m_new;
                }
            }
            if (t < A.N) {
                const float av = o * __builtin_amdgcn_rcpf(l);   // a crosses the chip as bf16
                const float an = dpp_odd_neighbour(av);
                if (!(lane & 1))
                    ll_store(A.a_ll + par * half_d + pair_word<32>(h * kHeadDim + lane, b), tag,
                             (unsigned)f32_to_bf16(av) | ((unsigned)f32_to_bf16(an) << 16));
            }
            // the stores of the finished pair follow a: only a is on the critical path of the position
            if (t >= 1) {
                const size_t off = (size_t)(t - 1) * rs + (size_t)u * kHeadDim + lane;
                A.K[off] = kb;
                A.V[off] = vb;
                if (!A.win_rows) A.VT[((size_t)u * kHeadDim + lane) * A.vt_stride + (t - 1)] = vb;   // else: from the ring, below
                A.Klo[off] = f32_to_bf16(kr - bf16_to_f32(kb));   // what the stored bf16 key lost; the 32-key tiles add it back
                A.Kh[off] = f32_to_f16_bits(kr);
                if (A.win_rows) {   // ring slot of key t-1; only this wavefront reads it back
                    const size_t ring = (size_t)(u / G) * A.win_rows;
                    const size_t slot = ring + ((t - 1) & (A.win_rows - 1));
                    win_k[slot * (kHeadDim + 4) + lane] = kr;
                    win_v[slot * kHeadDim + lane] = vb;
                    // The transposed value copy is written from the ring: 32 positions of a head dimension at a time (one
                    // 64-byte run per lane) when key t-1 completes a group of 32 - before any tile reads them, the first
                    // block that contains key t-1 closes at t - and the last, incomplete group two bytes at a time at the
                    // end.  (One 2-byte store per lane and position cost a 64-byte write each: 0.93 GB of the 3.28 GB this
                    // kernel wrote per cfg3 call, measured with the stores taken out.)
                    if ((t & 31) == 0) {
                        uint32_t w[16];
#pragma unroll
                        for (int j = 0; j < 16; ++j) {
                            const size_t s0 = ring + ((t - 32 + 2 * j) & (A.win_rows - 1)), s1 = ring + ((t - 31 + 2 * j) & (A.win_rows - 1));
                            w[j] = (uint32_t)win_v[s0 * kHeadDim + lane] | ((uint32_t)win_v[s1 * kHeadDim + lane] << 16);
                        }
                        bf16_t *dst = A.VT + ((size_t)u * kHeadDim + lane) * A.vt_stride + (t - 32);
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            *reinterpret_cast<uint4 *>(dst + 8 * j) = make_uint4(w[4 * j], w[4 * j + 1], w[4 * j + 2], w[4 * j + 3]);
                    } else if (t == A.N) {
                        for (int k = t & ~31; k < t; ++k)
                            A.VT[((size_t)u * kHeadDim + lane) * A.vt_stride + k] = win_v[(ring + (k & (A.win_rows - 1))) * kHeadDim + lane];
                    }
                }
            }
        }
        RT_ABORT_IF(fail);
        if (t == A.N) break;
        RT_STAMP(1);

        // ================================================================ cross-block items of the block ending at key t-1
        if (t >= A.p_min && t < A.N - 1 && (t & -t) >= A.p_min) {
            const int P = t & -t;
            const int nq = min(P, A.N - 1 - t);
            const int qblocks = (nq + 31) / 32;
            const int items = BH * qblocks;
            int level = A.log2_pmin;
            while ((1 << level) < P) ++level;
            if (P < kGlobalP) {
                // Small blocks stay inside the workgroup that owns the (b, h): all their keys and values were stored by
                // its merge wavefront, the partial states will be read by its own helper wavefront, so no other
                // workgroup is involved and no grid barrier is needed (a grid barrier with its fences and the cold
                // misses behind it costs about 30 us, the 128-key tile a few).  The other workgroups already have a_t
                // and go on with phase O.
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                __syncthreads();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                for (int w = 0; w < A.upw; ++w) {
                    const int bh = wg + G * w;   // workgroup-uniform
                    if (bh >= BH) break;
                    if (P >= kKC) {   // nq <= P < kGlobalP <= 32 kPW: one pass covers all queries
                        cross_tile_item<ALIBI>(A, bh, t, P, wave * 32, nq, level, reinterpret_cast<unsigned char *>(act_s));
                        __syncthreads();
                    } else if (wave * 32 < nq) {
                        if (ALIBI)
                            cross_mfma_wave<true, true>(A.Q, A.Qf, A.K, A.Klo, A.VT, A.vt_stride, A.pm, A.pl, A.po, BH, bh, t, 1,
                                                        t - P, P, wave * 32, nq, level, level - A.log2_pmin, A.slots, A.scale,
                                                        alibi_slope(A.alibi, bh % A.H, A.H));
                        else
                        cross_mfma_wave<true>(A.Q, A.Qf, A.K, A.Klo, A.VT, A.vt_stride, A.pm, A.pl, A.po, BH, bh, t, 1, t - P, P,
                                              wave * 32, nq, level, level - A.log2_pmin, A.slots, A.scale);
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                __syncthreads();
                RT_STAMP(14);
                RT_STAMP(15);
            } else {
            if (grid_barrier(A, (++nbar) * (unsigned long long)G, flag_s)) { fail = 1; }
            RT_ABORT_IF(fail);
            RT_STAMP(14);
            if (P >= kKC) {
                // blocks of 64 keys and more: the whole workgroup takes one (b, h) and up to 256 queries at a time,
                // with the key and value tiles staged in the LDS area that the phases use for staged activations
                // and pre-fetched merge inputs (both idle between phase M and phase O)
                const int qgroups = (nq + 32 * kPW - 1) / (32 * kPW);
                for (int it = wg; it < BH * qgroups; it += G) {
                    const int bh = it % BH, qg = it / BH;
                    cross_tile_item<ALIBI>(A, bh, t, P, qg * 32 * kPW + wave * 32, nq, level, reinterpret_cast<unsigned char *>(act_s));
                    __syncthreads();   // the next item overwrites the tiles
                }
            } else {
                for (int it = wave * G + wg; it < items; it += G * kPW) {
                    const int bh = it % BH, qb = it / BH;
                    if (ALIBI)
                        cross_mfma_wave<true, true>(A.Q, A.Qf, A.K, A.Klo, A.VT, A.vt_stride, A.pm, A.pl, A.po, BH, bh, t, 1, t - P, P,
                                                    qb * 32, nq, level, level - A.log2_pmin, A.slots, A.scale,
                                                    alibi_slope(A.alibi, bh % A.H, A.H));
                    else
                    cross_mfma_wave<true>(A.Q, A.Qf, A.K, A.Klo, A.VT, A.vt_stride, A.pm, A.pl, A.po, BH, bh, t, 1, t - P, P, qb * 32,
                                          nq, level, level - A.log2_pmin, A.slots, A.scale);
                }
            }
            RT_STAMP(15);
            if (grid_barrier(A, (++nbar) * (unsigned long long)G, flag_s)) { fail = 1; }
            RT_ABORT_IF(fail);
            }
        }
        RT_STAMP(2);

        // ================================================================ phase O:  h = x_t + alpha Wo a
        RT_STAMP(7);
        wg_gemv_ll<KSD, 32>(wo_s, A.ldw_d, o_n, A.a_ll + par * half_d, B, tag, A, red, act_s, A.ldw_d, fail, nullptr, A.ps_o);
        RT_ABORT_IF(fail);
        RT_STAMP(8);
        if (tid < kRMax * kBMax) {
            float hv = 0.f;
            const int o = o_lo + erow;
            if (erow < o_n && eb < B) hv = sq[erow * kBMax + eb] + A.alpha * red_sum(red, erow, eb);
            const float hn = next_row(hv);
            if (!(erow & 1) && erow < o_n && eb < B)
                ll_store(A.h_ll + par * half_d + pair_word<RO / 2>(o, eb), tag,
                         (unsigned)f32_to_bf16(hv) | ((unsigned)f32_to_bf16(hn) << 16));
            h_loc[erow * kBMax + eb] = hv;
        }
        __syncthreads();
        RT_STAMP(3);

        // ================================================================ phase 1:  u = gelu(rinv_h * W1 h)
        wg_gemv_ll<KSD, RO / 2, true>(w1_s, A.ldw_d, f_n, A.h_ll + par * half_d, B, tag, A, red, act_s, A.ldw_d, fail, sq, A.ps_1);
        RT_ABORT_IF(fail);
        RT_STAMP(11);
        RT_STAMP(12);
        if (tid < kRMax * kBMax) {
            float uv = 0.f;
            if (erow < f_n && eb < B) {
                float s = 0.f;   // |h|^2 of batch row eb from the values this workgroup just received, one part per wavefront
#pragma unroll
                for (int w = 0; w < kPW; ++w) s += sq[w * kBMax + eb];
                const float rinv = A.norm_free ? 1.f : rsqrtf(s / (float)d + A.eps);
                uv = gelu_bf16_out(red_sum(red, erow, eb) * rinv);   // u crosses the chip as bf16
            }
            const float un = next_row(uv);
            if (!(erow & 1) && erow < f_n && eb < B)
                ll_store(A.u_ll + par * half_F + pair_word<R1 / 2>(f_lo + erow, eb), tag,
                         (unsigned)f32_to_bf16(uv) | ((unsigned)f32_to_bf16(un) << 16));
        }
        __syncthreads();
        RT_STAMP(4);

        // ================================================================ phase 2a:  partial W2 u over contraction block jb
        RT_STAMP(9);
        wg_gemv_ll<KSD, R1 / 2>(w2_s, A.ldw_d, RB, A.u_ll + par * half_F + (size_t)jb * (kBMax * (d / 2)), B, tag, A, red, act_s,
                                A.ldw_d, fail, nullptr, A.ps_2a);
        RT_ABORT_IF(fail);
        RT_STAMP(10);
        if (tid < kRMax * kBMax && erow < RB && eb < B)
            ll_store(A.zp_ll + ((size_t)(par * 4 + jb) * kBMax + eb) * d + rb * RB + erow, tag,
                     __float_as_uint(red_sum(red, erow, eb)));
        __syncthreads();
        RT_STAMP(13);

        // ================================================================ phase 2b:  z = h + alpha (sum of the four partials)
        if (is_helper && t + 1 < A.N) {   // wavefronts 4.. are idle in this phase
            PreLoad L;
            float *slot = pre_s + (size_t)help_slot * kPreFloats;
            if (early) {   // combine what phase M fetched; the window holds key t-1 since phase M
                float rq, rm, rl, ro;
                pre_from_lds(slot, L);
                pre_finish<ALIBI>(A, t + 1, help_u, L, help_wk, help_wv, rq, rm, rl, ro);
                slot[lane] = rq; slot[64 + lane] = rm; slot[128 + lane] = rl; slot[192 + lane] = ro;
            } else {       // fetch the next position's merge inputs
                pre_issue(A, t + 1, help_u, L);
                pre_to_lds(L, slot);
            }
        }
        if (tid < kRMax * kBMax) {   // four full wavefronts
            float zv = 0.f, zg = 0.f;
            const int o = o_lo + erow;
            const bool own = erow < o_n && eb < B;
            const ll_t *pp[4];
            bool act[4];
            ll_t w4[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                act[j] = own;
                pp[j] = A.zp_ll + ((size_t)(par * 4 + j) * kBMax + (own ? eb : 0)) * d + (own ? o : 0);
            }
            ll_wait_n<4>(pp, act, tag, A, w4, fail);
            if (own) {
                const float acc = (__uint_as_float((unsigned)w4[0]) + __uint_as_float((unsigned)w4[1])) +
                                  (__uint_as_float((unsigned)w4[2]) + __uint_as_float((unsigned)w4[3]));
                zv = h_loc[erow * kBMax + eb] + A.alpha * acc;
                A.y[((size_t)eb * A.N + t) * d + o] = f32_to_bf16(zv);
                zg = zv;   // the gain of RMS(z) is folded into the stationary Wk, Wv
            }
            const float zn = next_row(zg);
            if (!(erow & 1) && own)
                ll_store(A.z_ll + par * half_d + pair_word<RO / 2>(o, eb), tag,
                         (unsigned)f32_to_bf16(zg) | ((unsigned)f32_to_bf16(zn) << 16));
            sq[erow * kBMax + eb] = zv * zv;
        }
        RT_ABORT_IF(fail);
        if (tid < kBMax) {
            float s = 0.f;
#pragma unroll
            for (int r = 0; r < kRMax; ++r) s += sq[r * kBMax + tid];
            if (tid < B) ll_store(A.zss_ll + par * sz_ss + (size_t)wg * kBMax + tid, tag, __float_as_uint(s));
        }
        __syncthreads();
        RT_STAMP(5);

        // ================================================================ phase KV:  [Wk; Wv] (z g_kv)
        const bool pre = has_u && t + 1 < A.N;
        wg_gemv_ll<KSD, RO / 2>(wkv_s, A.ldw_d, kv_n, A.z_ll + par * half_d, B, tag, A, red, act_s, A.ldw_d, fail, nullptr, A.ps_kv);
        RT_ABORT_IF(fail);
        if (tid < kRMax * kBMax && erow < kv_n && eb < B)
            ll_store(A.kv_ll + par * sz_kv + single_word<RKV>(kv_lo + erow, eb), tag, __float_as_uint(red_sum(red, erow, eb)));
        if (pre) {
            const float *slot = pre_s + (size_t)wave * kPreFloats;
            if (early) {   // finished by the helper in phase 2b
                cq = slot[lane]; cm = slot[64 + lane]; cl = slot[128 + lane]; co = slot[192 + lane];
            } else {       // overlaps the raw k, v crossing the chip
                PreLoad L;
                pre_from_lds(slot, L);
                pre_finish<ALIBI>(A, t + 1, my_u, L, my_wk, my_wv, cq, cm, cl, co);
            }
        }
        __syncthreads();
        RT_STAMP(6);
    }
}

// =============================================================================================
// Host side
// =============================================================================================
// a captured stream must not record memset nodes: clear the counters with a kernel
__global__ void clear_words_kernel(unsigned long long *p, int n)
{
    if ((int)threadIdx.x < n) p[threadIdx.x] = 0ULL;
}

__global__ void clear_slab_kernel(unsigned long long *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0ULL;
}

typedef void (*persist_fn)(PersistArgs);
static persist_fn pick_kernel(int d, int F, bool alibi)
{
    if (d % (32 * kPW) != 0 || F != 4 * d) return nullptr;
    switch (d / (32 * kPW)) {
    case 1: return alibi ? persistent_kernel<1, 4, true> : persistent_kernel<1, 4>;
    case 2: return alibi ? persistent_kernel<2, 8, true> : persistent_kernel<2, 8>;
    case 3: return alibi ? persistent_kernel<3, 12, true> : persistent_kernel<3, 12>;
    case 4: return alibi ? persistent_kernel<4, 16, true> : persistent_kernel<4, 16>;
    default: return nullptr;
    }
}

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

static size_t lds_bytes_for(int d, int F, int G, int win_rows, int upw, int max_batch, int *R_o, int *R_1, int *R_kv)
{
    // rows per workgroup, rounded up to even so that a bf16 pair never straddles two producers
    *R_o = 2 * ((d + 2 * G - 1) / (2 * G));
    *R_1 = 2 * ((F + 2 * G - 1) / (2 * G));
    *R_kv = 2 * ((2 * d + 2 * G - 1) / (2 * G));
    const size_t ldw_d = d + 8;
    (void)F;
    size_t b = ((size_t)*R_o * ldw_d + (size_t)*R_1 * ldw_d + (size_t)(d / 64) * ldw_d + (size_t)*R_kv * ldw_d) * 2;
    b = align_up(b, 16);
    b += (size_t)(kPW * kRMax * kBMax + kRMax * kBMax + 32 * kBMax + kBMax) * 4 + 16;
    b += (size_t)upw * win_rows * ((kHeadDim + 4) * 4 + kHeadDim * 2);   // direct-window rows (fp32 keys, bf16 values)
    b = align_up(b, 16);
    size_t tail = (size_t)max_batch * ldw_d * 2;       // staged activation rows of the phase in flight
    tail += (size_t)upw * kPreFloats * 4;              // pre-fetched merge inputs
    const size_t tiles = (size_t)cross_tile_lds_bytes<true>();   // the cross-block tiles reuse the same area
    b += tail > tiles ? tail : tiles;
    return b;
}

rt_status persistent_create(PersistentState &P, const rt_config &cfg, const LayerDims &D)
{
    P.available = false;
    if (cfg.dtype != RT_BF16 || (cfg.flags & RT_FLAG_NO_MFMA)) return RT_ERR_UNSUPPORTED;
    persist_fn fn = pick_kernel(D.d, D.F, D.alibi > 0.f);   // d in {256, 512, 768, 1024}, F = 4 d
    if (!fn) return RT_ERR_UNSUPPORTED;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, cfg.device) != hipSuccess) return RT_ERR_HIP;
    if (!prop.cooperativeLaunch) return RT_ERR_UNSUPPORTED;
    const int G = prop.multiProcessorCount;
    if (G != 256) return RT_ERR_UNSUPPORTED;   // W2 is laid out as 64 row blocks x 4 contraction blocks of workgroups
    int R_o, R_1, R_kv;
    P.upw = ((cfg.max_batch < kBMax ? cfg.max_batch : kBMax) * D.H + G - 1) / G;
    P.max_batch = cfg.max_batch < kBMax ? cfg.max_batch : kBMax;   // larger batches take the per-position engine
    if (P.upw > 4 || (cfg.max_batch < kBMax ? cfg.max_batch : kBMax) * D.H > 256) return RT_ERR_UNSUPPORTED;
    P.win_rows = D.p_min <= 64 ? D.p_min : 0;
    const size_t lds = lds_bytes_for(D.d, D.F, G, P.win_rows, P.upw, P.max_batch, &R_o, &R_1, &R_kv);
    if (R_o > kRMax || R_1 > kRMax || R_kv > kRMax) return RT_ERR_UNSUPPORTED;
    if (lds > (size_t)160 * 1024) return RT_ERR_UNSUPPORTED;
    if (hipFuncSetAttribute((const void *)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) !=
        hipSuccess) {
        (void)hipGetLastError();
        return RT_ERR_UNSUPPORTED;
    }
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, fn, kPThreads, lds) != hipSuccess || nb < 1) {
        (void)hipGetLastError();
        return RT_ERR_UNSUPPORTED;
    }
    P.num_cu = G;
    P.grid = G;
    P.lds_bytes = lds;

    const bool want_trace = getenv("RT_PERSIST_TRACE") != nullptr;
    const size_t d = D.d, F = D.F;
    size_t off = 0;
    auto carve = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    const size_t o_bar = carve(256);
    // exchange words (8 bytes), two parities each
    const size_t o_a = carve(2 * kBMax * (d / 2) * 8), o_h = carve(2 * kBMax * (d / 2) * 8);
    const size_t o_u = carve(2 * kBMax * (F / 2) * 8), o_z = carve(2 * kBMax * (d / 2) * 8);
    const size_t o_kv = carve(2 * kBMax * 2 * d * 8);
    const size_t o_zss = carve((size_t)2 * kBMax * G * 8);
    const size_t o_zp = carve((size_t)2 * 4 * kBMax * d * 8);
    P.exchange_bytes = off;   // counters and exchange words; the trace follows
    const size_t o_tr = want_trace ? carve((size_t)2 * cfg.max_seq * 16 * 8) : 0;
    P.slab_bytes = off;
    if (hipMalloc(&P.slab, P.slab_bytes) != hipSuccess) {
        (void)hipGetLastError();
        P.slab = nullptr;
        P.slab_bytes = 0;
        return RT_ERR_OOM;
    }
    if (hipMemset(P.slab, 0, P.slab_bytes) != hipSuccess) {
        (void)hipFree(P.slab);
        P.slab = nullptr;
        return RT_ERR_HIP;
    }
    char *p = (char *)P.slab;
    P.bar = (unsigned long long *)(p + o_bar);
    P.a_ll = p + o_a; P.h_ll = p + o_h; P.u_ll = p + o_u; P.z_ll = p + o_z;
    P.kv_ll = p + o_kv; P.zss_ll = p + o_zss; P.zp_ll = p + o_zp;
    P.trace = want_trace ? (unsigned long long *)(p + o_tr) : nullptr;
    P.trace_rows = want_trace ? cfg.max_seq : 0;
    const char *sl = getenv("RT_SPIN_LIMIT");
    P.spin_limit = sl ? atoll(sl) : (1LL << 21);
    if (P.spin_limit < 1) P.spin_limit = 1;
    P.available = true;
    return RT_OK;
}

void persistent_destroy(PersistentState &P)
{
    if (P.slab) (void)hipFree(P.slab);
    P.slab = nullptr;
    P.available = false;
}

size_t persistent_bytes(const PersistentState &P) { return P.slab ? P.slab_bytes : 0; }

bool persistent_supported(const PersistentState &P, const LayerDims &D)
{
    return P.available && D.B <= P.max_batch && D.N >= 1 && D.N < (1 << 20) - 2 && D.p_min >= 32;
}

rt_status persistent_prefill(PersistentState &P, const LayerDims &D, const Weights &W, const Scratch &S, const void *x,
                             void *y, void *K, void *V, hipStream_t st, std::string &err)
{
    PersistArgs A;
    A.B = D.B; A.N = D.N; A.d = D.d; A.H = D.H; A.F = D.F; A.BH = D.B * D.H;
    A.p_min = D.p_min; A.log2_pmin = D.log2_pmin;
    A.alpha = D.alpha; A.scale = D.scale; A.eps = D.eps; A.norm_free = D.norm_free;
    A.G = P.grid;
    (void)lds_bytes_for(D.d, D.F, P.grid, P.win_rows, P.upw, P.max_batch, &A.R_o, &A.R_1, &A.R_kv);
    A.win_rows = P.win_rows; A.upw = P.upw; A.max_batch = P.max_batch;
    A.ldw_d = D.d + 8; A.ldw_F = D.F + 8;
    A.Wo = (const bf16_t *)W.Wo; A.W1 = (const bf16_t *)W.W1; A.W2 = (const bf16_t *)W.W2;
    A.Wk = (const bf16_t *)W.Wk; A.Wv = (const bf16_t *)W.Wv;
    A.g_mlp = (const bf16_t *)W.g_mlp; A.g_kv = (const bf16_t *)W.g_kv; A.g_k = (const bf16_t *)W.g_k;
    A.x = (const bf16_t *)x; A.y = (bf16_t *)y; A.K = (bf16_t *)K; A.V = (bf16_t *)V;
    A.Q = (const bf16_t *)S.Q; A.Kt = (const bf16_t *)S.Kt; A.Vt = (const bf16_t *)S.Vt;
    A.Qf = S.Qf; A.Ktf = S.Ktf; A.Klo = S.Klo; A.Kh = S.Kh;
    A.VT = S.VT; A.vt_stride = S.vt_stride;
    A.pm = S.pm; A.pl = S.pl; A.po = S.po; A.levels = S.levels; A.slots = S.slots;
    A.a_ll = (ll_t *)P.a_ll; A.h_ll = (ll_t *)P.h_ll; A.u_ll = (ll_t *)P.u_ll; A.z_ll = (ll_t *)P.z_ll;
    A.kv_ll = (ll_t *)P.kv_ll; A.zss_ll = (ll_t *)P.zss_ll; A.zp_ll = (ll_t *)P.zp_ll;
    A.R_2 = D.d / 64;
    A.bar = P.bar; A.trace = P.trace; A.spin_limit = P.spin_limit;
    A.trace_rows = P.trace_rows;
    // Waits before the first poll of the pulls of phases O, 1, 2a, KV in units of 4 x 64 clocks (0.1 us): a poll that leaves
    // before the producers' stores have landed costs a whole extra trip.  Measured at cfg3 (ms per call, units of 0.2 us):
    // 1,1,1,1 31.45; 1,2,1,1 30.80; 2,2,1,1 30.76; 2,2,1,0 30.5; 3,2,1,0 30.84; 2,3,1,0 30.91; 1,1,0,1 32.7; 1,1,1,2 31.8.
    // In units of 0.1 us: 4,4,2,0 30.2; 3,4,2,0 30.07; 5,4,2,0 30.43; 4,3,2,0 30.3; 4,4,1,0 30.6; 4,4,2,1 30.3.
    // RT_PRE_SLEEPS (four digits) or RT_PRE_SLEEP (one number for all four) override them.
    A.pre_sleep = getenv("RT_PRE_SLEEP") ? atoi(getenv("RT_PRE_SLEEP")) : 2;
    {
        const char *ps = getenv("RT_PRE_SLEEPS");
        const bool ok = ps && strlen(ps) == 4;
        const bool one = getenv("RT_PRE_SLEEP") != nullptr;
        A.ps_o = ok ? ps[0] - '0' : (one ? A.pre_sleep : 3);
        A.ps_1 = ok ? ps[1] - '0' : (one ? A.pre_sleep : 4);
        A.ps_2a = ok ? ps[2] - '0' : (one ? A.pre_sleep : 2);
        A.ps_kv = ok ? ps[3] - '0' : (one ? A.pre_sleep : 0);
    }
    A.early_premerge = (getenv("RT_EARLY_PREMERGE") ? atoi(getenv("RT_EARLY_PREMERGE")) : 1) && P.win_rows != 0;
    {
        const char *tw = getenv("RT_PERSIST_TRACE_WG");
        A.trace_wg = tw ? atoi(tw) : P.grid - 1;
    }
    P.nonce = (P.nonce % 4095u) + 1u;          // 1..4095; fresh buffers hold tag 0
    A.tag_base = P.nonce << 20;
    if (P.nonce == 1u && P.launched) {
        // the nonce has wrapped: words left by a call 4095 calls ago (rows of a larger batch, positions of a longer
        // sequence) could carry this call's tags.  Start over from cleared buffers.
        hipLaunchKernelGGL(clear_slab_kernel, dim3(256), dim3(256), 0, st, (unsigned long long *)P.slab, P.exchange_bytes / 8);
        hipError_t ce = hipGetLastError();
        if (ce != hipSuccess) { err = std::string("clear_slab_kernel: ") + hipGetErrorString(ce); return RT_ERR_HIP; }
    }

    hipLaunchKernelGGL(clear_words_kernel, dim3(1), dim3(64), 0, st, P.bar, 32);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { err = std::string("clear_words_kernel: ") + hipGetErrorString(e); return RT_ERR_HIP; }
    void *args[] = {&A};
    A.alibi = D.alibi;
    e = hipLaunchCooperativeKernel((const void *)pick_kernel(D.d, D.F, D.alibi > 0.f), dim3(P.grid), dim3(kPThreads), args,
                                   (unsigned int)P.lds_bytes, st);
    if (e != hipSuccess) { err = std::string("hipLaunchCooperativeKernel: ") + hipGetErrorString(e); return RT_ERR_HIP; }
    P.launched = true;
    return RT_OK;
}

int persistent_wait_expired(PersistentState &P)
{
    if (!P.slab || !P.launched) return 0;
    unsigned long long v = 0;
    if (hipMemcpy(&v, P.bar + 8, sizeof(v), hipMemcpyDeviceToHost) != hipSuccess) return -1;
    return v != 0 ? 1 : 0;
}

int persistent_read_trace(PersistentState &P, unsigned long long *out, int rows)
{
    if (!P.trace || !out) return 0;
    const int n = rows < 2 * P.trace_rows ? rows : 2 * P.trace_rows;
    if (hipMemcpy(out, P.trace, (size_t)n * 16 * 8, hipMemcpyDeviceToHost) != hipSuccess) return -1;
    return n;
}

}  // namespace rt
