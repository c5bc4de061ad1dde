// Single-launch decoding step (paper Sec. 7.3: one position of the recurrence of Sec. 2.2 over a cache of persistent
// pairs), bf16 storage.
//
// One grid of 256 workgroups (one per compute unit) x 512 threads evaluates the whole position:
//
//   Q    raw [q | k_tmp | v_tmp] = [Wq; Wk; Wv]' x_t / rms(x_t): 3d / 256 rows per workgroup                  -> raw q, k, v
//   A    attention over the cache rows 0 .. t-1: the 64-key chunks of one (b, h) are dealt to the wavefronts of the
//        S = 256 / (B H) workgroups that share it; every wavefront keeps a running softmax state (Appendix C,
//        Algorithm 2 for one query row), the eight states of a workgroup are combined in LDS                   -> S partial states
//   M    one wavefront per (b, h): the partial states and the temporary pair                                   -> a
//   O, 1, 2a, 2b, KV   the base case exactly as in the single-launch prefill engine (rt_persistent.hip): every
//        workgroup holds its rows of Wo, W1, [Wk; Wv] and its block of W2 in LDS, the vectors between the products
//        cross the chip in self-validating words (rt_ll.h)                                                     -> y_t, raw k, v
//   F    one wavefront per (b, h): RMS scale of z, qkRMS of k, the cache row t of K and V
//
// The multi-launch step spends most of its time in the start-up and tail of eight dependent kernels that move 2-8 MB
// each.  Here every byte the step needs - the cache rows (2 t B d elements) and all six matrices (12 d^2) - is requested
// early in the launch by the workgroup that will use it (none of it depends on a result of the step; the order of the
// requests - phase Q's rows, a first chunk per wavefront, the second chunk, the other weight slices - follows the
// order of use, because a wavefront gets its loads back in the order it issued them), and the dependent part that
// follows is seven exchanges of small vectors.
// RMS gains are folded into the rows as they are copied to LDS (W diag(g), rounded once), as in the prefill engine.
// Every wait is bounded (spin limit -> abort word -> every workgroup leaves).
#include "rt_decode_persistent.h"
#include "rt_ll.h"

#include <cstdlib>

namespace rt {

constexpr int kDecMaxSplit = 16;   // workgroups that can share the cache rows of one (b, h)
constexpr int kPartWords = 72;     // words of an exchanged partial state: o[64], m, l, padded to whole 64-byte lines
constexpr int kPartLds = 68;       // floats of a wavefront's state in LDS

struct DecArgs {
    int B, d, H, F, BH, G, t;
    int S;                         // workgroups per (b, h) in the attention phase
    float alpha, scale, eps, alibi;
    int norm_free;
    int R_q, R_o, R_1, R_kv, R_2, ldw, max_batch;
    const bf16_t *Wq, *Wk, *Wv, *Wo, *W1, *W2, *g_attn, *g_mlp, *g_kv, *g_q, *g_k;
    const bf16_t *x;               // [B][d]
    bf16_t *y;                     // [B][d]
    bf16_t *K, *V;                 // [kv_cap][B][H][64]: rows 0 .. t-1 read, row t written
    size_t kv_rs;                  // elements between cache rows: B H 64, or the whole batch's when this call is a chunk of it
    ll_t *qkv_ll;                  // [3d] x kBMax, one fp32 per word
    ll_t *part_ll;                 // [B H][kDecMaxSplit][kPartWords]
    ll_t *a_ll, *h_ll, *z_ll;      // [kBMax][d/2]   two bf16 per word
    ll_t *u_ll;                    // [kBMax][F/2]
    ll_t *kv_ll;                   // [kBMax][2d]    one fp32 per word
    ll_t *zss_ll;                  // [G][kBMax]
    ll_t *zp_ll;                   // [4][kBMax][d]
    unsigned tag;
    unsigned long long *bar;       // [0] unused, [8] abort word
    long long spin_limit;
    int pre_sleep;
    unsigned long long *trace;     // optional: [G][16] 100 MHz clock stamps of every workgroup's phases
};

#define RT_DEC_STAMP(k)                                                              \
    do {                                                                             \
        if (A.trace && threadIdx.x == 0) A.trace[(size_t)blockIdx.x * 16 + (k)] = wall_clock64(); \
    } while (0)

// Workgroup barrier behind which every wavefront leaves when any of them has given up waiting: that wavefront raises an LDS
// flag before the barrier, all read it behind the barrier (it is never lowered again).  One barrier and one LDS read instead
// of a workgroup-wide reduction of the predicate (two barriers and LDS atomics).
#define RT_DEC_ABORT_IF(cond)                                                                                           \
    do {                                                                                                                \
        if (cond) gave_up_s = 1;                                                                                        \
        __syncthreads();                                                                                                \
        if (gave_up_s != 0) {                                                                                           \
            if (threadIdx.x == 0) __hip_atomic_store(A.bar + 8, 1ULL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);     \
            return;                                                                                                     \
        }                                                                                                               \
    } while (0)

// The 64 cache rows k_lo .. k_lo + cnt - 1 of one (b, h): 16 KB requested at once.  Piece i of a lane is row
// 8 i + lane / 8, columns 8 (lane % 8) .. + 7 (eight lanes cover one 128-byte row); rows past the end repeat the last.
__device__ __forceinline__ void dec_load_chunk(const bf16_t *K, const bf16_t *V, size_t rs, int u, int k_lo, int cnt, uint4 (&kr)[8],
                                               uint4 (&vr)[8])
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const size_t off = (size_t)(k_lo + min(8 * i + (lane >> 3), cnt - 1)) * rs + (size_t)u * kHeadDim + (lane & 7) * 8;
        kr[i] = global_load16(K + off);
        vr[i] = global_load16(V + off);
    }
}

// One chunk folded into a wavefront's running state (Appendix C, Algorithm 2, one query row): m, l wave-uniform,
// o8 this lane's share of the output (its eight columns over the rows it holds; the lanes that share columns are
// summed once, after the last chunk).  q8: the query's elements at this lane's columns.  dist_first: distance of the
// chunk's first key from the query (ALiBi).
// The logit of row 8 i + lane / 8 is summed over the eight lanes of the row with three DPP steps and stays in all
// eight of them (register i), which is where the softmax weight is needed for the value rows: no value crosses the
// LDS crossbar.  (With the logits gathered to one key per lane - four dependent ds_bpermute per piece and one more
// per value piece - a chunk took 2 us of a wavefront's time.)  Every weight is computed by the eight lanes of its
// row, so the row sum over all lanes counts it eight times.
__device__ __forceinline__ void dec_attend_chunk(const uint4 (&kr)[8], const uint4 (&vr)[8], const float (&q8)[8], int cnt,
                                                 int dist_first, float scale, float slope, float &m, float &l, float (&o8)[8])
{
    const int lane = threadIdx.x & 63, r8 = lane >> 3;
    float sc[8];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t w[4] = {kr[i].x, kr[i].y, kr[i].z, kr[i].w};
        float dsum = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            dsum = fmaf(q8[2 * e], __uint_as_float(w[e] << 16), dsum);
            dsum = fmaf(q8[2 * e + 1], __uint_as_float(w[e] & 0xFFFF0000u), dsum);
        }
        dsum += dpp_f(dsum, 0);
        dsum += dpp_f(dsum, 1);
        dsum += dpp_f(dsum, 2);   // all eight lanes of the row hold its sum
        const int j = 8 * i + r8;
        sc[i] = j < cnt ? fmaf(-slope, (float)(dist_first - j), dsum * scale) : -INFINITY;
        mx = fmaxf(mx, sc[i]);
    }
    const float m_new = fmaxf(m, fast_max(mx));
    const float resc = __expf(m - m_new);   // exp(-inf) = 0 on the first chunk
    float psum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) o8[e] *= resc;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float pr = __expf(sc[i] - m_new);   // exp(-inf) = 0 for rows past the end
        psum += pr;
        const uint32_t w[4] = {vr[i].x, vr[i].y, vr[i].z, vr[i].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            o8[2 * e] = fmaf(pr, __uint_as_float(w[e] << 16), o8[2 * e]);
            o8[2 * e + 1] = fmaf(pr, __uint_as_float(w[e] & 0xFFFF0000u), o8[2 * e + 1]);
        }
    }
    l = l * resc + fast_sum(psum) * 0.125f;
    m = m_new;
}

// two softmax states into one; an empty state has m = -inf, l = 0
__device__ __forceinline__ void dec_combine(float &m, float &l, float &o, float m2, float l2, float o2)
{
    if (m2 == -INFINITY) return;   // wave-uniform
    const float m_new = fmaxf(m, m2);
    const float e1 = __expf(m - m_new), e2 = __expf(m2 - m_new);
    l = l * e1 + l2 * e2;
    o = o * e1 + o2 * e2;
    m = m_new;
}

// KSD = d / 256.
template <int KSD>
__global__ __launch_bounds__(kPThreads) void decode_coop_kernel(DecArgs A)
{
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int gave_up_s;   // raised by a wavefront whose bounded wait ran out; the first barrier below precedes its first use
    if (threadIdx.x == 0) gave_up_s = 0;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wg = blockIdx.x, G = A.G;
    const int d = A.d, F = A.F, B = A.B, BH = A.BH, H = A.H, t = A.t;
    constexpr int RQ = 3 * KSD, RO = 2 * ((KSD + 1) / 2), R1 = 4 * KSD, RKV = 2 * KSD;
    constexpr int PER = 32 * KSD;   // 16-byte pieces of a d-long bf16 row
    const unsigned tag = A.tag;

    // ---- LDS carve-up (the five weight slices are contiguous: one copy loop fills the last four)
    bf16_t *wq_s = reinterpret_cast<bf16_t *>(smem);
    bf16_t *wo_s = wq_s + (size_t)A.R_q * A.ldw;
    bf16_t *w1_s = wo_s + (size_t)A.R_o * A.ldw;
    bf16_t *w2_s = w1_s + (size_t)A.R_1 * A.ldw;
    bf16_t *wkv_s = w2_s + (size_t)A.R_2 * A.ldw;
    float *red = reinterpret_cast<float *>(wkv_s + (size_t)A.R_kv * A.ldw);   // [kPW][kRMax][kBMax]
    float *h_loc = red + kPW * kRMax * kBMax;                                 // [kRMax][kBMax]
    float *sq = h_loc + kRMax * kBMax;                                        // [32][kBMax]
    float *rinv_s = sq + 32 * kBMax;                                          // [kBMax]
    float *part_s = rinv_s + kBMax;                                           // [kPW][kPartLds]
    bf16_t *act_s = reinterpret_cast<bf16_t *>(part_s + kPW * kPartLds);      // [max_batch][ldw]

    // ---- this workgroup's rows
    const int q_lo = wg * RQ;                                                          // rows of [Wq; Wk; Wv] (3 d = 256 RQ)
    const int o_lo = min(wg * A.R_o, d), o_n = min(d, o_lo + A.R_o) - o_lo;            // Wo, and the z rows it finishes
    const int f_lo = min(wg * A.R_1, F), f_n = min(F, f_lo + A.R_1) - f_lo;            // W1
    const int kv_lo = min(wg * A.R_kv, 2 * d), kv_n = min(2 * d, kv_lo + A.R_kv) - kv_lo;   // [Wk; Wv]
    const int rb = wg >> 2, jb = wg & 3, RB = A.R_2;                                   // W2: row block x contraction block

    // ---- this wavefront's share of the cache
    const int S = A.S;
    const int u = wg / S, s = wg - u * S;     // (b, h) and split of this workgroup
    const bool att = u < BH;
    const int ub = att ? u / H : 0, uh = att ? u - ub * H : 0;
    const int nch = (t + 63) >> 6;            // chunks of 64 cached keys
    const int nworkers = kPW * S;
    const size_t rs = A.kv_rs;
    const bool is_merger = att && s == 0 && wave == 0;

    RT_DEC_STAMP(0);
    // ---- One straight run of requests: the input rows and this workgroup's rows of [Wq; Wk; Wv] (what phase Q waits
    // for), then the first cache chunk of every wavefront (most of the step's bytes are cache rows: 2 t B d of
    // 2 t B d + 12 d^2; with them in flight from the start the memory system is busy while phase Q runs).  Loads return
    // to a wavefront in the order it issued them, so the few bytes of phase Q must be asked for first: with the chunk
    // ahead of them the rows were staged at 7.5 us instead of 3.  A wavefront without a chunk reads row 0 (unused).
    constexpr int NXB = (kBMax * PER + kPThreads - 1) / kPThreads, NQB = (RQ * PER + kPThreads - 1) / kPThreads;
    const bf16_t *g_in = A.norm_free ? nullptr : A.g_attn;
    uint4 xr[NXB], wr[NQB], gr[NQB];
#pragma unroll
    for (int j = 0; j < NXB; ++j) {
        const int idx = j * kPThreads + tid, r = min(idx / PER, B - 1), c = idx % PER;
        xr[j] = global_load16(A.x + (size_t)r * d + c * 8);
    }
#pragma unroll
    for (int j = 0; j < NQB; ++j) {
        const int idx = j * kPThreads + tid, r = min(idx / PER, RQ - 1), c = idx % PER;
        const int o = q_lo + r, which = o / d, row = o - which * d;
        const bf16_t *Wm = which == 0 ? A.Wq : (which == 1 ? A.Wk : A.Wv);
        wr[j] = global_load16(Wm + (size_t)row * d + c * 8);
        gr[j] = global_load16((g_in ? g_in : A.Wq) + c * 8);   // unconditional: a branch here would end the run of requests
    }
    uint4 krA[8], vrA[8], krB[8], vrB[8];
    int cA = wave * S + s, cB = cA + nworkers;
    {
        const bool hasA = att && cA < nch;
        dec_load_chunk(A.K, A.V, rs, att ? u : 0, hasA ? cA * 64 : 0, hasA ? min(64, t - cA * 64) : 1, krA, vrA);
    }
    // gains of the per-head normalisation of this wavefront's head: requested behind the run above (loads come back in issue
    // order), long before the three places on the critical path that use them
    const float gq_r = (att && A.g_q) ? bf16_to_f32(A.g_q[uh * kHeadDim + lane]) : 1.f;
    const float gk_r = (att && A.g_k) ? bf16_to_f32(A.g_k[uh * kHeadDim + lane]) : 1.f;
    // ================================================================ input rows and the rows of [Wq; Wk; Wv] into LDS
#pragma unroll
    for (int j = 0; j < NXB; ++j) {
        const int idx = j * kPThreads + tid, r = idx / PER, c = idx % PER;
        if (r < B) *reinterpret_cast<uint4 *>(act_s + (size_t)r * A.ldw + c * 8) = xr[j];
    }
#pragma unroll
    for (int j = 0; j < NQB; ++j) {
        const int idx = j * kPThreads + tid, r = idx / PER, c = idx % PER;
        if (r >= RQ) continue;
        uint4 v = wr[j];
        if (g_in) {
            float gg[8], ww[8];
            load8(reinterpret_cast<const bf16_t *>(&gr[j]), gg);
            load8(reinterpret_cast<const bf16_t *>(&v), ww);
            v.x = pack_bf16(ww[0] * gg[0], ww[1] * gg[1]);
            v.y = pack_bf16(ww[2] * gg[2], ww[3] * gg[3]);
            v.z = pack_bf16(ww[4] * gg[4], ww[5] * gg[5]);
            v.w = pack_bf16(ww[6] * gg[6], ww[7] * gg[7]);
        }
        *reinterpret_cast<uint4 *>(wq_s + (size_t)r * A.ldw + c * 8) = v;
    }

    __syncthreads();
    RT_DEC_STAMP(1);

    // ================================================================ phase Q
    const int erow = tid >> 4, eb = tid & 15;   // epilogue thread -> (row, batch row) for tid < 256
    wg_product_staged<KSD, true>(wq_s, A.ldw, RQ, B, red, act_s, A.ldw, sq);
    __syncthreads();
    if (tid < kBMax) {
        float ssum = 0.f;
#pragma unroll
        for (int w = 0; w < kPW; ++w) ssum += sq[w * kBMax + tid];
        rinv_s[tid] = A.norm_free ? 1.f : rsqrtf(ssum / (float)d + A.eps);
    }
    __syncthreads();
    if (tid < kRMax * kBMax && erow < RQ && eb < B)
        ll_store(A.qkv_ll + single_word<RQ>(q_lo + erow, eb), tag, __float_as_uint(red_sum(red, erow, eb) * rinv_s[eb]));
    float xv = 0.f;   // residual input of this workgroup's rows
    if (tid < kRMax * kBMax && erow < o_n && eb < B) xv = bf16_to_f32(A.x[(size_t)eb * d + o_lo + erow]);
    __syncthreads();   // red, sq and the staged rows are reused
    RT_DEC_STAMP(2);
    if (att && cB < nch) dec_load_chunk(A.K, A.V, rs, u, cB * 64, min(64, t - cB * 64), krB, vrB);

    // ================================================================ the other four weight slices
    // Requested (into registers) after this wavefront's first chunk, so that the cache rows, which the step needs first,
    // are served first; stored to LDS before phase O.  The gains of W1's and [Wk; Wv]'s columns wait in the LDS rows
    // that held [Wq; Wk; Wv].
    constexpr int WROWS = RO + R1 + 4 * KSD + RKV;
    constexpr int NBW = (WROWS * PER + kPThreads - 1) / kPThreads;
    const int n1 = A.R_o, n2 = n1 + A.R_1, n3 = n2 + A.R_2, n4 = n3 + A.R_kv;
    const bf16_t *gm = A.norm_free ? nullptr : A.g_mlp, *gkv = A.norm_free ? nullptr : A.g_kv;
    bf16_t *gm_s = wq_s, *gkv_s = wq_s + A.ldw;
    if (tid < 2 * PER) {
        const bf16_t *g = tid < PER ? gm : gkv;
        if (g) *reinterpret_cast<uint4 *>((tid < PER ? gm_s : gkv_s) + (tid % PER) * 8) = global_load16(g + (tid % PER) * 8);
    }
    uint4 wreg[NBW];
    auto weight_row = [&](int r) -> const bf16_t * {
        if (r < n1) return r < o_n ? A.Wo + (size_t)(o_lo + r) * d : nullptr;
        if (r < n2) return r - n1 < f_n ? A.W1 + (size_t)(f_lo + r - n1) * d : nullptr;
        if (r < n3) return A.W2 + (size_t)(rb * RB + r - n2) * F + (size_t)jb * d;
        const int rr = r - n3, o = kv_lo + rr;
        if (rr >= kv_n) return nullptr;
        return o < d ? A.Wk + (size_t)o * d : A.Wv + (size_t)(o - d) * d;
    };
    auto weight_gain = [&](int r) -> const bf16_t * {
        if (r >= n1 && r < n2) return gm ? gm_s : nullptr;
        if (r >= n3) return gkv ? gkv_s : nullptr;
        return nullptr;
    };

    RT_DEC_STAMP(3);
    // ================================================================ phase A: this wavefront's chunks
    int fail = 0;
    float qn = 0.f;
    if (att) {
        const ll_t wq = ll_wait(A.qkv_ll + single_word<RQ>(uh * kHeadDim + lane, ub), true, tag, A, fail);
        qn = __uint_as_float((unsigned)wq);
        if (!A.norm_free)
            qn *= rsqrtf(fast_sum(qn * qn) / (float)kHeadDim + A.eps) * gq_r;
        float q8[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) q8[e] = __shfl(qn, (lane & 7) * 8 + e, 64);
        const float slope = alibi_slope(A.alibi, uh, H);
        float m = -INFINITY, l = 0.f, o8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        while (cA + 2 * nworkers < nch) {   // both chunks in hand have a successor or are followed by one
            dec_attend_chunk(krA, vrA, q8, 64, t - cA * 64, A.scale, slope, m, l, o8);
            cA += 2 * nworkers;
            dec_load_chunk(A.K, A.V, rs, u, cA * 64, min(64, t - cA * 64), krA, vrA);
            dec_attend_chunk(krB, vrB, q8, 64, t - cB * 64, A.scale, slope, m, l, o8);
            cB += 2 * nworkers;
            if (cB < nch) dec_load_chunk(A.K, A.V, rs, u, cB * 64, min(64, t - cB * 64), krB, vrB);
        }
        // the last one or two chunks; the weight rows are requested between them (into the registers of the first)
        if (cA < nch) dec_attend_chunk(krA, vrA, q8, min(64, t - cA * 64), t - cA * 64, A.scale, slope, m, l, o8);
        __builtin_amdgcn_sched_barrier(0);   // the requests below must not move up: their registers are the first chunk's
        rows_issue<NBW, PER>(wreg, n4, weight_row);
        __builtin_amdgcn_sched_barrier(0);
        if (cB < nch) dec_attend_chunk(krB, vrB, q8, min(64, t - cB * 64), t - cB * 64, A.scale, slope, m, l, o8);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            o8[e] += __shfl_xor(o8[e], 8, 64);
            o8[e] += __shfl_xor(o8[e], 16, 64);
            o8[e] += __shfl_xor(o8[e], 32, 64);
        }
        float *ps = part_s + wave * kPartLds;
        if (lane < 8) {
#pragma unroll
            for (int e = 0; e < 8; ++e) ps[lane * 8 + e] = o8[e];
        }
        if (lane == 0) { ps[64] = m; ps[65] = l; }
    } else {
        rows_issue<NBW, PER>(wreg, n4, weight_row);
    }
    RT_DEC_STAMP(4);
    RT_DEC_ABORT_IF(fail);   // also orders the eight states in LDS before wavefront 0 reads them
    RT_DEC_STAMP(5);

    // ================================================================ phase M: partial states -> a
    bool committed = false;   // wavefront-uniform
    if (att && wave == 0) {
        float M = -INFINITY, L = 0.f, O = 0.f;
#pragma unroll
        for (int w = 0; w < kPW; ++w) {
            const float *ps = part_s + w * kPartLds;
            dec_combine(M, L, O, ps[64], ps[65], ps[lane]);
        }
        ll_t *mine = A.part_ll + ((size_t)u * kDecMaxSplit + s) * kPartWords;
        if (s != 0) {
            ll_store(mine + lane, tag, __float_as_uint(O));
            if (lane < 2) ll_store(mine + 64 + lane, tag, __float_as_uint(lane == 0 ? M : L));
        } else {
            // The weight slices go from registers to LDS first: the other workgroups' partial states are still crossing the chip,
            // and the workgroup's barrier before phase O waits for this wavefront.
            rows_commit<NBW, PER>(wreg, wo_s, A.ldw, n4, weight_gain);
            committed = true;
            // the temporary pair of this position (distance 0: no positional bias) and the first partial state in one round
            const ll_t *src1 = A.part_ll + ((size_t)u * kDecMaxSplit + 1) * kPartWords;
            const ll_t *p4[4] = {A.qkv_ll + single_word<RQ>(d + uh * kHeadDim + lane, ub),
                                 A.qkv_ll + single_word<RQ>(2 * d + uh * kHeadDim + lane, ub), src1 + lane, src1 + 64 + (lane & 1)};
            const bool on4[4] = {true, true, S > 1, S > 1};
            const bool on2[2] = {true, true};
            ll_t w4[4];
            ll_wait_n<4>(p4, on4, tag, A, w4, fail);
            float kt = __uint_as_float((unsigned)w4[0]);
            const float vt = bf16_to_f32(f32_to_bf16(__uint_as_float((unsigned)w4[1])));
            if (!A.norm_free)
                kt *= rsqrtf(fast_sum(kt * kt) / (float)kHeadDim + A.eps) * gk_r;
            dec_combine(M, L, O, A.scale * fast_sum(qn * kt), 1.f, vt);
            if (S > 1) {
                const float ml = __uint_as_float((unsigned)w4[3]);
                dec_combine(M, L, O, lane_bcast(ml, 0), lane_bcast(ml, 1), __uint_as_float((unsigned)w4[2]));
            }
            for (int sp = 2; sp < S; ++sp) {
                const ll_t *src = A.part_ll + ((size_t)u * kDecMaxSplit + sp) * kPartWords;
                const ll_t *pp[2] = {src + lane, src + 64 + (lane & 1)};
                ll_t wp[2];
                ll_wait_n<2>(pp, on2, tag, A, wp, fail);
                const float ml = __uint_as_float((unsigned)wp[1]);
                dec_combine(M, L, O, lane_bcast(ml, 0), lane_bcast(ml, 1), __uint_as_float((unsigned)wp[0]));
            }
            const float av = O * __builtin_amdgcn_rcpf(L);   // a crosses the chip as bf16
            const float an = dpp_odd_neighbour(av);
            if (!(lane & 1))
                ll_store(A.a_ll + pair_word<32>(uh * kHeadDim + lane, ub), tag,
                         (unsigned)f32_to_bf16(av) | ((unsigned)f32_to_bf16(an) << 16));
        }
    }
    if (!committed) rows_commit<NBW, PER>(wreg, wo_s, A.ldw, n4, weight_gain);
    RT_DEC_ABORT_IF(fail);
    RT_DEC_STAMP(6);

    // ================================================================ phase O:  h = x_t + alpha Wo a
    wg_gemv_ll<KSD, 32>(wo_s, A.ldw, o_n, A.a_ll, B, tag, A, red, act_s, A.ldw, fail);
    RT_DEC_ABORT_IF(fail);
    if (tid < kRMax * kBMax) {
        float hv = 0.f;
        const int o = o_lo + erow;
        if (erow < o_n && eb < B) hv = xv + A.alpha * red_sum(red, erow, eb);
        const float hn = next_row(hv);
        if (!(erow & 1) && erow < o_n && eb < B)
            ll_store(A.h_ll + pair_word<RO / 2>(o, eb), tag, (unsigned)f32_to_bf16(hv) | ((unsigned)f32_to_bf16(hn) << 16));
        h_loc[erow * kBMax + eb] = hv;
    }
    __syncthreads();
    RT_DEC_STAMP(7);

    // ================================================================ phase 1:  u = gelu(W1' h / rms(h))
    wg_gemv_ll<KSD, RO / 2, true>(w1_s, A.ldw, f_n, A.h_ll, B, tag, A, red, act_s, A.ldw, fail, sq);
    RT_DEC_ABORT_IF(fail);
    if (tid < kRMax * kBMax) {
        float uv = 0.f;
        if (erow < f_n && eb < B) {
            float ssum = 0.f;   // |h|^2 of batch row eb from the values this workgroup just received, one part per wavefront
#pragma unroll
            for (int w = 0; w < kPW; ++w) ssum += sq[w * kBMax + eb];
            const float rinv = A.norm_free ? 1.f : rsqrtf(ssum / (float)d + A.eps);
            uv = gelu_bf16_out(red_sum(red, erow, eb) * rinv);   // u crosses the chip as bf16
        }
        const float un = next_row(uv);
        if (!(erow & 1) && erow < f_n && eb < B)
            ll_store(A.u_ll + pair_word<R1 / 2>(f_lo + erow, eb), tag, (unsigned)f32_to_bf16(uv) | ((unsigned)f32_to_bf16(un) << 16));
    }
    __syncthreads();
    RT_DEC_STAMP(8);

    // ================================================================ phase 2a:  partial W2 u over contraction block jb
    wg_gemv_ll<KSD, R1 / 2>(w2_s, A.ldw, RB, A.u_ll + (size_t)jb * (kBMax * (d / 2)), B, tag, A, red, act_s, A.ldw, fail);
    RT_DEC_ABORT_IF(fail);
    if (tid < kRMax * kBMax && erow < RB && eb < B)
        ll_store(A.zp_ll + ((size_t)jb * kBMax + eb) * d + rb * RB + erow, tag, __float_as_uint(red_sum(red, erow, eb)));
    __syncthreads();
    RT_DEC_STAMP(9);

    // ================================================================ phase 2b:  z = h + alpha (sum of the four partials)
    if (tid < kRMax * kBMax) {
        float zv = 0.f;
        const int o = o_lo + erow;
        const bool own = erow < o_n && eb < B;
        const ll_t *pp[4];
        bool on4[4];
        ll_t w4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            on4[j] = own;
            pp[j] = A.zp_ll + ((size_t)j * kBMax + (own ? eb : 0)) * d + (own ? o : 0);
        }
        ll_wait_n<4>(pp, on4, tag, A, w4, fail);
        if (own) {
            const float acc = (__uint_as_float((unsigned)w4[0]) + __uint_as_float((unsigned)w4[1])) +
                              (__uint_as_float((unsigned)w4[2]) + __uint_as_float((unsigned)w4[3]));
            zv = h_loc[erow * kBMax + eb] + A.alpha * acc;
            A.y[(size_t)eb * d + o] = f32_to_bf16(zv);
        }
        const float zn = next_row(zv);
        if (!(erow & 1) && own)
            ll_store(A.z_ll + pair_word<RO / 2>(o, eb), tag, (unsigned)f32_to_bf16(zv) | ((unsigned)f32_to_bf16(zn) << 16));
        sq[erow * kBMax + eb] = zv * zv;
    }
    RT_DEC_ABORT_IF(fail);
    if (tid < kBMax) {
        float ssum = 0.f;
#pragma unroll
        for (int r = 0; r < kRMax; ++r) ssum += sq[r * kBMax + tid];
        if (tid < B) ll_store(A.zss_ll + (size_t)wg * kBMax + tid, tag, __float_as_uint(ssum));
    }
    __syncthreads();
    RT_DEC_STAMP(10);

    // ================================================================ phase KV:  [Wk'; Wv'] z  (1 / rms(z) applied in F)
    wg_gemv_ll<KSD, RO / 2>(wkv_s, A.ldw, kv_n, A.z_ll, B, tag, A, red, act_s, A.ldw, fail);
    RT_DEC_ABORT_IF(fail);
    if (tid < kRMax * kBMax && erow < kv_n && eb < B)
        ll_store(A.kv_ll + single_word<RKV>(kv_lo + erow, eb), tag, __float_as_uint(red_sum(red, erow, eb)));

    RT_DEC_STAMP(11);
    // ================================================================ phase F: the persistent pair of position t
    if (is_merger) {
        const ll_t *p[6];
        bool on6[6];
        ll_t w6[6];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            on6[i] = i * 64 + lane < G;
            p[i] = A.zss_ll + (size_t)(on6[i] ? i * 64 + lane : 0) * kBMax + ub;
        }
        p[4] = A.kv_ll + single_word<RKV>(uh * kHeadDim + lane, ub);
        p[5] = A.kv_ll + single_word<RKV>(d + uh * kHeadDim + lane, ub);
        on6[4] = on6[5] = true;
        ll_wait_n<6>(p, on6, tag, A, w6, fail);
        float ssum = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (on6[i]) ssum += __uint_as_float((unsigned)w6[i]);
        // |z|^2 and |k|^2 of the raw key are independent reductions; the scales multiply the finished sums
        const float k0 = __uint_as_float((unsigned)w6[4]);
        const float Sz = fast_sum(ssum), Sk = fast_sum(k0 * k0);
        const float rz = A.norm_free ? 1.f : rsqrtf(Sz / (float)d + A.eps);
        const float kr = A.norm_free ? k0 : k0 * gk_r * (rz * rsqrtf(rz * rz * Sk / (float)kHeadDim + A.eps));
        const float vr = __uint_as_float((unsigned)w6[5]) * rz;
        if (!fail) {
            const size_t off = (size_t)t * rs + (size_t)u * kHeadDim + lane;
            A.K[off] = f32_to_bf16(kr);
            A.V[off] = f32_to_bf16(vr);
        }
    }
    RT_DEC_ABORT_IF(fail);
    RT_DEC_STAMP(12);
}

// =============================================================================================
// Host side
// =============================================================================================
namespace {

typedef void (*dec_fn)(DecArgs);
dec_fn pick(int d, int F)
{
    if (d % (32 * kPW) != 0 || F != 4 * d) return nullptr;
    switch (d / (32 * kPW)) {
    case 1: return decode_coop_kernel<1>;
    case 2: return decode_coop_kernel<2>;
    case 3: return decode_coop_kernel<3>;
    case 4: return decode_coop_kernel<4>;
    default: return nullptr;
    }
}

size_t up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Rows {
    int R_q, R_o, R_1, R_kv, R_2;
};
Rows rows_for(int d, int F, int G)
{
    Rows r;
    r.R_q = (3 * d + G - 1) / G;
    r.R_o = 2 * ((d + 2 * G - 1) / (2 * G));
    r.R_1 = 2 * ((F + 2 * G - 1) / (2 * G));
    r.R_kv = 2 * ((2 * d + 2 * G - 1) / (2 * G));
    r.R_2 = d / 64;
    return r;
}
size_t lds_bytes_for(int d, int F, int G, int max_batch)
{
    const Rows r = rows_for(d, F, G);
    const size_t ldw = d + 8;
    size_t b = (size_t)(r.R_q + r.R_o + r.R_1 + r.R_2 + r.R_kv) * ldw * 2;
    b = up(b, 16);
    b += (size_t)(kPW * kRMax * kBMax + kRMax * kBMax + 32 * kBMax + kBMax + kPW * kPartLds) * 4;
    b = up(b, 16);
    b += (size_t)max_batch * ldw * 2;
    return b;
}

// layout of the exchange slab (offsets in bytes)
struct Slab {
    size_t bar, qkv, part, a, h, z, u, kv, zss, zp, trace, total;
};
Slab slab_for(int d, int F, int G)
{
    Slab s;
    size_t off = 0;
    auto carve = [&](size_t bytes) { size_t o = off; off = up(off + bytes, 256); return o; };
    s.bar = carve(256);
    s.qkv = carve((size_t)kBMax * 3 * d * 8);
    s.part = carve((size_t)256 * kDecMaxSplit * kPartWords * 8);
    s.a = carve((size_t)kBMax * (d / 2) * 8);
    s.h = carve((size_t)kBMax * (d / 2) * 8);
    s.z = carve((size_t)kBMax * (d / 2) * 8);
    s.u = carve((size_t)kBMax * (F / 2) * 8);
    s.kv = carve((size_t)kBMax * 2 * d * 8);
    s.zss = carve((size_t)kBMax * G * 8);
    s.zp = carve((size_t)4 * kBMax * d * 8);
    s.trace = carve((size_t)G * 16 * 8);
    s.total = off;
    return s;
}

__global__ void dec_clear_kernel(unsigned long long *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0ULL;
}

}  // namespace

rt_status decode_coop_create(DecodeCoopState &P, const rt_config &cfg, const LayerDims &D)
{
    P.available = false;
    if (cfg.dtype != RT_BF16 || (cfg.flags & (RT_FLAG_NO_MFMA | RT_FLAG_ENGINE_STEPWISE)) || getenv("RT_DECODE_MULTI_LAUNCH"))
        return RT_ERR_UNSUPPORTED;
    dec_fn fn = pick(D.d, D.F);   // d in {256, 512, 768, 1024}, F = 4 d
    if (!fn) return RT_ERR_UNSUPPORTED;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, cfg.device) != hipSuccess) return RT_ERR_HIP;
    if (!prop.cooperativeLaunch || prop.multiProcessorCount != 256) return RT_ERR_UNSUPPORTED;   // W2: 64 x 4 workgroups
    const int G = 256;
    P.max_batch = cfg.max_batch < kBMax ? cfg.max_batch : kBMax;
    if (P.max_batch * D.H > G) P.max_batch = G / D.H;
    if (P.max_batch < 1) return RT_ERR_UNSUPPORTED;
    const Rows r = rows_for(D.d, D.F, G);
    if (r.R_q > kRMax || r.R_o > kRMax || r.R_1 > kRMax || r.R_kv > kRMax || r.R_2 > kRMax) return RT_ERR_UNSUPPORTED;
    const size_t lds = lds_bytes_for(D.d, D.F, G, P.max_batch);
    if (lds + 16 > (size_t)160 * 1024) return RT_ERR_UNSUPPORTED;   // 16: the statically allocated flag word
    if (hipFuncSetAttribute((const void *)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
        (void)hipGetLastError();
        return RT_ERR_UNSUPPORTED;
    }
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, fn, kPThreads, lds) != hipSuccess || nb < 1) {
        (void)hipGetLastError();
        return RT_ERR_UNSUPPORTED;
    }
    const Slab s = slab_for(D.d, D.F, G);
    if (hipMalloc(&P.slab, s.total) != hipSuccess) {
        (void)hipGetLastError();
        P.slab = nullptr;
        return RT_ERR_OOM;
    }
    if (hipMemset(P.slab, 0, s.total) != hipSuccess) {
        (void)hipFree(P.slab);
        P.slab = nullptr;
        return RT_ERR_HIP;
    }
    P.slab_bytes = s.total;
    P.d = D.d;
    P.F = D.F;
    P.grid = G;
    P.lds_bytes = lds;
    const char *sl = getenv("RT_SPIN_LIMIT");
    P.spin_limit = sl ? atoll(sl) : (1LL << 21);
    if (P.spin_limit < 1) P.spin_limit = 1;
    P.nonce = 0;
    P.want_trace = getenv("RT_DECODE_TRACE") != nullptr;
    P.cooperative = getenv("RT_DECODE_COOPERATIVE") != nullptr;
    P.split_override = getenv("RT_DECODE_SPLIT") ? atoi(getenv("RT_DECODE_SPLIT")) : 0;
    P.available = true;
    return RT_OK;
}

void decode_coop_destroy(DecodeCoopState &P)
{
    if (P.slab) (void)hipFree(P.slab);
    P.slab = nullptr;
    P.available = false;
}

size_t decode_coop_bytes(const DecodeCoopState &P) { return P.slab ? P.slab_bytes : 0; }

bool decode_coop_supported(const DecodeCoopState &P, const LayerDims &D) { return P.available && D.B <= P.max_batch; }

rt_status decode_coop_step(DecodeCoopState &P, const LayerDims &D, const Weights &W, const void *x_t, int t, void *y_t, void *K,
                           void *V, hipStream_t st, std::string &err, size_t kv_row_elems)
{
    DecArgs A;
    A.B = D.B; A.d = D.d; A.H = D.H; A.F = D.F; A.BH = D.B * D.H; A.G = P.grid; A.t = t;
    A.S = P.grid / A.BH < kDecMaxSplit ? P.grid / A.BH : kDecMaxSplit;
    if (P.split_override > 0 && P.split_override < A.S) A.S = P.split_override;
    A.alpha = D.alpha; A.scale = D.scale; A.eps = D.eps; A.alibi = D.alibi; A.norm_free = D.norm_free;
    const Rows r = rows_for(D.d, D.F, P.grid);
    A.R_q = r.R_q; A.R_o = r.R_o; A.R_1 = r.R_1; A.R_kv = r.R_kv; A.R_2 = r.R_2;
    A.ldw = D.d + 8; A.max_batch = P.max_batch;
    A.Wq = (const bf16_t *)W.Wq; A.Wk = (const bf16_t *)W.Wk; A.Wv = (const bf16_t *)W.Wv; A.Wo = (const bf16_t *)W.Wo;
    A.W1 = (const bf16_t *)W.W1; A.W2 = (const bf16_t *)W.W2;
    A.g_attn = (const bf16_t *)W.g_attn; A.g_mlp = (const bf16_t *)W.g_mlp; A.g_kv = (const bf16_t *)W.g_kv;
    A.g_q = (const bf16_t *)W.g_q; A.g_k = (const bf16_t *)W.g_k;
    A.x = (const bf16_t *)x_t; A.y = (bf16_t *)y_t; A.K = (bf16_t *)K; A.V = (bf16_t *)V;
    A.kv_rs = kv_row_elems ? kv_row_elems : (size_t)A.BH * kHeadDim;
    const Slab s = slab_for(D.d, D.F, P.grid);
    char *p = (char *)P.slab;
    A.bar = (unsigned long long *)(p + s.bar);
    A.qkv_ll = (ll_t *)(p + s.qkv); A.part_ll = (ll_t *)(p + s.part);
    A.a_ll = (ll_t *)(p + s.a); A.h_ll = (ll_t *)(p + s.h); A.z_ll = (ll_t *)(p + s.z); A.u_ll = (ll_t *)(p + s.u);
    A.kv_ll = (ll_t *)(p + s.kv); A.zss_ll = (ll_t *)(p + s.zss); A.zp_ll = (ll_t *)(p + s.zp);
    A.spin_limit = P.spin_limit;
    A.pre_sleep = 2;   // units of 4 x 64 clocks
    A.trace = P.want_trace ? (unsigned long long *)(p + s.trace) : nullptr;
    // every word of the slab is written at most once per call and carries the call's number; when the numbers start
    // over, no word of an earlier call may survive (the abort word at bar[8] is only ever set, never cleared here)
    if (P.nonce == 0xFFFFFFFFu) {
        hipLaunchKernelGGL(dec_clear_kernel, dim3(256), dim3(256), 0, st, (unsigned long long *)(p + s.qkv), (s.trace - s.qkv) / 8);
        hipError_t ce = hipGetLastError();
        if (ce != hipSuccess) { err = std::string("dec_clear_kernel: ") + hipGetErrorString(ce); return RT_ERR_HIP; }
        P.nonce = 0;
    }
    P.nonce += 1;
    A.tag = P.nonce;
    // An ordinary launch: one workgroup fills a compute unit (LDS), the grid is one workgroup per compute unit, so every
    // workgroup becomes resident as soon as the kernels before it on the stream have drained.  (A cooperative launch
    // guarantees the same, but goes through the device's cooperative queue, which measured 19 us per step between
    // two launches against 39 us of kernel.)  Two such launches on different streams at the same time could each
    // hold a part of the chip and wait for the rest: their bounded waits then expire (rt_device_wait_expired).
    hipError_t e;
    if (P.cooperative) {
        void *args[] = {&A};
        e = hipLaunchCooperativeKernel((const void *)pick(D.d, D.F), dim3(P.grid), dim3(kPThreads), args, (unsigned int)P.lds_bytes, st);
    } else {
        hipLaunchKernelGGL(pick(D.d, D.F), dim3(P.grid), dim3(kPThreads), (unsigned int)P.lds_bytes, st, A);
        e = hipGetLastError();
    }
    if (e != hipSuccess) { err = std::string("decode_coop_kernel launch: ") + hipGetErrorString(e); return RT_ERR_HIP; }
    P.launched = true;
    return RT_OK;
}

int decode_coop_wait_expired(DecodeCoopState &P)
{
    if (!P.slab || !P.launched) return 0;
    unsigned long long v = 0;
    if (hipMemcpy(&v, (char *)P.slab + 64, sizeof(v), hipMemcpyDeviceToHost) != hipSuccess) return -1;
    return v != 0 ? 1 : 0;
}

int decode_coop_read_trace(DecodeCoopState &P, unsigned long long *out, int workgroups)
{
    if (!P.slab || !P.want_trace || !out) return 0;
    const int n = workgroups < P.grid ? workgroups : P.grid;
    const Slab s = slab_for(P.d, P.F, P.grid);
    if (hipMemcpy(out, (char *)P.slab + s.trace, (size_t)n * 16 * 8, hipMemcpyDeviceToHost) != hipSuccess) return -1;
    return n;
}

}  // namespace rt
