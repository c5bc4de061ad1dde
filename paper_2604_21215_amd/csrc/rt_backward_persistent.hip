// The reverse loop of the backward pass (paper Sec. 6.4) as a single cooperative launch per block of 32 positions,
// bf16 storage: the structure of the forward's single-launch engine (rt_persistent.hip) applied to the transposed chain.
//
// Per position i the loop has to take the complete gradient of the persistent pair (dK_i, dV_i) back to the attention
// output of that position:
//     d_rz = Wk^T dkraw + Wv^T dV_i                     dkraw = per-head normalisation backward of dK_i
//     Gz   = gy_i + RMS-backward_z(d_rz)                (gradient of z_i)
//     dpre = gelu'(pre_i) * (W2^T alpha Gz)
//     t1   = W1^T dpre,   dh = Gz + RMS-backward_h(t1)
//     dc   = Wo^T alpha dh                              -> softmax backward of query i, which adds to dK_j, dV_j, j < i
// The four transposed matrices (11 d^2 elements, the same amount as the forward's) are split over the 256 workgroups by
// output rows (W1^T in 64 row blocks x 4 contraction blocks) and stay in LDS; the vectors between the products cross the
// chip in self-validating words (rt_ll.h).  An RMS backward needs a sum over the whole row, dot = <unit, w>, which would
// cost an exchange of its own; instead it is applied AFTER the next product, which is linear in it:
//     W (base + r (w - unit dot / d)) = W base + r (W w - (dot / d) W unit),
// where W base and W unit (base = gy_i or, for dh, the terms of Gz; unit = the normalised z_i or h_i) do not depend on the
// loop and are formed for all positions by batched products before it (A_gy, A_uz = W2^T gy, W2^T unit_z; C_gy, C_uz,
// C_uh = Wo^T gy, Wo^T unit_z, Wo^T unit_h), and every workgroup forms dot itself from the vector it has just pulled.
// Six exchanges per position:
//   U    per (b, h) wavefront: dK_i, dV_i (complete) -> dkraw                                   -> [dkraw | dV_i]
//   G1   d_rz rows = Wk^T dkraw + Wv^T dV_i;  w = d_rz g_kv                                      -> w
//   G2   dot = <unit_z, w>;  W2^T w and Wo^T w;  dpre rows                                       -> dpre;   Gz rows
//   G3a  partial W1^T dpre over one quarter of the hidden dimension                              -> 4 partial sums
//   G3b  t1 rows = sum of the partials;  w2 = t1 g_mlp                                           -> w2
//   G4   dot2 = <unit_h, w2>;  Wo^T w2;  dc rows, dh rows                                        -> dc
//   A    per (b, h) wavefront: softmax backward of query i: its own temporary pair (dq, dk_tmp, dv_tmp of the row) and
//        the keys of its block before it, whose K, V rows and dK, dV accumulators this wavefront keeps in LDS.
// A launch covers the positions of ONE block of 32 (i_hi down to i_lo): the keys before the block receive this block's
// queries through Algorithm 1's tiles run backwards (bw_event_kernel), which are ordinary launches between two of these.
// Every wait is bounded (spin limit -> abort word -> every workgroup leaves).
#include "rt_backward_persistent.h"
#include "rt_ll.h"
#include <cstring>
#include <cstdlib>

#include <cstdlib>

namespace rt {

constexpr int kBwpBlock = 32;          // positions per launch = the block below which queries reach keys directly
constexpr int kWinLd = kHeadDim + 4;   // row stride of the window tiles in floats

struct BwpArgs {
    int B, N, d, H, F, BH, G;
    int i_hi, i_lo;
    float alpha, scale, alibi;
    int norm_free;
    int R_o, R_1, R_2, ldw;
    const bf16_t *WkvT, *W2T, *W1T, *WoT;        // [d][2d], [F][d], [d][F], [d][d]
    const bf16_t *g_kv, *g_mlp, *g_k;
    const bf16_t *gy;                            // [B][N][d]
    const float *unit_k, *rk;                    // [M][2d] (first d columns), [M][H]
    const float *unit_z, *rinv_z, *unit_h, *rinv_h;
    const float *gp, *A_gy, *A_uz;               // [M][F]
    const float *C_gy, *C_uz, *C_uh;             // [M][d]
    const float *Qn, *Ktn, *Vt, *Kp, *Vp, *c, *lse;
    float *dK, *dV;                              // [M][d]: read at launch (upstream + tiles), final values written back
    float *dkraw, *d_rz, *Gz, *dpre, *t1, *d_h, *dc, *Ds, *dq, *dkt, *dvt;
    ll_t *e1k, *e1v, *e2, *e5;                   // [2][kBMax][d/2]   two bf16 per word
    ll_t *e3;                                    // [2][kBMax][F/2]
    ll_t *e4;                                    // [2][4][kBMax][d]  one fp32 per word
    ll_t *e6;                                    // [2][kBMax][d]     one fp32 per word
    unsigned tag_base;
    unsigned long long *bar;
    long long spin_limit;
    int pre_sleep;
    int ps_g1, ps_g2, ps_g3, ps_g4;   // waits before the first poll of the four pulls, units of 4 x 64 clocks
};

// Workgroup barrier behind which every wavefront leaves when any of them has given up waiting: that wavefront raises an LDS
// flag before the barrier, all read it behind the barrier (it is never lowered again).  One barrier and one LDS read instead
// of a workgroup-wide reduction of the predicate (two barriers and LDS atomics).
#define RT_BWP_ABORT_IF(cond)                                                                                           \
    do {                                                                                                                \
        if (cond) gave_up_s = 1;                                                                                        \
        __syncthreads();                                                                                                \
        if (gave_up_s != 0) {                                                                                           \
            if (threadIdx.x == 0) __hip_atomic_store(A.bar + 8, 1ULL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);     \
            return;                                                                                                     \
        }                                                                                                               \
    } while (0)

// This wavefront's part of <unit row, staged bf16 vector> for every batch row: the wavefront owns the KS * 32 elements of
// every staged row that it has pulled itself, eight lanes per batch row (b = lane / 8) with PER = KS * 4 elements each;
// u = those elements of the unit row.  Lanes lane % 8 == 0 return the part of their batch row (B <= 8).  No other
// wavefront's staging is read: this runs behind the wavefront's own pull, not behind a workgroup barrier.
template <int PER>
__device__ __forceinline__ float row_dot_part(const float (&u)[PER], const bf16_t *act_mine, int lane)
{
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < PER; e += 2) {
        const unsigned pr = *reinterpret_cast<const unsigned *>(act_mine + e);
        s = fmaf(u[e], __uint_as_float(pr << 16), s);
        s = fmaf(u[e + 1], __uint_as_float(pr & 0xFFFF0000u), s);
    }
    s += dpp_f(s, 0);
    s += dpp_f(s, 1);
    s += dpp_f(s, 2);   // the eight lanes of a batch row (half a row of 16 lanes)
    return s;
}

// KSD = d / 256.  One workgroup per compute unit, 512 threads.
template <int KSD>
__global__ __launch_bounds__(kPThreads) void bwp_kernel(BwpArgs A)
{
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int gave_up_s;   // raised by a wavefront whose bounded wait ran out; the first barrier below precedes its first use
    if (threadIdx.x == 0) gave_up_s = 0;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wg = blockIdx.x, G = A.G;
    const int d = A.d, F = A.F, B = A.B, BH = A.BH, H = A.H;
    constexpr int RO = 2 * ((KSD + 1) / 2), R1 = 4 * KSD;
    constexpr int PER = 4 * KSD;   // elements of a d-long row per lane
    static_assert((KSD * 32) % RO == 0, "a wavefront pulls exactly the slice of the d-long vectors that it multiplies (wg_gemv_ll)");

    // ---- LDS carve-up
    bf16_t *wk_s = reinterpret_cast<bf16_t *>(smem);                 // Wk^T rows  [R_o][ldw]
    bf16_t *wv_s = wk_s + (size_t)A.R_o * A.ldw;                      // Wv^T rows
    bf16_t *wo_s = wv_s + (size_t)A.R_o * A.ldw;                      // Wo^T rows
    bf16_t *w2_s = wo_s + (size_t)A.R_o * A.ldw;                      // W2^T rows  [R_1][ldw]
    bf16_t *w1_s = w2_s + (size_t)A.R_1 * A.ldw;                      // W1^T block [R_2][ldw]
    float *red = reinterpret_cast<float *>(w1_s + (size_t)A.R_2 * A.ldw);   // [kPW][kRMax][kBMax]
    float *red2 = red + kPW * kRMax * kBMax;
    float *w_loc = red2 + kPW * kRMax * kBMax;                        // [kRMax][kBMax] each
    float *gz_loc = w_loc + kRMax * kBMax;
    float *cw_loc = gz_loc + kRMax * kBMax;
    float *w2_loc = cw_loc + kRMax * kBMax;
    float *dot_s = w2_loc + kRMax * kBMax;                            // [kPW][kBMax]: one part per wavefront
    float *dot2_s = dot_s + kPW * kBMax;
    float *winK = dot2_s + kPW * kBMax;                                     // [32][kWinLd] keys of the block (this workgroup's (b, h))
    float *winV = winK + kBwpBlock * kWinLd;
    float *accK = winV + kBwpBlock * kWinLd;                          // [32][64] dK, dV of the block's positions
    float *accV = accK + kBwpBlock * kHeadDim;
    bf16_t *act_s = reinterpret_cast<bf16_t *>(accV + kBwpBlock * kHeadDim);   // [8][ldw] staged vector of the phase in flight

    // ---- this workgroup's rows
    const int o_lo = min(wg * A.R_o, d), o_n = min(d, o_lo + A.R_o) - o_lo;          // rows of the d-row matrices
    const int f_lo = min(wg * A.R_1, F), f_n = min(F, f_lo + A.R_1) - f_lo;          // rows of W2^T
    const int rb = wg >> 2, jb = wg & 3, RB = A.R_2;                                  // W1^T: row block x contraction block
    {   // the five slices are contiguous in LDS: one run of requests (a launch covers only 32 positions, so its start-up counts)
        constexpr int PERW = 32 * KSD;   // 16-byte pieces of a d-long row
        constexpr int WROWS = 3 * RO + R1 + 4 * KSD, NBW = (WROWS * PERW + kPThreads - 1) / kPThreads;
        const int n1 = A.R_o, n2 = 2 * A.R_o, n3 = 3 * A.R_o, n4 = n3 + A.R_1, n5 = n4 + A.R_2;
        uint4 wreg[NBW];
        rows_issue<NBW, PERW>(wreg, n5, [&](int r) -> const bf16_t * {
            if (r < n1) return r < o_n ? A.WkvT + (size_t)(o_lo + r) * 2 * d : nullptr;
            if (r < n2) return r - n1 < o_n ? A.WkvT + (size_t)(o_lo + r - n1) * 2 * d + d : nullptr;
            if (r < n3) return r - n2 < o_n ? A.WoT + (size_t)(o_lo + r - n2) * d : nullptr;
            if (r < n4) return r - n3 < f_n ? A.W2T + (size_t)(f_lo + r - n3) * d : nullptr;
            return A.W1T + (size_t)(rb * RB + r - n4) * F + (size_t)jb * d;
        });
        rows_commit<NBW, PERW>(wreg, wk_s, A.ldw, n5, [](int) -> const bf16_t * { return nullptr; });
    }

    const size_t rs = (size_t)BH * kHeadDim;   // = B d: one position of a position-first tensor
    const int blk_lo = A.i_lo;                 // first position of the block
    const int my_u = wg;                       // the (b, h) of wavefront 0 of workgroups 0 .. BH - 1
    const bool has_u = wave == 0 && my_u < BH;
    if (my_u < BH) {   // the block's keys, values and gradient accumulators of this (b, h): every wavefront four rows, all
                       // sixteen loads of a wavefront in flight at once
        float kv4[kBwpBlock / kPW][4];
#pragma unroll
        for (int jj = 0; jj < kBwpBlock / kPW; ++jj) {
            const int pos = min(blk_lo + wave + kPW * jj, A.N - 1);
            const size_t o = (size_t)pos * rs + (size_t)my_u * kHeadDim + lane;
            kv4[jj][0] = A.Kp[o]; kv4[jj][1] = A.Vp[o]; kv4[jj][2] = A.dK[o]; kv4[jj][3] = A.dV[o];
        }
#pragma unroll
        for (int jj = 0; jj < kBwpBlock / kPW; ++jj) {
            const int j = wave + kPW * jj;
            winK[j * kWinLd + lane] = kv4[jj][0];
            winV[j * kWinLd + lane] = kv4[jj][1];
            accK[j * kHeadDim + lane] = kv4[jj][2];
            accV[j * kHeadDim + lane] = kv4[jj][3];
        }
    }
    __syncthreads();

    const int erow = tid >> 4, eb = tid & 15;   // epilogue thread -> (row, batch row) for tid < 256
    const size_t half_d = (size_t)kBMax * (d / 2), half_F = (size_t)kBMax * (F / 2), sz_d = (size_t)kBMax * d;
    const float inv_d = 1.f / (float)d;
    const bool ep = tid < kRMax * kBMax && eb < B;
    const bool ep_o = ep && erow < o_n, ep_f = ep && erow < f_n;
    const float gkv_o = (ep_o && A.g_kv && !A.norm_free) ? bf16_to_f32(A.g_kv[o_lo + erow]) : 1.f;
    const float gmlp_o = (ep_o && A.g_mlp && !A.norm_free) ? bf16_to_f32(A.g_mlp[o_lo + erow]) : 1.f;

    // phase U opens every position: what it needs from memory is requested one position ahead (the gain once)
    const float gk_u = (has_u && A.g_k) ? bf16_to_f32(A.g_k[(my_u % H) * kHeadDim + lane]) : 1.f;
    float un_nx = 0.f, rk_nx = 1.f;
    if (has_u && !A.norm_free) {
        const size_t rb0 = (size_t)A.i_hi * B + my_u / H;
        un_nx = A.unit_k[rb0 * 2 * d + (my_u % H) * kHeadDim + lane];
        rk_nx = A.rk[rb0 * H + my_u % H];
    }

    // Phase U: the complete pair gradient (dk_, dv_) of position ipos_ goes out as the vectors of step tag_ / parity par_.  It runs
    // at the end of the previous position's phase A, as soon as that query's contribution to this one slot is in (the other slots
    // are updated afterwards, while the vectors cross the chip); for the block's last position it runs before the loop.
#define RT_BWP_PHASE_U(ipos_, par_, tag_, dk_, dv_)                                                                        \
    {                                                                                                                      \
        const int ub_ = my_u / H, uh_ = my_u - ub_ * H;                                                                    \
        const size_t off_ = (size_t)(ipos_) * rs + (size_t)my_u * kHeadDim + lane;                                         \
        float du_ = (dk_);                                                                                                 \
        if (!A.norm_free) {                                                                                                \
            const float wv_ = (dk_) * gk_u;                                                                                \
            const float un_ = un_nx, rk_ = rk_nx;                                                                          \
            du_ = rk_ * (wv_ - un_ * (fast_sum(un_ * wv_) * (1.f / (float)kHeadDim)));                                     \
            if ((ipos_) > A.i_lo) {                                                                                        \
                const size_t rbn_ = (size_t)((ipos_) - 1) * B + ub_;                                                       \
                un_nx = A.unit_k[rbn_ * 2 * d + uh_ * kHeadDim + lane];                                                    \
                rk_nx = A.rk[rbn_ * H + uh_];                                                                              \
            }                                                                                                              \
        }                                                                                                                  \
        const float dun_ = dpp_odd_neighbour(du_), dvn_ = dpp_odd_neighbour((dv_));                                        \
        if (!(lane & 1)) {                                                                                                 \
            ll_store(A.e1k + (par_) * half_d + pair_word<32>(uh_ * kHeadDim + lane, ub_), (tag_),                          \
                     (unsigned)f32_to_bf16(du_) | ((unsigned)f32_to_bf16(dun_) << 16));                                    \
            ll_store(A.e1v + (par_) * half_d + pair_word<32>(uh_ * kHeadDim + lane, ub_), (tag_),                          \
                     (unsigned)f32_to_bf16((dv_)) | ((unsigned)f32_to_bf16(dvn_) << 16));                                  \
        }                                                                                                                  \
        A.dK[off_] = (dk_);                                                                                                \
        A.dV[off_] = (dv_);                                                                                                \
        A.dkraw[off_] = du_;                                                                                               \
    }
    if (has_u && A.i_hi >= A.i_lo) {
        const int slot = A.i_hi - blk_lo;
        const float dk0 = accK[slot * kHeadDim + lane], dv0 = accV[slot * kHeadDim + lane];
        RT_BWP_PHASE_U(A.i_hi, 0, A.tag_base | 1u, dk0, dv0)
    }

    for (int i = A.i_hi; i >= A.i_lo; --i) {
        const int step = A.i_hi - i, par = step & 1;
        const unsigned tag = A.tag_base | (unsigned)(step + 1);
        const size_t r0 = (size_t)i * B;
        int fail = 0;
        // ---- what the epilogues of this position need from the recompute (issued now, used phases later)
        float e_gy = 0.f, e_uz = 0.f, e_uh = 0.f, e_cgy = 0.f, e_cuz = 0.f, e_cuh = 0.f, e_rz = 1.f, e_rh = 1.f;
        float e_gp = 0.f, e_agy = 0.f, e_auz = 0.f;
        if (ep) {
            const size_t r = r0 + eb;
            e_rz = A.rinv_z[r];
            e_rh = A.rinv_h[r];
            if (ep_o) {
                const size_t o = r * d + o_lo + erow;
                e_gy = bf16_to_f32(A.gy[((size_t)eb * A.N + i) * d + o_lo + erow]);
                e_uz = A.unit_z[o]; e_uh = A.unit_h[o];
                e_cgy = A.C_gy[o]; e_cuz = A.C_uz[o]; e_cuh = A.C_uh[o];
            }
            if (ep_f) {
                const size_t f = r * F + f_lo + erow;
                e_gp = A.gp[f]; e_agy = A.A_gy[f]; e_auz = A.A_uz[f];
            }
        }
        // this wavefront's slice of the normalised rows of every batch row, for its parts of the two row-wide sums (B <= 8)
        float uz[PER], uh[PER];
        const int db = lane >> 3, dcol = wave * (KSD * 32) + (lane & 7) * PER;
        if (db < B) {
            const float *pz = A.unit_z + (r0 + db) * d + dcol, *ph = A.unit_h + (r0 + db) * d + dcol;
#pragma unroll
            for (int e = 0; e < PER; e += 4) {
                const float4 a = *reinterpret_cast<const float4 *>(pz + e), b4 = *reinterpret_cast<const float4 *>(ph + e);
                uz[e] = a.x; uz[e + 1] = a.y; uz[e + 2] = a.z; uz[e + 3] = a.w;
                uh[e] = b4.x; uh[e + 1] = b4.y; uh[e + 2] = b4.z; uh[e + 3] = b4.w;
            }
        } else {
#pragma unroll
            for (int e = 0; e < PER; ++e) uz[e] = uh[e] = 0.f;
        }

        // ================================================================ G1: d_rz = Wk^T dkraw + Wv^T dV_i
        wg_gemv_ll_pair<KSD, 32>(wk_s, wv_s, A.ldw, o_n, A.e1k + par * half_d, A.e1v + par * half_d, B, tag, A, red, act_s, A.ldw,
                                 fail, A.ps_g1);
        RT_BWP_ABORT_IF(fail);
        if (tid < kRMax * kBMax) {
            float wv = 0.f;
            if (ep_o) {
                const float drz = red_sum(red, erow, eb);
                A.d_rz[(r0 + eb) * d + o_lo + erow] = drz;
                wv = drz * gkv_o;
            }
            const float wn = next_row(wv);
            if (!(erow & 1) && ep_o)
                ll_store(A.e2 + par * half_d + pair_word<RO / 2>(o_lo + erow, eb), tag,
                         (unsigned)f32_to_bf16(wv) | ((unsigned)f32_to_bf16(wn) << 16));
            w_loc[erow * kBMax + eb] = wv;
        }
        __syncthreads();

        // ================================================================ G2: dot, W2^T w, Wo^T w; dpre rows, Gz rows
        wg_gemv_ll<KSD, RO / 2>(w2_s, A.ldw, f_n, A.e2 + par * half_d, B, tag, A, red, act_s, A.ldw, fail, nullptr, A.ps_g2);
        // the second product and this wavefront's part of the row-wide sum read only what the wavefront staged itself: both
        // run before the barrier
        wg_product_staged<KSD>(wo_s, A.ldw, o_n, B, red2, act_s, A.ldw);
        {
            const float dt = (A.norm_free || db >= B) ? 0.f : row_dot_part<PER>(uz, act_s + (size_t)min(db, B - 1) * A.ldw + dcol, lane);
            if ((lane & 7) == 0) dot_s[wave * kBMax + db] = dt;
        }
        RT_BWP_ABORT_IF(fail);
        if (tid < kRMax * kBMax) {
            float dp = 0.f, dot = 0.f;
            if (ep) {
#pragma unroll
                for (int w = 0; w < kPW; ++w) dot += dot_s[w * kBMax + eb];
            }
            if (ep_f) {
                const float v = red_sum(red, erow, eb);
                const float lin = A.norm_free ? e_agy + v : e_agy + e_rz * (v - dot * inv_d * e_auz);
                dp = e_gp * A.alpha * lin;
            }
            const float dn = next_row(dp);
            if (!(erow & 1) && ep_f)
                ll_store(A.e3 + par * half_F + pair_word<R1 / 2>(f_lo + erow, eb), tag,
                         (unsigned)f32_to_bf16(dp) | ((unsigned)f32_to_bf16(dn) << 16));
            if (ep_f) A.dpre[(r0 + eb) * F + f_lo + erow] = dp;
            if (ep_o) {
                const float wv = w_loc[erow * kBMax + eb];
                const float gz = A.norm_free ? e_gy + wv : e_gy + e_rz * (wv - e_uz * dot * inv_d);
                A.Gz[(r0 + eb) * d + o_lo + erow] = gz;
                gz_loc[erow * kBMax + eb] = gz;
                cw_loc[erow * kBMax + eb] = red_sum(red2, erow, eb);
            }
        }
        __syncthreads();

        // ================================================================ G3a: partial W1^T dpre over contraction block jb
        wg_gemv_ll<KSD, R1 / 2>(w1_s, A.ldw, RB, A.e3 + par * half_F + (size_t)jb * (kBMax * (d / 2)), B, tag, A, red, act_s, A.ldw,
                                fail, nullptr, A.ps_g3);
        RT_BWP_ABORT_IF(fail);
        if (tid < kRMax * kBMax && erow < RB && eb < B)
            ll_store(A.e4 + ((size_t)(par * 4 + jb) * kBMax + eb) * d + rb * RB + erow, tag, __float_as_uint(red_sum(red, erow, eb)));
        __syncthreads();

        // ================================================================ G3b: t1 rows, w2 = t1 g_mlp
        if (tid < kRMax * kBMax) {
            const int o = o_lo + erow;
            const ll_t *pp[4];
            bool act[4];
            ll_t w4[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                act[j] = ep_o;
                pp[j] = A.e4 + ((size_t)(par * 4 + j) * kBMax + (ep_o ? eb : 0)) * d + (ep_o ? o : 0);
            }
            ll_wait_n<4>(pp, act, tag, A, w4, fail);
            float w2v = 0.f;
            if (ep_o) {
                const float t1v = (__uint_as_float((unsigned)w4[0]) + __uint_as_float((unsigned)w4[1])) +
                                  (__uint_as_float((unsigned)w4[2]) + __uint_as_float((unsigned)w4[3]));
                A.t1[(r0 + eb) * d + o] = t1v;
                w2v = t1v * gmlp_o;
            }
            const float wn = next_row(w2v);
            if (!(erow & 1) && ep_o)
                ll_store(A.e5 + par * half_d + pair_word<RO / 2>(o, eb), tag,
                         (unsigned)f32_to_bf16(w2v) | ((unsigned)f32_to_bf16(wn) << 16));
            w2_loc[erow * kBMax + eb] = w2v;
        }
        RT_BWP_ABORT_IF(fail);

        // ================================================================ G4: dot2, Wo^T w2; dc rows, dh rows
        wg_gemv_ll<KSD, RO / 2>(wo_s, A.ldw, o_n, A.e5 + par * half_d, B, tag, A, red, act_s, A.ldw, fail, nullptr, A.ps_g4);
        {   // this wavefront's part of the second row-wide sum, before the barrier (see G2)
            const float dt = (A.norm_free || db >= B) ? 0.f : row_dot_part<PER>(uh, act_s + (size_t)min(db, B - 1) * A.ldw + dcol, lane);
            if ((lane & 7) == 0) dot2_s[wave * kBMax + db] = dt;
        }
        RT_BWP_ABORT_IF(fail);
        if (tid < kRMax * kBMax && ep_o) {
            const int o = o_lo + erow;
            const float v = red_sum(red, erow, eb), cw = cw_loc[erow * kBMax + eb];
            const float w2v = w2_loc[erow * kBMax + eb], gz = gz_loc[erow * kBMax + eb];
            float dcv, dh;
            if (A.norm_free) {
                dcv = A.alpha * (e_cgy + cw + v);
                dh = gz + w2v;
            } else {
                float k1 = 0.f, k2 = 0.f;
#pragma unroll
                for (int w = 0; w < kPW; ++w) { k1 += dot_s[w * kBMax + eb]; k2 += dot2_s[w * kBMax + eb]; }
                k1 *= inv_d; k2 *= inv_d;
                dcv = A.alpha * (e_cgy + e_rz * (cw - k1 * e_cuz) + e_rh * (v - k2 * e_cuh));
                dh = gz + e_rh * (w2v - e_uh * k2);
            }
            ll_store(A.e6 + par * sz_d + single_word<RO>(o, eb), tag, __float_as_uint(dcv));
            A.dc[(r0 + eb) * d + o] = dcv;
            A.d_h[(r0 + eb) * d + o] = dh;
        }
        __syncthreads();

        // ================================================================ A: softmax backward of query i
        float t_p = 0.f, t_ds = 0.f, t_g = 0.f, t_q = 0.f;   // for the older slots, updated behind the barrier below
        int t_w = 0;
        if (has_u) {
            const int u = my_u, b = u / H, h = u - b * H;
            const size_t off = (size_t)i * rs + (size_t)u * kHeadDim + lane;
            const float q = A.Qn[off], kt = A.Ktn[off], vt = A.Vt[off], cv = A.c[off];
            const float L = A.lse[(size_t)i * BH + u];
            const int w = i - blk_lo;   // keys of the block before the query: slots 0 .. w - 1
            // what does not need the gradient of the attention output is formed before the wait for it: the query's own
            // weight and the logits of the window
            const float p_own = __expf(A.scale * fast_sum(q * kt) - L);
            const float *krow = winK + (size_t)min(lane, max(w - 1, 0)) * kWinLd, *vrow = winV + (size_t)min(lane, max(w - 1, 0)) * kWinLd;
            float s = 0.f;
            if (w > 0) {
#pragma unroll
                for (int c8 = 0; c8 < 8; ++c8) {
                    float kk[8];
                    load8(krow + c8 * 8, kk);
#pragma unroll
                    for (int e = 0; e < 8; ++e) s = fmaf(lane_bcast(q, c8 * 8 + e), kk[e], s);
                }
            }
            const ll_t wd = ll_wait(A.e6 + par * sz_d + single_word<RO>(h * kHeadDim + lane, b), true, tag, A, fail);
            const float g = __uint_as_float((unsigned)wd);
            const float Dsum = fast_sum(g * cv);
            const float ds_own = p_own * (fast_sum(g * vt) - Dsum);
            if (w > 0) {
                float dp = 0.f;
#pragma unroll
                for (int c8 = 0; c8 < 8; ++c8) {
                    float vv[8];
                    load8(vrow + c8 * 8, vv);
#pragma unroll
                    for (int e = 0; e < 8; ++e) dp = fmaf(lane_bcast(g, c8 * 8 + e), vv[e], dp);
                }
                const float slope = alibi_slope(A.alibi, h, H);
                const float p = lane < w ? __expf(fmaf(-slope, (float)(w - lane), s * A.scale) - L) : 0.f;
                const float ds = p * (dp - Dsum);
                // the newest slot first: with it the pair gradient of position i - 1 is complete and goes out at once
                {
                    const int j = w - 1;
                    const float dvn = fmaf(lane_bcast(p, j), g, accV[j * kHeadDim + lane]);
                    const float dkn = fmaf(A.scale * lane_bcast(ds, j), q, accK[j * kHeadDim + lane]);
                    RT_BWP_PHASE_U(i - 1, par ^ 1, tag + 1u, dkn, dvn)
                }
                t_p = p; t_ds = ds; t_g = g; t_q = q; t_w = w;
            }
            // the query's own gradients follow the pair gradient of the next position: only that one is waited for
            A.dvt[off] = p_own * g;
            A.dkt[off] = A.scale * ds_own * q;
            A.dq[off] = A.scale * ds_own * kt;
            if (lane == 0) A.Ds[(size_t)i * BH + u] = Dsum;
        }
        // every other wavefront goes on as soon as the pair gradient has left; the owner follows after the older slots
        RT_BWP_ABORT_IF(fail);
        if (has_u && t_w > 1) {
            // the older slots eight keys at a time: all reads of a group before its writes (one key per trip is a chain of
            // dependent LDS round trips)
            for (int j0 = 0; j0 < t_w - 1; j0 += 8) {
                float av[8], ak[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int j = min(j0 + e, t_w - 2);
                    av[e] = accV[j * kHeadDim + lane];
                    ak[e] = accK[j * kHeadDim + lane];
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int j = j0 + e;
                    if (j < t_w - 1) {   // wavefront-uniform
                        accV[j * kHeadDim + lane] = fmaf(lane_bcast(t_p, j), t_g, av[e]);
                        accK[j * kHeadDim + lane] = fmaf(A.scale * lane_bcast(t_ds, j), t_q, ak[e]);
                    }
                }
            }
        }
    }
}

// =============================================================================================
// Host side
// =============================================================================================
namespace {
typedef void (*bwp_fn)(BwpArgs);
bwp_fn pick(int d, int F)
{
    if (d % (32 * kPW) != 0 || F != 4 * d) return nullptr;
    switch (d / (32 * kPW)) {
    case 1: return bwp_kernel<1>;
    case 2: return bwp_kernel<2>;
    case 3: return bwp_kernel<3>;
    case 4: return bwp_kernel<4>;
    default: return nullptr;
    }
}
size_t up256(size_t v) { return (v + 255) / 256 * 256; }
void rows_per_wg(int d, int F, int G, int *R_o, int *R_1)
{
    *R_o = 2 * ((d + 2 * G - 1) / (2 * G));
    *R_1 = 2 * ((F + 2 * G - 1) / (2 * G));
}
size_t lds_bytes(int d, int F, int G)
{
    int R_o, R_1;
    rows_per_wg(d, F, G, &R_o, &R_1);
    const size_t ldw = d + 8;
    size_t b = ((size_t)(3 * R_o + R_1 + d / 64) * ldw) * 2;
    b = (b + 15) / 16 * 16;
    b += (size_t)(2 * kPW * kRMax * kBMax + 4 * kRMax * kBMax + 2 * kPW * kBMax) * 4;
    b += (size_t)(2 * kBwpBlock * kWinLd + 2 * kBwpBlock * kHeadDim) * 4;
    b = (b + 15) / 16 * 16;
    b += (size_t)8 * ldw * 2;
    return b;
}
__global__ void bwp_clear_kernel(unsigned long long *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0ULL;
}
}  // namespace

size_t bwp_exchange_bytes(int d, int F)
{
    // bar (256) + e1k, e1v, e2, e5: 2 kBMax d/2 words; e3: 2 kBMax F/2; e4: 2 * 4 kBMax d; e6: 2 kBMax d
    size_t words = 4 * (size_t)2 * kBMax * (d / 2) + (size_t)2 * kBMax * (F / 2) + (size_t)2 * 4 * kBMax * d + (size_t)2 * kBMax * d;
    return 256 + up256(words * 8) + 8 * 256;
}

bool bwp_create(BwpState &P, int device, int d, int F, int H, int max_batch, bool bf16_mfma)
{
    P.available = false;
    if (!bf16_mfma || getenv("RT_BWD_NO_PERSISTENT")) return false;
    bwp_fn fn = pick(d, F);
    if (!fn || max_batch < 1) return false;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return false;
    if (!prop.cooperativeLaunch || prop.multiProcessorCount != 256) return false;   // W1^T is laid out as 64 x 4 workgroups
    const int G = 256;
    int R_o, R_1;
    rows_per_wg(d, F, G, &R_o, &R_1);
    if (R_o > kRMax || R_1 > kRMax || d / 64 > kRMax) return false;
    const size_t lds = lds_bytes(d, F, G);
    if (lds + 16 > (size_t)160 * 1024) return false;   // 16: the statically allocated flag word
    if (hipFuncSetAttribute((const void *)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, fn, kPThreads, lds) != hipSuccess || nb < 1) {
        (void)hipGetLastError();
        return false;
    }
    P.grid = G;
    P.lds_bytes = lds;
    P.H = H;
    const char *sl = getenv("RT_SPIN_LIMIT");
    P.spin_limit = sl ? atoll(sl) : (1LL << 21);
    if (P.spin_limit < 1) P.spin_limit = 1;
    P.available = true;
    return true;
}

bool bwp_supported(const BwpState &P, const LayerDims &D)
{
    return P.available && D.B <= 8 && D.B * D.H <= P.grid && D.H == P.H;
}

hipError_t bwp_clear(void *exchange, size_t bytes, hipStream_t st)
{
    hipLaunchKernelGGL(bwp_clear_kernel, dim3(256), dim3(256), 0, st, (unsigned long long *)exchange, bytes / 8);
    return hipGetLastError();
}

hipError_t bwp_run_block(BwpState &P, const LayerDims &D, const BwpTensors &T, void *exchange, int i_hi, int i_lo, hipStream_t st)
{
    BwpArgs A;
    A.B = D.B; A.N = D.N; A.d = D.d; A.H = D.H; A.F = D.F; A.BH = D.B * D.H; A.G = P.grid;
    A.i_hi = i_hi; A.i_lo = i_lo;
    A.alpha = D.alpha; A.scale = D.scale; A.alibi = D.alibi; A.norm_free = D.norm_free;
    rows_per_wg(D.d, D.F, P.grid, &A.R_o, &A.R_1);
    A.R_2 = D.d / 64; A.ldw = D.d + 8;
    A.WkvT = T.WkvT; A.W2T = T.W2T; A.W1T = T.W1T; A.WoT = T.WoT;
    A.g_kv = T.g_kv; A.g_mlp = T.g_mlp; A.g_k = T.g_k; A.gy = T.gy;
    A.unit_k = T.unit_k; A.rk = T.rk; A.unit_z = T.unit_z; A.rinv_z = T.rinv_z; A.unit_h = T.unit_h; A.rinv_h = T.rinv_h;
    A.gp = T.gp; A.A_gy = T.A_gy; A.A_uz = T.A_uz; A.C_gy = T.C_gy; A.C_uz = T.C_uz; A.C_uh = T.C_uh;
    A.Qn = T.Qn; A.Ktn = T.Ktn; A.Vt = T.Vt; A.Kp = T.Kp; A.Vp = T.Vp; A.c = T.c; A.lse = T.lse;
    A.dK = T.dK; A.dV = T.dV; A.dkraw = T.dkraw; A.d_rz = T.d_rz; A.Gz = T.Gz; A.dpre = T.dpre; A.t1 = T.t1; A.d_h = T.d_h;
    A.dc = T.dc; A.Ds = T.Ds; A.dq = T.dq; A.dkt = T.dkt; A.dvt = T.dvt;
    char *p = (char *)exchange;
    A.bar = (unsigned long long *)p; p += 256;
    const size_t d = D.d, F = D.F;
    auto take = [&](size_t words) { ll_t *q = (ll_t *)p; p += words * 8; return q; };
    A.e1k = take(2 * kBMax * (d / 2)); A.e1v = take(2 * kBMax * (d / 2)); A.e2 = take(2 * kBMax * (d / 2)); A.e5 = take(2 * kBMax * (d / 2));
    A.e3 = take(2 * kBMax * (F / 2)); A.e4 = take((size_t)2 * 4 * kBMax * d); A.e6 = take(2 * kBMax * d);
    A.spin_limit = P.spin_limit;
    A.pre_sleep = 2;   // units of 4 x 64 clocks
    {
        const char *ps = getenv("RT_BWD_PRE_SLEEPS");   // four digits: the pulls of phases G1, G2, G3a, G4
        const bool ok = ps && strlen(ps) == 4;
        // measured at cfg3 (ms per backward pass, units of 8 x 64 clocks): 1,1,1,1 48.2; 1,2,1,1 47.8; 1,1,1,2 47.8; 1,2,1,2 47.3; 0,2,1,2 47.2; 1,3,1,2 47.2; 0,0,0,0 49.5
        A.ps_g1 = ok ? ps[0] - '0' : 0; A.ps_g2 = ok ? ps[1] - '0' : 4; A.ps_g3 = ok ? ps[2] - '0' : 2; A.ps_g4 = ok ? ps[3] - '0' : 4;
    }
    if (P.nonce >= 4095u) {   // the tags start over: no word of an earlier launch may survive
        hipError_t ce = bwp_clear(exchange, bwp_exchange_bytes(D.d, D.F), st);
        if (ce != hipSuccess) return ce;
        P.nonce = 0;
    }
    P.nonce += 1;
    A.tag_base = P.nonce << 20;
    // an ordinary launch: one workgroup fills a compute unit and the grid is one workgroup per compute unit, so all of
    // them are resident once the kernels before it on the stream have drained (the cooperative queue costs about
    // 20 us per launch, measured on the decoding step)
    hipLaunchKernelGGL(pick(D.d, D.F), dim3(P.grid), dim3(kPThreads), (unsigned int)P.lds_bytes, st, A);
    return hipGetLastError();
}

}  // namespace rt
