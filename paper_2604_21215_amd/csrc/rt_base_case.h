// Device-side bodies of the base case of Algorithm 1 (Appendix C): finishing a position's attention output
// and the small-M matrix products behind it.  Shared by the per-position engine (one layer per launch,
// rt_stepwise.hip) and the layer-wavefront engine (several layers per launch, rt_wavefront.hip).
#pragma once
#include "rt_common.h"

namespace rt {

// =============================================================================================
// Finish the attention output of position t (0-based) of one (b, h); one wavefront.
//   start from the temporary pair (Algorithm 1, "temporary self contribution"), fold in the stored
//   partial of every level whose bit is set in t, then the direct window of the last (t mod p_min)
//   persistent rows; a = o / l.
//   Decode mode (n_splits >= 0): the partials are slots 0..n_splits-1 of relative level 0, no window.
//   far_rel >= 0 (chunked schedule of the layer-wavefront engine): `levels` covers the blocks inside the
//   position's chunk of 2^log2_chunk positions only; all keys before the chunk were folded into one more
//   partial state, stored at slot t of relative level far_rel.
//   op_a: if not null, a is also written as a bf16 head row and a bf16 remainder row (rows 2b, 2b + 1 of [2B][d]).
//   alibi > 0: linear positional bias; the temporary pair is at distance 0 and every stored partial state was
//   written with its maximum already expressed relative to this query's position, so only the window needs it.
//   HP: the query and the temporary key come unrounded from Qf / Ktf and the window keys are head K plus
//   remainder Klo, so that no logit carries a bf16 rounding of q or k.
// =============================================================================================
// Returns a (lane = head dimension); attn_cat may be null when the caller stores it elsewhere.
template <typename T, bool HP>
__device__ __forceinline__ float merge_body(const T *__restrict__ Q, const float *__restrict__ Qf,
                                           const T *__restrict__ Kt, const float *__restrict__ Ktf,
                                           const T *__restrict__ Vt, const T *__restrict__ K,
                                           const bf16_t *__restrict__ Klo, const T *__restrict__ V,
                                           const float *__restrict__ pm, const float *__restrict__ pl,
                                           const float *__restrict__ po, float *__restrict__ attn_cat, int BH, int H,
                                           int bh, int t, int q_row, int p_min, int log2_pmin, int levels, int slots,
                                           int n_splits, float scale, int far_rel = -1, int log2_chunk = 0,
                                           bf16_t *__restrict__ op_a = nullptr, float alibi = 0.f)
{
    const int lane = threadIdx.x & 63;
    const size_t rs = (size_t)BH * kHeadDim;
    const size_t qoff = (size_t)q_row * rs + (size_t)bh * kHeadDim + lane;
    const float q = HP ? Qf[qoff] : to_f32(Q[qoff]);
    const float kt = HP ? Ktf[qoff] : to_f32(Kt[qoff]);
    float m = scale * wave_sum(q * kt);
    float l = 1.f;
    float o = to_f32(Vt[qoff]);
    if (n_splits >= 0) {
        // two passes, so that no load waits for an exponential: the overall maximum first (lanes read the splits'
        // maxima side by side), then the weighted sums in split order
        float mx = m;
        for (int s0 = 0; s0 < n_splits; s0 += 64) {
            const int sidx = s0 + lane;
            mx = fmaxf(mx, sidx < n_splits ? pm[partial_index(0, sidx, slots, BH, bh)] : -INFINITY);
        }
        mx = wave_max(mx);
        const float e0 = expf(m - mx);
        l = e0;
        o = o * e0;
        for (int s0 = 0; s0 < n_splits; s0 += 64) {
            const int sidx = s0 + lane, cnt = min(64, n_splits - s0);
            float wgt = 0.f, lw = 0.f;
            if (sidx < n_splits) {
                const size_t idx = partial_index(0, sidx, slots, BH, bh);
                wgt = expf(pm[idx] - mx);
                lw = wgt * pl[idx];
            }
            for (int j0 = 0; j0 < cnt; j0 += 8) {   // eight state rows in flight at a time
                float pv[8];
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    pv[e] = po[partial_index(0, s0 + min(j0 + e, cnt - 1), slots, BH, bh) * kHeadDim + lane];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const bool in = j0 + e < cnt;
                    l += in ? lane_bcast(lw, min(j0 + e, 63)) : 0.f;
                    o = fmaf(in ? lane_bcast(wgt, min(j0 + e, 63)) : 0.f, pv[e], o);
                }
            }
        }
        m = mx;
    } else {
        for (int lr = 0; lr < levels; ++lr) {
            const int lv = lr + log2_pmin;
            if ((t >> lv) & 1) {
                const size_t idx = partial_index(lr, partial_slot(lv, t), slots, BH, bh);
                const float pmv = pm[idx], plv = pl[idx], pov = po[idx * kHeadDim + lane];
                const float m_new = fmaxf(m, pmv);
                const float e1 = expf(m - m_new), e2 = expf(pmv - m_new);
                l = l * e1 + plv * e2;
                o = o * e1 + pov * e2;
                m = m_new;
            }
        }
        if (far_rel >= 0 && (t >> log2_chunk) > 0) {
            const size_t idx = partial_index(far_rel, t, slots, BH, bh);
            const float pmv = pm[idx], plv = pl[idx], pov = po[idx * kHeadDim + lane];
            const float m_new = fmaxf(m, pmv);
            const float e1 = expf(m - m_new), e2 = expf(pmv - m_new);
            l = l * e1 + plv * e2;
            o = o * e1 + pov * e2;
            m = m_new;
        }
        const int w = t & (p_min - 1);
        if (w > 0) {
            const size_t base = (size_t)(t - w) * rs + (size_t)bh * kHeadDim;
            // window key j is w - j positions before the query; stored partial states are already in this query's frame
            attend_keys<T, HP>(q, K + base, V + base, rs, w, scale, m, l, o, HP ? Klo + base : nullptr,
                               alibi_slope(alibi, bh % H, H), w);
        }
    }
    const int b = bh / H, h = bh % H;
    const float a = o / l;
    if (attn_cat) attn_cat[(size_t)b * H * kHeadDim + h * kHeadDim + lane] = a;
    if (op_a) {   // the same value as bf16 head + remainder rows (2b, 2b + 1) for the matrix-core products
        const size_t d = (size_t)H * kHeadDim;
        const bf16_t hi = f32_to_bf16(a);
        op_a[(size_t)(2 * b) * d + h * kHeadDim + lane] = hi;
        op_a[(size_t)(2 * b + 1) * d + h * kHeadDim + lane] = f32_to_bf16(a - bf16_to_f32(hi));
    }
    return a;
}

// =============================================================================================
// The same merge for the layer-wavefront engine's bf16 path with p_min = 32, written for latency: one wavefront per
// (b, h) is all the parallelism there is, so every load is issued before anything is computed - the query and the
// temporary pair, up to kFastLevels stored partial states and the far state (absent ones read slot 0 and get weight
// 0), the window keys (lanes 0..31: head rows, lanes 32..63: remainder rows of the same keys) and the window values
// out of the transposed copy (lane = head dimension, 32 consecutive positions = 64 contiguous bytes) - and the
// softmax over all terms is taken in one pass.  Same value as merge_body up to the order of the sums.
// =============================================================================================
constexpr int kFastLevels = 3;

__device__ __forceinline__ float merge_window32_hp(const float *__restrict__ Qf, const float *__restrict__ Ktf,
                                                   const bf16_t *__restrict__ Vt, const bf16_t *__restrict__ K,
                                                   const bf16_t *__restrict__ Klo, const bf16_t *__restrict__ VT,
                                                   int vt_stride, const float *__restrict__ pm, const float *__restrict__ pl,
                                                   const float *__restrict__ po, int BH, int H, int bh, int t, int levels,
                                                   int slots, float scale, int far_rel, int log2_chunk, float alibi)
{
    const int lane = threadIdx.x & 63;
    const size_t rs = (size_t)BH * kHeadDim;
    const size_t qoff = (size_t)t * rs + (size_t)bh * kHeadDim + lane;
    const float q = Qf[qoff], kt = Ktf[qoff], vt = bf16_to_f32(Vt[qoff]);
    // stored states: levels 5 .. 5 + levels - 1 (bits of t), then the far state
    float sm[kFastLevels + 1], sl[kFastLevels + 1], so[kFastLevels + 1];
#pragma unroll
    for (int lr = 0; lr <= kFastLevels; ++lr) {
        const bool far = lr == kFastLevels;
        const bool on = far ? (far_rel >= 0 && (t >> log2_chunk) > 0) : (lr < levels && ((t >> (lr + 5)) & 1));
        const size_t idx = on ? (far ? partial_index(far_rel, t, slots, BH, bh) : partial_index(lr, partial_slot(lr + 5, t), slots, BH, bh))
                              : (size_t)bh;
        const float m_ = pm[idx], l_ = pl[idx], o_ = po[idx * kHeadDim + lane];
        sm[lr] = on ? m_ : -INFINITY;
        sl[lr] = on ? l_ : 0.f;
        so[lr] = on ? o_ : 0.f;
    }
    // window: keys t - w .. t - 1, w = t mod 32
    const int w = t & 31, j = lane & 31;
    const size_t kbase = (size_t)(t - w + min(j, max(w - 1, 0))) * rs + (size_t)bh * kHeadDim;
    const bf16_t *krow = (lane < 32 ? K : Klo) + kbase;
    uint4 kr[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) kr[c] = *reinterpret_cast<const uint4 *>(krow + 8 * c);
    const bf16_t *vrow = VT + ((size_t)bh * kHeadDim + lane) * vt_stride + (t - w);
    uint4 vr[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) vr[c] = *reinterpret_cast<const uint4 *>(vrow + 8 * c);

    const float m0 = scale * wave_sum(q * kt);
    float acc = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const uint32_t u4[4] = {kr[c].x, kr[c].y, kr[c].z, kr[c].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc = fmaf(lane_bcast(q, 8 * c + 2 * e), __uint_as_float(u4[e] << 16), acc);
            acc = fmaf(lane_bcast(q, 8 * c + 2 * e + 1), __uint_as_float(u4[e] & 0xFFFF0000u), acc);
        }
    }
    acc += __shfl_xor(acc, 32, 64);   // head + remainder
    const float slope = alibi_slope(alibi, bh % H, H);
    const float logit = j < w ? fmaf(-slope, (float)(w - j), acc * scale) : -INFINITY;
    float mx = fmaxf(m0, wave_max(logit));
#pragma unroll
    for (int lr = 0; lr <= kFastLevels; ++lr) mx = fmaxf(mx, sm[lr]);
    const float e0 = expf(m0 - mx);
    float l = e0, o = e0 * vt;
#pragma unroll
    for (int lr = 0; lr <= kFastLevels; ++lr) {
        const float f = expf(sm[lr] - mx);   // exp(-inf) = 0 for absent states
        l = fmaf(sl[lr], f, l);
        o = fmaf(so[lr], f, o);
    }
    const float p = expf(logit - mx);        // 0 beyond the window; lanes 32..63 mirror lanes 0..31
    l += 0.5f * wave_sum(p);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const uint32_t u4[4] = {vr[c].x, vr[c].y, vr[c].z, vr[c].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            o = fmaf(lane_bcast(p, 8 * c + 2 * e), __uint_as_float(u4[e] << 16), o);
            o = fmaf(lane_bcast(p, 8 * c + 2 * e + 1), __uint_as_float(u4[e] & 0xFFFF0000u), o);
        }
    }
    return o / l;
}

// =============================================================================================
// Small-M matrix products of the base case:  out[b][o] = epilogue( sum_k W[o][k] * in[b][k] ),
// b < Bn <= 8.  Bandwidth is the bound (every weight is used for at most 8 multiply-adds), so the
// work is cut for memory parallelism: groups of KS wavefronts own 4 output rows each (a workgroup
// of 4 wavefronts: 16 / KS rows), a wavefront takes every KS-th 512-column slice of the contraction
// (16-byte weight loads, 4 rows in flight), the partial sums meet in LDS in a fixed order (runs are
// bit-reproducible).  KS = 2 for contractions up to 1024 columns (every wavefront then has exactly
// one slice), else 4.  The B input rows come out of L2.  With do_norm the
// input is RMS-normalised: the sum of squares is accumulated from the same values on the way and
// the scale 1/rms is applied to the finished sums (the product is linear in its input); the gain
// multiplies the input elements as they are read.
// Where the rows come from is the caller's: rows.row(o) is the weight row of output o, rows.gain()
// the gain vector (or null).
// =============================================================================================
enum Epi { EPI_WO = 0, EPI_W1 = 1, EPI_W2 = 2, EPI_KV = 3, EPI_MUL = 5 };   // EPI_MUL: out_f = v * res_f (backward pass)

constexpr int kGemvRows = 4;      // output rows per group of wavefronts
constexpr int kGemvPart = kGemvRows * kBatchTile + kBatchTile;   // floats one wavefront leaves in LDS

__device__ __forceinline__ void load8_in(const float *p, float *o) { load8(p, o); }
__device__ __forceinline__ void load8_in(const bf16_t *p, float *o) { load8(p, o); }

template <typename T, typename IN_T, int EPI, int KS, typename Rows>
__device__ __forceinline__ void gemv_body(const Rows &rows, int block, int n_out, int n_in, const IN_T *__restrict__ in,
                                          size_t in_stride, int Bn, float eps, int do_norm, float alpha,
                                          const T *__restrict__ res_T, size_t res_stride, const float *__restrict__ res_f,
                                          float *__restrict__ out_f, T *__restrict__ out_T, size_t out_T_stride,
                                          float (*part)[kGemvPart])
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int kGroups = 4 / KS;   // row groups per workgroup
    const int rg = wave / KS, kw = wave % KS;
    const int o0 = (block * kGroups + rg) * kGemvRows;
    const T *wrow[kGemvRows];
#pragma unroll
    for (int r = 0; r < kGemvRows; ++r) wrow[r] = rows.row(min(o0 + r, n_out - 1));
    const T *gain = rows.gain();
    float acc[kGemvRows][kBatchTile], ssq[kBatchTile];
#pragma unroll
    for (int b = 0; b < kBatchTile; ++b) {
        ssq[b] = 0.f;
#pragma unroll
        for (int r = 0; r < kGemvRows; ++r) acc[r][b] = 0.f;
    }
    for (int k = kw * 512 + lane * 8; k < n_in; k += 512 * KS) {
        float w[kGemvRows][8];
#pragma unroll
        for (int r = 0; r < kGemvRows; ++r) load8(wrow[r] + k, w[r]);
        float g8[8];
        const bool use_g = do_norm && gain != nullptr;
        if (use_g) load8(gain + k, g8);
#pragma unroll
        for (int b = 0; b < kBatchTile; ++b) {
            if (b < Bn) {
                float x8[8];
                load8_in(in + (size_t)b * in_stride + k, x8);
                if (do_norm) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) ssq[b] = fmaf(x8[e], x8[e], ssq[b]);
                    if (use_g) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) x8[e] *= g8[e];
                    }
                }
#pragma unroll
                for (int r = 0; r < kGemvRows; ++r) {
                    float a = acc[r][b];
#pragma unroll
                    for (int e = 0; e < 8; ++e) a = fmaf(w[r][e], x8[e], a);
                    acc[r][b] = a;
                }
            }
        }
    }
#pragma unroll
    for (int b = 0; b < kBatchTile; ++b) {
        ssq[b] = wave_sum(ssq[b]);
#pragma unroll
        for (int r = 0; r < kGemvRows; ++r) acc[r][b] = wave_sum(acc[r][b]);
    }
    if (lane == 0) {
#pragma unroll
        for (int b = 0; b < kBatchTile; ++b) {
            part[wave][kGemvRows * kBatchTile + b] = ssq[b];
#pragma unroll
            for (int r = 0; r < kGemvRows; ++r) part[wave][r * kBatchTile + b] = acc[r][b];
        }
    }
    __syncthreads();
    // 32 threads per row group each finish one (row, batch) pair
    if (tid < kGroups * kGemvRows * kBatchTile) {
        const int grp = tid / (kGemvRows * kBatchTile), pi = tid % (kGemvRows * kBatchTile);
        const int r = pi / kBatchTile, b = pi % kBatchTile;
        const int si = kGemvRows * kBatchTile + b;
        float v = 0.f, tot = 0.f;
#pragma unroll
        for (int j = 0; j < KS; ++j) { v += part[grp * KS + j][pi]; tot += part[grp * KS + j][si]; }
        if (do_norm) v *= rsqrtf(tot / (float)n_in + eps);
        const int o = (block * kGroups + grp) * kGemvRows + r;
        if (o < n_out && b < Bn) {
            if (EPI == EPI_WO) {
                out_f[(size_t)b * n_out + o] = to_f32(res_T[(size_t)b * res_stride + o]) + alpha * v;
            } else if (EPI == EPI_W1) {
                out_f[(size_t)b * n_out + o] = gelu_erf(v);
            } else if (EPI == EPI_W2) {
                const float z = res_f[(size_t)b * n_out + o] + alpha * v;
                out_f[(size_t)b * n_out + o] = z;
                out_T[(size_t)b * out_T_stride + o] = from_f32<T>(z);
            } else if (EPI == EPI_MUL) {
                out_f[(size_t)b * n_out + o] = v * res_f[(size_t)b * n_out + o];
            } else {
                out_f[(size_t)b * n_out + o] = v;
            }
        }
    }
}

// qkRMS of one head's 64 values held one per lane (identity when norm_free); gain may be null.
template <typename T>
__device__ __forceinline__ float head_rms(float v, const T *__restrict__ g, int h, float eps, int norm_free)
{
    if (norm_free) return v;
    const int lane = threadIdx.x & 63;
    return v * rsqrtf(wave_sum(v * v) / (float)kHeadDim + eps) * (g ? to_f32(g[h * kHeadDim + lane]) : 1.f);
}

}  // namespace rt
