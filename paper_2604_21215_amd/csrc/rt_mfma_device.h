// Device-side core of the bf16 MFMA kernels (gfx950), shared by the stand-alone kernels and the
// single-launch engine.
//
// Operand layout of v_mfma_f32_16x16x32_bf16 (D = A*B + C, A 16x32, B 32x16, 64 lanes, g = lane/16):
//   A: lane holds A[row = lane%16][k = 8g .. 8g+7]          (8 bf16 = 16 bytes)
//   B: lane holds B[k = 8g .. 8g+7][col = lane%16]
//   D: lane holds D[row = 4g + r][col = lane%16], r = 0..3   (4 fp32)
#pragma once
#include "rt_common.h"

namespace rt {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

union Frag {
    uint4 u;
    uint2 h[2];
    bf16x8_t v;
};

__device__ __forceinline__ f32x4_t mfma16(const Frag &a, const Frag &b, f32x4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}


// One wavefront's share of a cross-block UpdateTile (Appendix C, Algorithm 2): 32 queries against the
// P keys [k_first, k_first + P) of one (b, h); P is a multiple of 32.  Query j of the block sits in row
// (c_first + q_shift + j) of Q and its partial state goes to the slot of (level, c_first + j).
// The transposed products are formed so that the softmax state of a query lives in one lane column:
//     S^T[key][query] = K Q^T              (A = K rows, B = Q rows)
//     O^T[dh][query] += V^T P^T            (A = V^T rows from the transposed value copy, B = P^T)
// P^T comes out of the first product already in the B-operand layout once the 32 keys of a chunk
// are assigned to contraction slots as  slot 8g+e  <->  key 4g+e (e < 4), 16+4g+(e-4) (e >= 4);
// the V^T fragment is gathered with the same assignment (two 8-byte loads).
// With HP (high-precision logits) the queries come as fp32 rows Qf and are split into a bf16 head and a
// bf16 remainder, the keys come as head K plus remainder Klo, and S^T = Khi Qhi + Khi Qlo + Klo Qhi:
// the logits then carry no bf16 rounding of q or k (they are sharp here: |q| = |k| = 8, and every
// rounding of a logit input shows up as a few per cent on individual softmax weights).
// ALIBI: the logit of key j is lowered by slope * (distance to the query).  Inside the tile the bias is taken
// relative to the block's last key (slope * (j - j_last) <= 0, the same for every query), and the stored maximum
// is moved into the query's own frame when it is written: m -= slope * (i_query - j_last).
template <bool HP, bool ALIBI = false>
__device__ __forceinline__ void cross_mfma_wave(const bf16_t *Q, const float *Qf, const bf16_t *K, const bf16_t *Klo,
                                                const bf16_t *VT, int vt_stride, float *pm, float *pl, float *po, int BH,
                                                int bh, int c_first, int q_shift, int k_first, int P, int q0, int nq,
                                                int level, int level_rel, int slots, float scale, float slope = 0.f)
{
    const int lane = threadIdx.x & 63;
    const int l16 = lane & 15, g = lane >> 4;
    const size_t rs = (size_t)BH * kHeadDim;

    Frag bq[2][2], bql[2][2];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        const int qi = min(q0 + qt * 16 + l16, nq - 1);
        const size_t qo = (size_t)(c_first + q_shift + qi) * rs + (size_t)bh * kHeadDim + 8 * g;
        if (HP) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                float f[8], r[8];
                load8(Qf + qo + ks * 32, f);
#pragma unroll
                for (int e = 0; e < 8; ++e) r[e] = f[e] - bf16_to_f32(f32_to_bf16(f[e]));
                bq[qt][ks].u = make_uint4(pack_bf16(f[0], f[1]), pack_bf16(f[2], f[3]), pack_bf16(f[4], f[5]), pack_bf16(f[6], f[7]));
                bql[qt][ks].u = make_uint4(pack_bf16(r[0], r[1]), pack_bf16(r[2], r[3]), pack_bf16(r[4], r[5]), pack_bf16(r[6], r[7]));
            }
        } else {
            bq[qt][0].u = *reinterpret_cast<const uint4 *>(Q + qo);
            bq[qt][1].u = *reinterpret_cast<const uint4 *>(Q + qo + 32);
        }
    }
    float m[2] = {-INFINITY, -INFINITY}, lsum[2] = {0.f, 0.f};
    f32x4_t O[2][4];
#pragma unroll
    for (int qt = 0; qt < 2; ++qt)
#pragma unroll
        for (int blk = 0; blk < 4; ++blk) O[qt][blk] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    const bf16_t *kbase = K + (size_t)k_first * rs + (size_t)bh * kHeadDim + 8 * g;
    const bf16_t *klbase = HP ? Klo + (size_t)k_first * rs + (size_t)bh * kHeadDim + 8 * g : nullptr;
    const bf16_t *vbase = VT + ((size_t)bh * kHeadDim + l16) * vt_stride + k_first + 4 * g;
    for (int kc = 0; kc < P; kc += 32) {
        f32x4_t S[2][2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            const bf16_t *krow = kbase + (size_t)(kc + kt * 16 + l16) * rs;
            Frag a0, a1, l0, l1;
            a0.u = *reinterpret_cast<const uint4 *>(krow);
            a1.u = *reinterpret_cast<const uint4 *>(krow + 32);
            if (HP) {
                const bf16_t *klrow = klbase + (size_t)(kc + kt * 16 + l16) * rs;
                l0.u = *reinterpret_cast<const uint4 *>(klrow);
                l1.u = *reinterpret_cast<const uint4 *>(klrow + 32);
            }
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                f32x4_t s = f32x4_t{0.f, 0.f, 0.f, 0.f};
                if (HP) {   // small terms first
                    s = mfma16(l0, bq[qt][0], s);
                    s = mfma16(l1, bq[qt][1], s);
                    s = mfma16(a0, bql[qt][0], s);
                    s = mfma16(a1, bql[qt][1], s);
                }
                s = mfma16(a0, bq[qt][0], s);
                s = mfma16(a1, bq[qt][1], s);
                S[qt][kt] = s;
            }
        }
        Frag bp[2];
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            float s[8];
#pragma unroll
            for (int r = 0; r < 4; ++r) { s[r] = S[qt][0][r] * scale; s[4 + r] = S[qt][1][r] * scale; }
            if (ALIBI) {   // element r of tile kt is key kc + 16 kt + 4g + r of the block
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    s[r] = fmaf(slope, (float)(kc + 4 * g + r - (P - 1)), s[r]);
                    s[4 + r] = fmaf(slope, (float)(kc + 16 + 4 * g + r - (P - 1)), s[4 + r]);
                }
            }
            float mx = s[0];
#pragma unroll
            for (int e = 1; e < 8; ++e) mx = fmaxf(mx, s[e]);
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m[qt], mx);
            const float resc = __expf(m[qt] - m_new);
            float ps = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) { s[e] = __expf(s[e] - m_new); ps += s[e]; }
            lsum[qt] = lsum[qt] * resc + ps;
            m[qt] = m_new;
#pragma unroll
            for (int blk = 0; blk < 4; ++blk) O[qt][blk] *= resc;
            bp[qt].u.x = pack_bf16(s[0], s[1]);
            bp[qt].u.y = pack_bf16(s[2], s[3]);
            bp[qt].u.z = pack_bf16(s[4], s[5]);
            bp[qt].u.w = pack_bf16(s[6], s[7]);
        }
#pragma unroll
        for (int blk = 0; blk < 4; ++blk) {
            const bf16_t *vrow = vbase + (size_t)(blk * 16) * vt_stride + kc;
            Frag av;
            av.h[0] = *reinterpret_cast<const uint2 *>(vrow);
            av.h[1] = *reinterpret_cast<const uint2 *>(vrow + 16);
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) O[qt][blk] = mfma16(av, bp[qt], O[qt][blk]);
        }
    }

#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        float l = lsum[qt];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        const int qi = q0 + qt * 16 + l16;
        if (qi < nq) {
            const size_t idx = partial_index(level_rel, partial_slot(level, c_first + qi), slots, BH, bh);
            if (g == 0) {
                // ALIBI: query row c_first + q_shift + qi is that many positions after the block's last key
                pm[idx] = ALIBI ? m[qt] - slope * (float)(c_first + q_shift + qi - (k_first + P - 1)) : m[qt];
                pl[idx] = l;
            }
            float *orow = po + idx * kHeadDim + 4 * g;
#pragma unroll
            for (int blk = 0; blk < 4; ++blk)
                *reinterpret_cast<float4 *>(orow + blk * 16) =
                    make_float4(O[qt][blk][0], O[qt][blk][1], O[qt][blk][2], O[qt][blk][3]);
        }
    }
}

}  // namespace rt
