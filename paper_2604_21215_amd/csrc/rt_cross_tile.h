// Cross-block UpdateTile (Appendix C, Algorithm 2) with the key and value tiles staged in LDS and shared by
// all wavefronts of a workgroup: NW wavefronts x 32 queries of one (b, h) against the P keys of the block.
//
// Per chunk of 64 keys the workgroup copies K[64][64] (and, for high-precision logits, the remainder
// tile) and V^T[64][64] into LDS once (next chunk prefetched into registers while the current one is
// being used); each wavefront then forms, with v_mfma_f32_32x32x16_bf16 (measured on MI355X: 2.1 PFLOP/s
// against 1.2-1.3 PFLOP/s for the 16x16x32 form),
//     S^T[key][query] = K Q^T          (A = K rows out of LDS, B = this wavefront's Q rows, registers)
//     O^T[dh][query] += V^T P^T        (A = V^T rows out of LDS, B = P^T straight from the S^T registers)
// Operand layout of v_mfma_f32_32x32x16_bf16 (A 32x16, B 16x32, hi = lane/32):
//   A: lane holds A[row = lane%32][k = 8hi .. 8hi+7],  B: lane holds B[k = 8hi .. 8hi+7][col = lane%32],
//   D: register i of a lane holds D[row = 8(i/4) + 4hi + i%4][col = lane%32], i = 0..15.
// Eight consecutive D registers 8s .. 8s+7 of a lane are therefore the keys 16s + 4hi + (0..3) and
// 16s + 8 + 4hi + (0..3) of one query: packed to bf16 they are the B fragment of contraction step s when
// the V^T fragment is gathered with the same key <-> slot assignment (two 8-byte reads).
// The softmax keeps one reference value per query (not necessarily the running maximum): it is moved up,
// and the accumulators rescaled, only when a logit exceeds it by more than kSlack (powers of two), which
// after the first chunk is rare.  Any reference gives the same (m, l, o) triple up to rounding (Algorithm 2
// tracks the maximum for stability only); p <= 2^kSlack keeps everything far from overflow.  The row sums
// l are accumulated with plain additions of the unrounded weights.  Measured on MI355X: the exponential
// and the bf16 dot-product instructions do not run beside the matrix pipeline, multiply-add, max3, add and
// the bf16 pair conversion do; the core clock is about 1.7 GHz while this kernel runs.
#pragma once
#include "rt_mfma_device.h"

namespace rt {

constexpr int kKC = 64;            // keys per chunk
constexpr int kTileLd = 72;        // LDS row stride of the key tiles in bf16 elements (64 + 8: 16-byte reads of 16 rows hit distinct banks)
constexpr int kVLd = 68;           // row stride of the V^T tile (8-byte reads of 32 rows hit distinct banks)
constexpr float kSlack = 16.f;     // how far (log2 units) a logit may exceed the reference before it is moved
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// one buffer (V^T tile padded to the key tiles' size); F16: the key tile holds fp16(head + remainder), no remainder tile
template <bool HP, bool F16 = HP> constexpr int cross_tile_lds_bytes() { return (HP && !F16 ? 3 : 2) * kKC * kTileLd * 2; }

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi)
{   // hardware round-to-nearest-even pair conversion
    f32x2_t v = {lo, hi};
    bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
    return *reinterpret_cast<uint32_t *>(&b);
}

typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
__device__ __forceinline__ uint32_t cvt_pk_f16(float lo, float hi)
{   // round-to-nearest-even pair conversion to fp16
    f32x2_t v = {lo, hi};
    f16x2_t h = __builtin_convertvector(v, f16x2_t);
    return __builtin_bit_cast(uint32_t, h);
}

typedef float f32x16_t __attribute__((ext_vector_type(16)));
__device__ __forceinline__ f32x16_t mfma32h(const uint4 &a, const uint4 &b, f32x16_t c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}
__device__ __forceinline__ f32x16_t mfma32u(const uint4 &a, const uint4 &b, f32x16_t c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}
// All 64 * NW threads of the workgroup must call this together (it contains workgroup barriers).
//   q0:       first query (relative to the block's first query) of this wavefront; wavefronts with q0 >= nq idle
//   lds:      NBUF * cross_tile_lds_bytes<HP>() bytes, 16-byte aligned; NBUF = 2 double-buffers the tiles
//   tid:      threadIdx.x (a caller inside a long loop may pass it through an opaque copy, so that nothing derived
//             from it is hoisted out of that loop and kept in registers)
// Query j sits in row (c_first + q_shift + j) of Q / Qf and its partial goes to the slot of (level, c_first + j).
// P is a multiple of 64.
// ALIBI (linear positional bias, slope per head): inside the tile the bias is taken relative to the block's last
// key, slope * (j - j_last) <= 0, the same for every query; the stored maximum is moved into the query's own frame
// when it is written (m -= slope * (i_query - j_last)).  The reference value then follows the biased logits.
// HP: logits from unrounded operands.  With F16 (the default for HP) queries (Qf, fp32) and keys are rounded ONCE to
// fp16 - 11 significant bits against bf16's 8; elements of unit-RMS heads are far inside fp16's range - and S^T is one
// v_mfma_f32_32x32x16_f16 product: the matrix work and the memory traffic of the plain bf16 tile with an eighth of its
// logit rounding.  The fp16 keys are then passed in the Klo argument ([N][B][H][64], Scratch::Kh) and K is not read.
// Without F16 the keys come as bf16 head K plus bf16 remainder Klo and go through three bf16 products
// (K_lo Q_hi + K_hi Q_lo + K_hi Q_hi, 16 significant bits, twice the matrix instructions of the whole chunk).
// VAR (bits): 1 = FOLD: with fp16 logits and no bias the factor scale * log2(e) goes into the fp16 queries and the
// accumulators of S^T start from minus the reference value, so the matrix product delivers S - m directly and the
// per-logit multiply-add before the exponential disappears (the reference moves rarely; then S is corrected by the
// difference).  2 = DOT: the row sums are taken from the bf16 weights that also multiply V (pairs through
// v_dot2c_f32_bf16 against (1, 1): 16 instead of 32 additions per chunk, and o / l then uses one set of weights).
// 4 = PRIO: a wavefront lowers its issue priority by one step per quarter of its chunks (see the chunk loop).
// Measured on MI355X (P = 1024 event, 128 (b, h), stand-alone launches): 51.0 us without, 49.8 us with FOLD, 51.2 us
// with DOT, 49.9 us with both: the instruction count of the softmax is not what bounds the tile.  Stamps at the start
// and end of every workgroup (all 1024 start within 0.6 us): lifetimes 22.6 .. 46.1 us, median 34.7 - the four
// wavefronts of a SIMD finish one after the other; with PRIO 33.7 .. 43.7 us and the launch ends at 43.9 instead of
// 46.3 us (512 keys: 16.2 instead of 17.2 us; no gain below 8 chunks).  One wavefront alone on a SIMD needs 1.55 us
// per chunk, two 1.69 us each, four 2.2 us each.  A whole cfg3 prefill of the persistent engine, whose tiles run inline:
// 35.88 ms without, 35.63 ms with FOLD, 36.68 ms with FOLD and PRIO.  FOLD is on everywhere, PRIO in stand-alone launches.
constexpr int kCtVarDefault = 5;
template <bool HP, int NW, int NBUF, bool ALIBI = false, bool F16 = HP, int VAR = kCtVarDefault>
__device__ __forceinline__ void cross_tile_wg(const bf16_t *__restrict__ Q, const float *__restrict__ Qf,
                                              const bf16_t *__restrict__ K, const bf16_t *__restrict__ Klo,
                                              const bf16_t *__restrict__ VT, int vt_stride, float *__restrict__ pm,
                                              float *__restrict__ pl, float *__restrict__ po, int BH, int bh, int c_first,
                                              int q_shift, int k_first, int P, int q0, int nq, int level, int level_rel,
                                              int slots, float scale, unsigned char *lds, int tid, float slope = 0.f)
{
    constexpr int T = 64 * NW;
    constexpr int kPieces = kKC * 8;              // 16-byte pieces of one 64 x 64 bf16 tile
    constexpr int PPT = (kPieces + T - 1) / T;    // pieces per thread and tile
    constexpr int TILE = kKC * kTileLd;           // elements of one LDS tile
    constexpr int BUF = (HP && !F16 ? 3 : 2) * TILE;
    const int lane = tid & 63;
    const int l32 = lane & 31, hi = lane >> 5;
    const size_t rs = (size_t)BH * kHeadDim;
    bf16_t *tiles = reinterpret_cast<bf16_t *>(lds);
    const bool active = q0 < nq;   // wave-uniform
    const float c2 = scale * kLog2e;
    constexpr bool FOLD = (VAR & 1) && HP && F16 && !ALIBI;
    constexpr bool DOT = (VAR & 2) != 0;
    constexpr bool PRIO = (VAR & 4) != 0 && NBUF == 2;   // stand-alone launches only: inside the persistent kernel it cost 3 % of a call

    // ---- this wavefront's 32 queries as B fragments (contraction step ks covers head dimensions 16ks .. 16ks+15)
    uint4 bq[4], bql[4];
    {
        const int qi = min(q0 + l32, nq - 1);
        const size_t qo = (size_t)(c_first + q_shift + qi) * rs + (size_t)bh * kHeadDim + 8 * hi;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (HP && F16) {
                float f[8];
                load8(Qf + qo + ks * 16, f);
                if (FOLD) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) f[e] *= c2;
                }
                bq[ks] = make_uint4(cvt_pk_f16(f[0], f[1]), cvt_pk_f16(f[2], f[3]), cvt_pk_f16(f[4], f[5]), cvt_pk_f16(f[6], f[7]));
            } else if (HP) {
                float f[8], r[8];
                load8(Qf + qo + ks * 16, f);
                uint32_t h2[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    h2[e] = cvt_pk_bf16(f[2 * e], f[2 * e + 1]);
                    r[2 * e] = f[2 * e] - __uint_as_float(h2[e] << 16);
                    r[2 * e + 1] = f[2 * e + 1] - __uint_as_float(h2[e] & 0xFFFF0000u);
                }
                bq[ks] = make_uint4(h2[0], h2[1], h2[2], h2[3]);
                bql[ks] = make_uint4(cvt_pk_bf16(r[0], r[1]), cvt_pk_bf16(r[2], r[3]), cvt_pk_bf16(r[4], r[5]), cvt_pk_bf16(r[6], r[7]));
            } else {
                bq[ks] = *reinterpret_cast<const uint4 *>(Q + qo + ks * 16);
            }
        }
    }

    // The query loads are issued before any key/value load: waiting for the first chunk then also covers them, and
    // the loop never has to wait on the memory counter for a query fragment (which would also wait for the chunk
    // that has just been requested).
    __builtin_amdgcn_sched_barrier(0);

    // ---- global -> register -> LDS staging of one chunk (thread -> 16-byte piece: 8 consecutive threads cover one row)
    u32x4_t rk[PPT], rl[PPT], rv[PPT];   // native vectors: these must stay in registers across the chunk's work
    const int prow = tid >> 3, pc16 = tid & 7;                    // piece i of this thread: row prow + i * (T / 8)
    const bf16_t *gk = K + (size_t)(k_first + prow) * rs + (size_t)bh * kHeadDim + pc16 * 8;
    const bf16_t *gl = HP ? Klo + (size_t)(k_first + prow) * rs + (size_t)bh * kHeadDim + pc16 * 8 : nullptr;
    const bf16_t *gv = VT + ((size_t)bh * kHeadDim + prow) * vt_stride + k_first + pc16 * 8;
    const int lds_off = prow * kTileLd + pc16 * 8, lds_off_v = prow * kVLd + pc16 * 8;
#define RT_CT_FETCH(kc)                                                                                              \
    _Pragma("unroll") for (int i = 0; i < PPT; ++i)                                                                  \
    {                                                                                                                \
        if (kPieces % T == 0 || tid + i * T < kPieces) {                                                             \
            if (HP && F16) rk[i] = *reinterpret_cast<const u32x4_t *>(gl + (size_t)((kc) + i * (T / 8)) * rs);       \
            else rk[i] = *reinterpret_cast<const u32x4_t *>(gk + (size_t)((kc) + i * (T / 8)) * rs);                  \
            if (HP && !F16) rl[i] = *reinterpret_cast<const u32x4_t *>(gl + (size_t)((kc) + i * (T / 8)) * rs);       \
            rv[i] = *reinterpret_cast<const u32x4_t *>(gv + (size_t)(i * (T / 8)) * vt_stride + (kc));                 \
        }                                                                                                            \
    }
#define RT_CT_STAGE(buf)                                                                                             \
    _Pragma("unroll") for (int i = 0; i < PPT; ++i)                                                                  \
    {                                                                                                                \
        if (kPieces % T == 0 || tid + i * T < kPieces) {                                                             \
            bf16_t *dst = tiles + (size_t)(buf) * BUF + lds_off + i * (T / 8) * kTileLd;                             \
            *reinterpret_cast<u32x4_t *>(dst) = rk[i];                                                               \
            {                                                                                                        \
                bf16_t *dv = tiles + (size_t)(buf) * BUF + TILE + lds_off_v + i * (T / 8) * kVLd;                    \
                *reinterpret_cast<uint2 *>(dv) = make_uint2(rv[i][0], rv[i][1]);                                     \
                *reinterpret_cast<uint2 *>(dv + 4) = make_uint2(rv[i][2], rv[i][3]);                                 \
            }                                                                                                        \
            if (HP && !F16) *reinterpret_cast<u32x4_t *>(dst + 2 * TILE) = rl[i];                                    \
        }                                                                                                            \
    }

    // reference value m2 (log2 units; the two lanes that share a query hold the same value), row sum l (each of
    // the two lanes sums its own keys), accumulators O^T (2 tiles of 32 head dimensions x 32 queries)
    float m2 = -INFINITY, lsum = 0.f;
    f32x16_t O[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[dt][i] = 0.f;

    RT_CT_FETCH(0)
    RT_CT_STAGE(0)
    __syncthreads();
    const int nchunks = P / kKC;
    for (int c = 0; c < nchunks; ++c) {
        const int cur = (NBUF == 2) ? (c & 1) : 0;
        if (PRIO && nchunks >= 8 && (4 * c) % nchunks == 0) {
            // The issue arbiter of a SIMD prefers its oldest wavefront, which then runs at its solo speed and leaves early
            // while the youngest takes twice as long, and the SIMD spends the second half of the launch with one to three
            // wavefronts instead of four.  A wavefront lowers its own priority as it gets ahead: those behind catch up.
            switch ((4 * c) / nchunks) {
            case 0: __builtin_amdgcn_s_setprio(3); break;
            case 1: __builtin_amdgcn_s_setprio(2); break;
            case 2: __builtin_amdgcn_s_setprio(1); break;
            default: __builtin_amdgcn_s_setprio(0); break;
            }
        }
        if (c + 1 < nchunks) { RT_CT_FETCH((c + 1) * kKC) }
        if (active) {
            const bf16_t *Ks = tiles + (size_t)cur * BUF, *Vs = Ks + TILE, *Kl = Ks + 2 * TILE;
            // ---- S^T = K Q^T for 64 keys x 32 queries (fragments are read next to their use: the kernel runs four
            // wavefronts per SIMD within 128 registers, and the other wavefronts cover the LDS latency)
            f32x16_t S[2];
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                const bf16_t *krow = Ks + (kt * 32 + l32) * kTileLd + 8 * hi;
                uint4 ka[4];
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) ka[ks] = *reinterpret_cast<const uint4 *>(krow + ks * 16);
                f32x16_t acc;
                const float init = FOLD ? (c == 0 ? 0.f : -m2) : 0.f;   // m2 is finite after the first chunk
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[i] = init;
                if (HP && F16) {
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) acc = mfma32h(ka[ks], bq[ks], acc);
                } else {
                if (HP) {   // small terms first
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks)
                        acc = mfma32u(*reinterpret_cast<const uint4 *>(krow + (Kl - Ks) + ks * 16), bq[ks], acc);
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) acc = mfma32u(ka[ks], bql[ks], acc);
                }
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) acc = mfma32u(ka[ks], bq[ks], acc);
                }
                S[kt] = acc;
            }
            if (ALIBI) {
                // register i of tile kt is key 64c + 32kt + 8(i/4) + 4hi + i%4 of the block; from here on S holds the
                // biased logits in log2 units (c2 is applied here instead of below)
                const float s2 = slope * kLog2e;
                const float base = s2 * (float)(c * kKC + 4 * hi - (P - 1));
#pragma unroll
                for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        S[kt][i] = fmaf(S[kt][i], c2, fmaf(s2, (float)(32 * kt + 8 * (i / 4) + (i % 4)), base));
            }
            const float c2e = (ALIBI || FOLD) ? 1.f : c2;   // what still multiplies S below
            // ---- move the reference where a logit runs more than kSlack ahead of it (always on the first chunk)
            float lmax = fmaxf(fmaxf(S[0][0], S[0][1]), S[0][2]);
#pragma unroll
            for (int i = 3; i < 15; i += 2) lmax = fmaxf(fmaxf(lmax, S[0][i]), S[0][i + 1]);
            lmax = fmaxf(fmaxf(lmax, S[0][15]), S[1][0]);
#pragma unroll
            for (int i = 1; i < 15; i += 2) lmax = fmaxf(fmaxf(lmax, S[1][i]), S[1][i + 1]);
            lmax = fmaxf(lmax, S[1][15]) * c2e;
            // FOLD: S is relative to the reference it started from (0 on the first chunk, m2 afterwards)
            const bool over = FOLD ? (c == 0 || lmax > kSlack) : lmax > m2 + kSlack;
            if (__any(over)) {
                const float mx = fmaxf(lmax, __shfl_xor(lmax, 32, 64));
                if (FOLD) {
                    const float rel_old = c == 0 ? -INFINITY : 0.f;
                    const float rel_new = fmaxf(rel_old, mx);
                    const float resc = __builtin_amdgcn_exp2f(rel_old - rel_new);
                    m2 = (c == 0 ? 0.f : m2) + rel_new;
                    lsum *= resc;
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt) O[dt] *= resc;
#pragma unroll
                    for (int kt = 0; kt < 2; ++kt) S[kt] -= rel_new;
                } else {
                const float m_new = fmaxf(m2, mx);
                const float resc = __builtin_amdgcn_exp2f(m2 - m_new);   // exp2(-inf) = 0 on the first chunk
                m2 = m_new;
                lsum *= resc;
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) O[dt] *= resc;
                }
            }
            // ---- P^T = exp2(S^T c2 - m2), packed: registers 8s .. 8s+7 of tile kt are the B fragment of step 2kt + s
            uint4 bp[4];
            const float nm = -m2;
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                float p[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float sv = S[s4 >> 1][8 * (s4 & 1) + e];
                    p[e] = FOLD ? __builtin_amdgcn_exp2f(sv) : __builtin_amdgcn_exp2f(fmaf(sv, c2e, nm));
                }
                bp[s4] = make_uint4(cvt_pk_bf16(p[0], p[1]), cvt_pk_bf16(p[2], p[3]), cvt_pk_bf16(p[4], p[5]), cvt_pk_bf16(p[6], p[7]));
                if (DOT) {
                    const bf16x2_t ones = __builtin_bit_cast(bf16x2_t, 0x3F803F80u);
                    lsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, bp[s4].x), ones, lsum, false);
                    lsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, bp[s4].y), ones, lsum, false);
                    lsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, bp[s4].z), ones, lsum, false);
                    lsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, bp[s4].w), ones, lsum, false);
                } else {
                // plain adds: they run beside the matrix pipeline, which the dot-product and exponential instructions do not
                lsum += ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
                }
            }
            // ---- O^T += V^T P^T
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) {
                    const bf16_t *vrow = Vs + (dt * 32 + l32) * kVLd + s4 * 16 + 4 * hi;
                    const uint2 v0 = *reinterpret_cast<const uint2 *>(vrow), v1 = *reinterpret_cast<const uint2 *>(vrow + 8);
                    O[dt] = mfma32u(make_uint4(v0.x, v0.y, v1.x, v1.y), bp[s4], O[dt]);
                }
            }
        }
        if (c + 1 < nchunks) {
            if (NBUF == 1) __syncthreads();   // everyone is done reading the single buffer
            RT_CT_STAGE((NBUF == 2) ? (cur ^ 1) : 0)
            __syncthreads();
        }
    }

    if (active) {
        const float l = lsum + __shfl_xor(lsum, 32, 64);
        const int qi = q0 + l32;
        if (qi < nq) {
            const size_t idx = partial_index(level_rel, partial_slot(level, c_first + qi), slots, BH, bh);
            if (hi == 0) {
                pm[idx] = ALIBI ? m2 * kLn2 - slope * (float)(c_first + q_shift + qi - (k_first + P - 1)) : m2 * kLn2;
                pl[idx] = l;
            }
            // register i of tile dt is head dimension 32dt + 8(i/4) + 4hi + i%4
            float *orow = po + idx * kHeadDim + 4 * hi;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    *reinterpret_cast<float4 *>(orow + dt * 32 + 8 * j) =
                        make_float4(O[dt][4 * j], O[dt][4 * j + 1], O[dt][4 * j + 2], O[dt][4 * j + 3]);
        }
    }
}

#undef RT_CT_FETCH
#undef RT_CT_STAGE

}  // namespace rt
