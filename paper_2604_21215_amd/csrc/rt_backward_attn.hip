// The two attention-shaped passes of the backward pass (paper Sec. 6.4) on the matrix cores, bf16 storage:
//   bw_dq_mfma      after the reverse loop: dq_i += scale sum_{j < i} dS_ij k_j over all persistent keys before query i;
//   bw_event_mfma   inside the loop: one block of Algorithm 1 (Appendix C) run backwards - the keys [k0, k0 + P) receive
//                   dV_j += sum_i P_ij dc_i,  dK_j += scale sum_i dS_ij q_i  from the queries [q0, q0 + nq) after them;
// with  P_ij = exp(scale <q_i, k_j> - bias - lse_i),  dP_ij = <dc_i, v_j>,  dS_ij = P_ij (dP_ij - D_i),  D_i = <dc_i, c_i>.
// Both read the fp32 rows of the recompute ([N][B H][64]) and split them into bf16 head + remainder while staging them in
// LDS.  The two products that feed the exponential and the cancellation dP - D (S and dP) take head and remainder of both
// operands (three v_mfma_f32_32x32x16_bf16 products: about 16 significant bits); the products that accumulate the
// gradients take the bf16 heads (the gradients are rounded once to bf16, as in the batched products of the pass).
// Fragment layout as in rt_cross_tile.h: with the "transposed" forms S^T[key][query] (dq) and S[query][key] (event) the
// softmax quantities of a query (or key) sit in one lane column and the weights come out of the accumulator registers
// in B-operand layout.
#include "rt_backward.h"
#include "rt_cross_tile.h"

namespace rt {

namespace {

// 8 floats -> bf16 heads and remainders, packed
__device__ __forceinline__ void split8(const float (&f)[8], uint4 &h, uint4 &l)
{
    uint32_t hw[4], lw[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        hw[e] = cvt_pk_bf16(f[2 * e], f[2 * e + 1]);
        lw[e] = cvt_pk_bf16(f[2 * e] - __uint_as_float(hw[e] << 16), f[2 * e + 1] - __uint_as_float(hw[e] & 0xFFFF0000u));
    }
    h = make_uint4(hw[0], hw[1], hw[2], hw[3]);
    l = make_uint4(lw[0], lw[1], lw[2], lw[3]);
}

// B fragments (head, remainder) of one fp32 row of 64: contraction step ks covers elements 16 ks + 8 hi .. + 7
__device__ __forceinline__ void row_frags(const float *row, int hi, uint4 (&h)[4], uint4 (&l)[4])
{
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        float f[8];
        load8(row + 16 * ks + 8 * hi, f);
        split8(f, h[ks], l[ks]);
    }
}

// 64 rows x 64 fp32 columns (row r at src + r * rs; rows >= nrows are staged as zeros) into LDS: row tiles
// hi_t, lo_t [64][kTileLd] (A operand with the rows as M and the columns as contraction) and, with TR, the heads
// transposed tr_t [64 columns][kVLd] (A operand with the columns as M and the rows as contraction).  256 threads.
template <bool TR>
__device__ __forceinline__ void stage_tile_f32(const float *__restrict__ src, size_t rs, int nrows, bf16_t *hi_t, bf16_t *lo_t,
                                               bf16_t *tr_t, int tid)
{
    const int r = tid >> 2, c16 = (tid & 3) * 16;
    float f[16];
    if (r < nrows) {
        const float *p = src + (size_t)r * rs + c16;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float4 v = *reinterpret_cast<const float4 *>(p + 4 * j);
            f[4 * j] = v.x; f[4 * j + 1] = v.y; f[4 * j + 2] = v.z; f[4 * j + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) f[e] = 0.f;
    }
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        float g[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) g[e] = f[8 * half + e];
        uint4 h, l;
        split8(g, h, l);
        *reinterpret_cast<uint4 *>(hi_t + r * kTileLd + c16 + 8 * half) = h;
        *reinterpret_cast<uint4 *>(lo_t + r * kTileLd + c16 + 8 * half) = l;
        if (TR) {
            const uint32_t hw[4] = {h.x, h.y, h.z, h.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                tr_t[(c16 + 8 * half + 2 * e) * kVLd + r] = (bf16_t)(hw[e] & 0xFFFFu);
                tr_t[(c16 + 8 * half + 2 * e + 1) * kVLd + r] = (bf16_t)(hw[e] >> 16);
            }
        }
    }
}

// acc[32 x 32] = A rows (LDS row tiles hi, lo: rows row0 .. row0 + 31) times the B fragments (head bh, remainder bl):
// lo * head + head * lo + head * head, small terms first
__device__ __forceinline__ f32x16_t product3(const bf16_t *hi_t, const bf16_t *lo_t, int row0, int l32, int hi, const uint4 (&bh)[4],
                                             const uint4 (&bl)[4])
{
    const bf16_t *hr = hi_t + (row0 + l32) * kTileLd + 8 * hi, *lr = lo_t + (row0 + l32) * kTileLd + 8 * hi;
    uint4 ah[4];
    f32x16_t acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        ah[ks] = *reinterpret_cast<const uint4 *>(hr + ks * 16);
        acc = mfma32u(*reinterpret_cast<const uint4 *>(lr + ks * 16), bh[ks], acc);
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) acc = mfma32u(ah[ks], bl[ks], acc);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) acc = mfma32u(ah[ks], bh[ks], acc);
    return acc;
}

// A fragment of a transposed tile: row `row` (an output row of the product), contraction slots of step s4
__device__ __forceinline__ uint4 tr_frag(const bf16_t *tr_t, int row, int s4, int hi)
{
    const bf16_t *p = tr_t + row * kVLd + s4 * 16 + 4 * hi;
    const uint2 v0 = *reinterpret_cast<const uint2 *>(p), v1 = *reinterpret_cast<const uint2 *>(p + 8);
    return make_uint4(v0.x, v0.y, v1.x, v1.y);
}

constexpr int kRowTile = kKC * kTileLd;   // elements
constexpr int kTrTile = kKC * kVLd;

}  // namespace

// ---------------------------------------------------------------------------------------------------------------------
// dq: one workgroup per (128 queries, b, h), four wavefronts of 32 queries; the keys before the tile in chunks of 64.
//   S^T[key][query] = K Q^T,  dP^T[key][query] = V dC^T  (A = key rows out of LDS, B = the wavefront's query / dc rows)
//   dS^T = exp2(S^T c2 + bias - lse2_q) (dP^T - D_q), zero for keys j >= i
//   dQ^T[dh][query] += K^T dS^T   (A = the chunk's keys transposed, B = dS^T straight from the registers)
// grid ceil(N / 128) * B H (numbered like the forward's masked pass: all tiles of a (b, h) on one XCD, longest first),
// block 256, LDS 4 row tiles + 1 transposed tile.
// ---------------------------------------------------------------------------------------------------------------------
template <bool ALIBI>
__global__ __launch_bounds__(256) void bw_dq_mfma_kernel(const float *__restrict__ Qn, const float *__restrict__ Kp,
                                                         const float *__restrict__ Vp, const float *__restrict__ dc,
                                                         const float *__restrict__ lse, const float *__restrict__ Ds,
                                                         float *__restrict__ dq, int BH, int H, int N, int ntiles, float scale,
                                                         float alibi)
{
    extern __shared__ __align__(16) unsigned char bwa_lds[];
    bf16_t *Kh = reinterpret_cast<bf16_t *>(bwa_lds), *Kl = Kh + kRowTile, *Vh = Kl + kRowTile, *Vl = Vh + kRowTile, *KT = Vl + kRowTile;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hi = lane >> 5;
    int bh, qt;
    {
        const int L = blockIdx.x;
        if (BH % 8 == 0) {
            const int xcd = L & 7, idx = L >> 3;
            bh = xcd + 8 * (idx / ntiles);
            qt = ntiles - 1 - idx % ntiles;
        } else {
            bh = L / ntiles;
            qt = ntiles - 1 - L % ntiles;
        }
    }
    const int q0w = qt * 128 + 32 * wave;
    const bool active = q0w < N;            // wave-uniform
    const int qpos = q0w + l32, qi = min(qpos, N - 1);
    const size_t rs = (size_t)BH * kHeadDim;
    const float c2 = scale * kLog2e;
    const float s2 = ALIBI ? alibi_slope(alibi, bh % H, H) * kLog2e : 0.f;

    uint4 bq[4], bql[4], bd[4], bdl[4];
    row_frags(Qn + (size_t)qi * rs + (size_t)bh * kHeadDim, hi, bq, bql);
    row_frags(dc + (size_t)qi * rs + (size_t)bh * kHeadDim, hi, bd, bdl);
    const float lse2 = lse[(size_t)qi * BH + bh] * kLog2e, Dq = Ds[(size_t)qi * BH + bh];
    f32x16_t O[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) O[dt][i] = 0.f;

    const int kend = min(qt * 128 + 128, N) - 1;   // keys 0 .. kend - 1 precede some query of the tile
    for (int kc = 0; kc < kend; kc += kKC) {
        __syncthreads();                            // the previous chunk's tiles are no longer read
        const float *kb = Kp + (size_t)kc * rs + (size_t)bh * kHeadDim, *vb = Vp + (size_t)kc * rs + (size_t)bh * kHeadDim;
        stage_tile_f32<true>(kb, rs, min(kKC, kend - kc), Kh, Kl, KT, tid);
        stage_tile_f32<false>(vb, rs, min(kKC, kend - kc), Vh, Vl, nullptr, tid);
        __syncthreads();
        if (!active || kc >= q0w + 31) continue;    // no key of the chunk precedes a query of this wavefront
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            const f32x16_t S = product3(Kh, Kl, kt * 32, l32, hi, bq, bql);
            const f32x16_t dP = product3(Vh, Vl, kt * 32, l32, hi, bd, bdl);
            // register i: key kc + 32 kt + 8 (i / 4) + 4 hi + i % 4, query qpos
            const int kbase = kc + 32 * kt + 4 * hi;
            float dsv[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int key = kbase + 8 * (i / 4) + (i % 4);
                const float arg = ALIBI ? fmaf(S[i], c2, fmaf(s2, (float)(key - qpos), -lse2)) : fmaf(S[i], c2, -lse2);
                const float p = key < qpos ? __builtin_amdgcn_exp2f(arg) : 0.f;
                dsv[i] = p * (dP[i] - Dq);
            }
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const uint4 bs = make_uint4(cvt_pk_bf16(dsv[8 * s], dsv[8 * s + 1]), cvt_pk_bf16(dsv[8 * s + 2], dsv[8 * s + 3]),
                                            cvt_pk_bf16(dsv[8 * s + 4], dsv[8 * s + 5]), cvt_pk_bf16(dsv[8 * s + 6], dsv[8 * s + 7]));
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) O[dt] = mfma32u(tr_frag(KT, dt * 32 + l32, 2 * kt + s, hi), bs, O[dt]);
            }
        }
    }
    if (active && qpos < N) {
        // register i of tile dt: head dimension 32 dt + 8 (i / 4) + 4 hi + i % 4
        float *row = dq + (size_t)qpos * rs + (size_t)bh * kHeadDim + 4 * hi;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float4 v = *reinterpret_cast<float4 *>(row + dt * 32 + 8 * j);
                v.x = fmaf(scale, O[dt][4 * j], v.x); v.y = fmaf(scale, O[dt][4 * j + 1], v.y);
                v.z = fmaf(scale, O[dt][4 * j + 2], v.z); v.w = fmaf(scale, O[dt][4 * j + 3], v.w);
                *reinterpret_cast<float4 *>(row + dt * 32 + 8 * j) = v;
            }
    }
}

// ---------------------------------------------------------------------------------------------------------------------
// One block of Algorithm 1 backwards: a workgroup owns 128 keys of one (b, h) (four wavefronts of 32), walks the block's
// queries in chunks of 64:
//   S[query][key] = Q K^T,  dP[query][key] = dC V^T   (A = query / dc rows out of LDS, B = the wavefront's key / value rows)
//   Pm = exp2(S c2 + bias - lse2_q),  dS = Pm (dP - D_q)   (rows past the last query are zero)
//   dV^T[dh][key] += dC^T Pm,  dK^T[dh][key] += Q^T dS   (A = the chunk's dc / q rows transposed, B = Pm, dS from registers)
// Every query of the block lies after every key: no mask.  grid (ceil(P / 128), B H), block 256.
// ---------------------------------------------------------------------------------------------------------------------
template <bool ALIBI>
__global__ __launch_bounds__(256) void bw_event_mfma_kernel(const float *__restrict__ Qn, const float *__restrict__ Kp,
                                                            const float *__restrict__ Vp, const float *__restrict__ dc,
                                                            const float *__restrict__ lse, const float *__restrict__ Ds,
                                                            float *__restrict__ dK, float *__restrict__ dV, int BH, int H, int k0,
                                                            int P, int q0, int nq, float scale, float alibi)
{
    extern __shared__ __align__(16) unsigned char bwa_lds[];
    bf16_t *Qh = reinterpret_cast<bf16_t *>(bwa_lds), *Ql = Qh + kRowTile, *Ch = Ql + kRowTile, *Cl = Ch + kRowTile;
    bf16_t *QT = Cl + kRowTile, *CT = QT + kTrTile;
    float *lse_s = reinterpret_cast<float *>(CT + kTrTile), *D_s = lse_s + kKC;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, hi = lane >> 5;
    const int bh = blockIdx.y, kw = k0 + blockIdx.x * 128 + 32 * wave;
    const bool active = kw < k0 + P;        // wave-uniform
    const int kpos = kw + l32, ki = min(kpos, k0 + P - 1);
    const size_t rs = (size_t)BH * kHeadDim;
    const float c2 = scale * kLog2e;
    const float s2 = ALIBI ? alibi_slope(alibi, bh % H, H) * kLog2e : 0.f;

    uint4 bk[4], bkl[4], bv[4], bvl[4];
    row_frags(Kp + (size_t)ki * rs + (size_t)bh * kHeadDim, hi, bk, bkl);
    row_frags(Vp + (size_t)ki * rs + (size_t)bh * kHeadDim, hi, bv, bvl);
    f32x16_t aK[2], aV[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) aK[dt][i] = aV[dt][i] = 0.f;

    for (int qc = 0; qc < nq; qc += kKC) {
        const int nqc = min(kKC, nq - qc);
        __syncthreads();
        const size_t ro = (size_t)(q0 + qc) * rs + (size_t)bh * kHeadDim;
        stage_tile_f32<true>(Qn + ro, rs, nqc, Qh, Ql, QT, tid);
        stage_tile_f32<true>(dc + ro, rs, nqc, Ch, Cl, CT, tid);
        if (tid < kKC) {
            const size_t o = (size_t)(q0 + qc + min(tid, nqc - 1)) * BH + bh;
            lse_s[tid] = lse[o] * kLog2e;
            D_s[tid] = Ds[o];
        }
        __syncthreads();
        if (!active) continue;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            const f32x16_t S = product3(Qh, Ql, kt * 32, l32, hi, bk, bkl);
            const f32x16_t dP = product3(Ch, Cl, kt * 32, l32, hi, bv, bvl);
            // register i: query (of the chunk) 32 kt + 8 (i / 4) + 4 hi + i % 4, key kpos
            float pv[16], dsv[16];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int qr = 32 * kt + 8 * j + 4 * hi;
                const float4 l4 = *reinterpret_cast<const float4 *>(lse_s + qr), d4 = *reinterpret_cast<const float4 *>(D_s + qr);
                const float ls[4] = {l4.x, l4.y, l4.z, l4.w}, dd[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int i = 4 * j + e, qrel = qr + e;
                    const float arg = ALIBI ? fmaf(S[i], c2, fmaf(s2, (float)(kpos - (q0 + qc + qrel)), -ls[e])) : fmaf(S[i], c2, -ls[e]);
                    const float p = qrel < nqc ? __builtin_amdgcn_exp2f(arg) : 0.f;
                    pv[i] = p;
                    dsv[i] = p * (dP[i] - dd[e]);
                }
            }
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const uint4 bp = make_uint4(cvt_pk_bf16(pv[8 * s], pv[8 * s + 1]), cvt_pk_bf16(pv[8 * s + 2], pv[8 * s + 3]),
                                            cvt_pk_bf16(pv[8 * s + 4], pv[8 * s + 5]), cvt_pk_bf16(pv[8 * s + 6], pv[8 * s + 7]));
                const uint4 bs = make_uint4(cvt_pk_bf16(dsv[8 * s], dsv[8 * s + 1]), cvt_pk_bf16(dsv[8 * s + 2], dsv[8 * s + 3]),
                                            cvt_pk_bf16(dsv[8 * s + 4], dsv[8 * s + 5]), cvt_pk_bf16(dsv[8 * s + 6], dsv[8 * s + 7]));
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) {
                    aV[dt] = mfma32u(tr_frag(CT, dt * 32 + l32, 2 * kt + s, hi), bp, aV[dt]);
                    aK[dt] = mfma32u(tr_frag(QT, dt * 32 + l32, 2 * kt + s, hi), bs, aK[dt]);
                }
            }
        }
    }
    if (active && kpos < k0 + P) {
        float *rk = dK + (size_t)kpos * rs + (size_t)bh * kHeadDim + 4 * hi, *rv = dV + (size_t)kpos * rs + (size_t)bh * kHeadDim + 4 * hi;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float4 a = *reinterpret_cast<float4 *>(rk + dt * 32 + 8 * j), b = *reinterpret_cast<float4 *>(rv + dt * 32 + 8 * j);
                a.x = fmaf(scale, aK[dt][4 * j], a.x); a.y = fmaf(scale, aK[dt][4 * j + 1], a.y);
                a.z = fmaf(scale, aK[dt][4 * j + 2], a.z); a.w = fmaf(scale, aK[dt][4 * j + 3], a.w);
                b.x += aV[dt][4 * j]; b.y += aV[dt][4 * j + 1]; b.z += aV[dt][4 * j + 2]; b.w += aV[dt][4 * j + 3];
                *reinterpret_cast<float4 *>(rk + dt * 32 + 8 * j) = a;
                *reinterpret_cast<float4 *>(rv + dt * 32 + 8 * j) = b;
            }
    }
}

// ---------------------------------------------------------------------------------------------------------------------
constexpr size_t kDqMfmaLds = (size_t)(4 * kRowTile + kTrTile) * 2;
constexpr size_t kEventMfmaLds = (size_t)(4 * kRowTile + 2 * kTrTile) * 2 + 2 * kKC * 4;

hipError_t bw_attn_mfma_init()
{
    static bool done = false;
    if (done) return hipSuccess;
    const void *fns[4] = {(const void *)bw_dq_mfma_kernel<false>, (const void *)bw_dq_mfma_kernel<true>,
                          (const void *)bw_event_mfma_kernel<false>, (const void *)bw_event_mfma_kernel<true>};
    const size_t lds[4] = {kDqMfmaLds, kDqMfmaLds, kEventMfmaLds, kEventMfmaLds};
    for (int i = 0; i < 4; ++i) {
        const hipError_t e = hipFuncSetAttribute(fns[i], hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds[i]);
        if (e != hipSuccess) return e;
    }
    done = true;
    return hipSuccess;
}

hipError_t bw_dq_mfma(const LayerDims &D, const float *Qn, const float *Kp, const float *Vp, const float *dc, const float *lse,
                      const float *Ds, float *dq, hipStream_t st)
{
    const int BH = D.B * D.H, ntiles = (D.N + 127) / 128;
    const dim3 grid((unsigned)(ntiles * BH));
    if (D.alibi > 0.f)
        hipLaunchKernelGGL(bw_dq_mfma_kernel<true>, grid, dim3(256), kDqMfmaLds, st, Qn, Kp, Vp, dc, lse, Ds, dq, BH, D.H, D.N, ntiles,
                           D.scale, D.alibi);
    else
        hipLaunchKernelGGL(bw_dq_mfma_kernel<false>, grid, dim3(256), kDqMfmaLds, st, Qn, Kp, Vp, dc, lse, Ds, dq, BH, D.H, D.N, ntiles,
                           D.scale, D.alibi);
    return hipGetLastError();
}

hipError_t bw_event_mfma(const LayerDims &D, const float *Qn, const float *Kp, const float *Vp, const float *dc, const float *lse,
                         const float *Ds, float *dK, float *dV, int k0, int P, int q0, int nq, hipStream_t st)
{
    const int BH = D.B * D.H;
    const dim3 grid((unsigned)((P + 127) / 128), (unsigned)BH);
    if (D.alibi > 0.f)
        hipLaunchKernelGGL(bw_event_mfma_kernel<true>, grid, dim3(256), kEventMfmaLds, st, Qn, Kp, Vp, dc, lse, Ds, dK, dV, BH, D.H, k0, P,
                           q0, nq, D.scale, D.alibi);
    else
        hipLaunchKernelGGL(bw_event_mfma_kernel<false>, grid, dim3(256), kEventMfmaLds, st, Qn, Kp, Vp, dc, lse, Ds, dK, dV, BH, D.H, k0, P,
                           q0, nq, D.scale, D.alibi);
    return hipGetLastError();
}

}  // namespace rt
