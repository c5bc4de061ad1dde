// Exchange primitives of the single-launch (cooperative) engines: self-validating 64-bit words [tag:32 | payload:32]
// written with one 8-byte agent-scope store and polled by their consumers, the thread-linear bulk pull of an exchanged
// vector with its small-M matrix-core product against an LDS-resident weight slice, and the bounded waits.  Shared by
// the forward engine (rt_persistent.hip) and the backward loop (rt_backward_persistent.hip).  The functions that wait
// take the kernel's argument struct as a template parameter; it must have the members spin_limit (long long), bar
// (unsigned long long *: [0] barrier counter, [8] abort word) and pre_sleep (int).
#pragma once
#include "rt_mfma_device.h"

namespace rt {

constexpr int kPW = 8;                 // wavefronts per workgroup
constexpr int kPThreads = kPW * 64;
constexpr int kBMax = 16;              // batch rows (MFMA N dimension)
constexpr int kRMax = 16;              // output rows per workgroup and matrix (MFMA M dimension)

typedef unsigned long long ll_t;       // exchange word: [tag:32 | payload:32]
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// 64-lane all-reduce with DPP inside each row of 16 lanes (no LDS crossbar), rows combined through
// scalar reads.  quad_perm [1,0,3,2] = 0xB1, [2,3,0,1] = 0x4E, row_half_mirror = 0x141, row_mirror = 0x140.
__device__ __forceinline__ float dpp_f(float v, int ctrl_sel)
{
    const int i = __float_as_int(v);
    int r;
    switch (ctrl_sel) {
    case 0: r = __builtin_amdgcn_mov_dpp(i, 0xB1, 0xF, 0xF, true); break;
    case 1: r = __builtin_amdgcn_mov_dpp(i, 0x4E, 0xF, 0xF, true); break;
    case 2: r = __builtin_amdgcn_mov_dpp(i, 0x141, 0xF, 0xF, true); break;
    default: r = __builtin_amdgcn_mov_dpp(i, 0x140, 0xF, 0xF, true); break;
    }
    return __int_as_float(r);
}
// value of lane + 1 for the even lanes (quad_perm [1,1,3,3]): the partner of a bf16 pair without the LDS crossbar
__device__ __forceinline__ float dpp_odd_neighbour(float v)
{
    return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0xF5, 0xF, 0xF, true));
}
// Exchanges between the rows of 16 lanes and between the halves of a wavefront with v_permlane16_swap / v_permlane32_swap
// (one vector instruction each instead of a trip through the LDS crossbar).  swap16(a, b) returns
// {[a row 0, b row 0, a row 2, b row 2], [a row 1, b row 1, a row 3, b row 3]}, swap32(a, b) {[a low, b low], [a high, b high]}.
// next_row: the value of lane + 16 for the lanes of rows 0 and 2 (the other lanes get their own value back).
__device__ __forceinline__ float next_row(float v)
{
    const unsigned u = __float_as_uint(v);
    return __uint_as_float(__builtin_amdgcn_permlane16_swap(u, u, false, false)[1]);
}
__device__ __forceinline__ float xor16(float v)   // value of lane ^ 16
{
    const unsigned u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    return __uint_as_float((threadIdx.x & 16) ? r[0] : r[1]);
}
__device__ __forceinline__ float xor32(float v)   // value of lane ^ 32
{
    const unsigned u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}
__device__ __forceinline__ float fast_sum(float v)
{
    v += dpp_f(v, 0);
    v += dpp_f(v, 1);
    v += dpp_f(v, 2);
    v += dpp_f(v, 3);
    return lane_bcast(v, 0) + lane_bcast(v, 16) + lane_bcast(v, 32) + lane_bcast(v, 48);
}
__device__ __forceinline__ float fast_max(float v)
{
    v = fmaxf(v, dpp_f(v, 0));
    v = fmaxf(v, dpp_f(v, 1));
    v = fmaxf(v, dpp_f(v, 2));
    v = fmaxf(v, dpp_f(v, 3));
    return fmaxf(fmaxf(lane_bcast(v, 0), lane_bcast(v, 16)), fmaxf(lane_bcast(v, 32), lane_bcast(v, 48)));
}

__device__ __forceinline__ ll_t ll_load(const ll_t *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void ll_store(ll_t *p, unsigned tag, unsigned payload)
{
    __hip_atomic_store(p, ((ll_t)tag << 32) | payload, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ bool ll_ok(ll_t w, unsigned tag) { return (unsigned)(w >> 32) == tag; }

// Layout of an exchange vector whose words hold element pairs (k, k+1) of kBMax batch rows: the words one producer
// writes - GW per batch row, all batch rows of its GW*2 elements - are contiguous,
//     word(k, b) = ((k / (2 GW)) * kBMax + b) * GW + (k / 2) % GW,
// so that every 64- or 128-byte line of the vector is written by ONE workgroup.  Measured on MI355X (cfg3, phase
// trace): with rows [b][k], where a line is assembled from the 16-byte pieces of eight workgroups, the h and z
// exchanges took 4.5 us from store to staged operand, against 3.1-3.5 us for the vectors whose producers write 64
// bytes and more in one piece.
template <int GW> __device__ __forceinline__ size_t pair_word(int k, int b)
{
    return ((size_t)(k / (2 * GW)) * kBMax + b) * GW + ((k >> 1) % GW);
}
// the same for vectors of one fp32 per word whose producers own R consecutive elements
template <int R> __device__ __forceinline__ size_t single_word(int o, int b)
{
    return ((size_t)(o / R) * kBMax + b) * R + (o % R);
}

// Wave-uniform bounded poll of one word per lane (inactive lanes pass active = false).
// Returns the word; sets fail when the bound is hit or the abort word is raised.
template <typename ARGS>
__device__ __forceinline__ ll_t ll_wait(const ll_t *p, bool active, unsigned tag, const ARGS &A, int &fail)
{
    ll_t w = active ? ll_load(p) : 0;
    bool bad = active && !ll_ok(w, tag);
    long long spins = 0;
    while (__any(bad)) {
        if (bad) { w = ll_load(p); bad = !ll_ok(w, tag); }
        if (++spins > A.spin_limit || ((spins & 255) == 0 && ll_load(A.bar + 8) != 0)) { fail = 1; break; }
    }
    return w;
}

// Fenced grid-wide barrier on a monotonically increasing counter (used around cross-block events).
// Returns true if the run is aborted.
template <typename ARGS>
__device__ __forceinline__ bool grid_barrier(const ARGS &A, unsigned long long target, int *flag_s)
{
    __syncthreads();
    if (threadIdx.x == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        __hip_atomic_fetch_add(A.bar, 1ULL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int ab = 0;
        long long spins = 0;
        for (;;) {
            const unsigned long long v = ll_load(A.bar);
            if (v >= target) break;
            if (++spins > A.spin_limit || ((spins & 255) == 0 && ll_load(A.bar + 8) != 0)) { ab = 1; break; }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        *flag_s = ab;
    }
    __syncthreads();
    return *flag_s != 0;
}

// acc tile of one workgroup: rows of an LDS-resident weight slice times the activation rows that
// arrive as exchange words act[b][row_words] (this call uses KS*32*kPW elements of each row).
// The words are pulled thread-linearly: consecutive threads fetch consecutive 16-byte chunks (two
// words) with agent-scope buffer loads -- measured on MI355X, 256 workgroups each pulling the same
// 32 KB: 0.82 us this way against 1.4 us for 32-byte pieces per lane and 2.6 us for 128-byte runs per
// lane.  Each word validates itself (a stale chunk is re-polled by its thread); the payloads are
// staged in LDS as plain bf16 rows act_s[b][lda], from which the MFMA B fragments are read.
//     step s of lane (b, g) of wave w  <->  k = w*KS*32 + s*32 + 8g .. +7
// The per-wavefront 16 x 16 tiles land in red[wave][row][b].  With SS the sum of squares of every
// received row goes to ss_s[wave][b] (the consumer's own RMS statistic).
// 16 bytes out of LDS through a pointer the compiler only knows as generic.  The weight slices and staged rows are
// addressed through pointers computed once before the position loop; the compiler kept them as 64-bit generic
// addresses and emitted flat loads (each waited for on both memory counters before its matrix instruction:
// four dependent round trips of about 0.3 us per product).  The low 32 bits of a generic LDS address are the LDS
// offset, so the cast below turns the access into ds_read_b128.
typedef unsigned v4u_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) const v4u_t *lds_v4u_ptr_t;
__device__ __forceinline__ uint4 lds_load16(const void *p)
{
    const v4u_t v = *(lds_v4u_ptr_t)(uintptr_t)p;
    return make_uint4(v[0], v[1], v[2], v[3]);
}

constexpr int kAuxAgent = 16;   // cache-policy operand of the buffer load: sc1 (agent scope)

// Which wavefront pulls which chunks: when a wavefront's share of the contraction (KS * 32 elements of every batch row) is a
// whole number of the layout's blocks (2 GW elements of all batch rows), the words it multiplies are one contiguous eighth of
// the vector, and it pulls exactly those, still consecutive lanes on consecutive 16-byte chunks.  Its product then depends on
// its own staging writes only: no workgroup barrier between pull and product (FULL_SYNC asks for one anyway: callers that
// read whole staged rows afterwards), and a wavefront whose words are in starts multiplying while others still poll.
__device__ __forceinline__ void wave_sync_lds()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
template <int KS, int GW, bool SS = false, bool FULL_SYNC = false, typename ARGS>
__device__ __forceinline__ void wg_gemv_ll(const bf16_t *w_s, int ldw, int R, const ll_t *act, int B,
                                           unsigned tag, const ARGS &A, float *red, bf16_t *act_s, int lda, int &fail,
                                           float *ss_s = nullptr, int pre_sleep_units = -1)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, g = lane >> 4;
    const int pre_sleep = pre_sleep_units >= 0 ? pre_sleep_units : A.pre_sleep;
    constexpr int K = KS * 32 * kPW;
    constexpr int kWords = kBMax * K / 2;                   // words of the vector, unused batch rows included
    constexpr int kMaxChunks = kWords / 2 / kPThreads;      // 16-byte chunks per thread  (= 2 KS)
    constexpr bool kWaveLocal = (KS * 32) % (2 * GW) == 0;
    const int c0 = kWaveLocal ? wave * (kMaxChunks * 64) + lane : tid;   // chunk i of this thread: c0 + i * cstep
    constexpr int cstep = kWaveLocal ? 64 : kPThreads;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<ll_t *>(act), 0, kWords * 8, 0x00020000);
    v4u_t v[kMaxChunks];
    unsigned need = 0;
    // chunk c = words 2c, 2c + 1 of the layout above: batch rows b0, b1 (equal unless GW is odd) and first elements k0, k1
#pragma unroll
    for (int i = 0; i < kMaxChunks; ++i) {
        v[i] = v4u_t{0u, 0u, 0u, 0u};
        const int w0 = 2 * (c0 + i * cstep);
        const int b0 = (w0 % (kBMax * GW)) / GW, b1 = ((w0 + 1) % (kBMax * GW)) / GW;
        if (b0 < B || b1 < B) need |= 1u << i;
    }
    long long spins = 0;
    // A poll that leaves before the producers' stores have landed costs a whole extra trip (about 1.2 us); measured,
    // a quarter of a microsecond of waiting first brings the average number of rounds from 1.5 to 1.1.
    for (int i = 0; i < pre_sleep; ++i) __builtin_amdgcn_s_sleep(4);
    while (__any(need != 0)) {
#pragma unroll
        for (int i = 0; i < kMaxChunks; ++i)
            if (need & (1u << i)) v[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (c0 + i * cstep) * 16, 0, kAuxAgent);
#pragma unroll
        for (int i = 0; i < kMaxChunks; ++i)
            if (need & (1u << i)) {
                const int w0 = 2 * (c0 + i * cstep), w1 = w0 + 1;
                const int b0 = (w0 % (kBMax * GW)) / GW, b1 = (w1 % (kBMax * GW)) / GW;
                const int k0 = 2 * ((w0 / (kBMax * GW)) * GW + w0 % GW), k1 = 2 * ((w1 / (kBMax * GW)) * GW + w1 % GW);
                const bool u0 = b0 < B, u1 = b1 < B;
                if ((!u0 || v[i][1] == tag) && (!u1 || v[i][3] == tag)) {
                    if (GW % 2 == 0) {   // both words belong to one batch row, four consecutive elements
                        *reinterpret_cast<uint2 *>(act_s + (size_t)b0 * lda + k0) = make_uint2(v[i][0], v[i][2]);
                    } else {
                        if (u0) *reinterpret_cast<unsigned *>(act_s + (size_t)b0 * lda + k0) = v[i][0];
                        if (u1) *reinterpret_cast<unsigned *>(act_s + (size_t)b1 * lda + k1) = v[i][2];
                    }
                    need &= ~(1u << i);
                }
            }
        if (++spins > A.spin_limit || ((spins & 255) == 0 && ll_load(A.bar + 8) != 0)) { fail = 1; break; }
    }
    if (kWaveLocal && !FULL_SYNC) wave_sync_lds();
    else __syncthreads();
    const bool has_w = l16 < R, has_a = l16 < B;
    constexpr int kw = KS * 32;
    const bf16_t *wrow = w_s + (size_t)l16 * ldw + wave * kw + 8 * g;
    const bf16_t *arow = act_s + (size_t)l16 * lda + wave * kw + 8 * g;
    f32x4_t acc = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
    float ssp[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        Frag a, b;
        a.u = has_w ? lds_load16(wrow + s * 32) : zero;
        b.u = has_a ? lds_load16(arow + s * 32) : zero;
        acc = mfma16(a, b, acc);
        if (SS) {   // four independent partial sums: one chain of 16 KS dependent multiply-adds is as long as the product
            const unsigned w4[4] = {b.u.x, b.u.y, b.u.z, b.u.w};
#pragma unroll
            for (int h = 0; h < 4; ++h) {   // lo lo + hi hi + sum in one instruction (v_dot2c_f32_bf16)
                const bf16x2_t pr = __builtin_bit_cast(bf16x2_t, w4[h]);
                ssp[h] = __builtin_amdgcn_fdot2_f32_bf16(pr, pr, ssp[h], false);
            }
        }
    }
    if (SS) {
        float ss = (ssp[0] + ssp[1]) + (ssp[2] + ssp[3]);
        ss += xor16(ss);
        ss += xor32(ss);
        if (g == 0) ss_s[wave * kBMax + l16] = ss;
    }
    float *r = red + ((size_t)wave * kRMax + 4 * g) * kBMax + l16;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i * kBMax] = acc[i];
}

// Two exchanged vectors of the same layout against two weight slices, summed: red = w1 act1 + w2 act2.  Both vectors are
// polled in the same rounds (one store-to-load trip for the pair instead of one each); the first is staged as it arrives,
// the second waits in registers until the first product has read the staging rows.
template <int KS, int GW, typename ARGS>
__device__ __forceinline__ void wg_gemv_ll_pair(const bf16_t *w1_s, const bf16_t *w2_s, int ldw, int R, const ll_t *act1,
                                                const ll_t *act2, int B, unsigned tag, const ARGS &A, float *red, bf16_t *act_s,
                                                int lda, int &fail, int pre_sleep_units = -1)
{
    static_assert(GW % 2 == 0, "both words of a chunk belong to one batch row");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, g = lane >> 4;
    constexpr int K = KS * 32 * kPW;
    constexpr int kWords = kBMax * K / 2;
    constexpr int kMaxChunks = kWords / 2 / kPThreads;
    constexpr bool kWaveLocal = (KS * 32) % (2 * GW) == 0;   // see wg_gemv_ll: then the three barriers below are wavefront-local
    const int c0 = kWaveLocal ? wave * (kMaxChunks * 64) + lane : tid;
    constexpr int cstep = kWaveLocal ? 64 : kPThreads;
    const __amdgpu_buffer_rsrc_t rsrc1 = __builtin_amdgcn_make_buffer_rsrc(const_cast<ll_t *>(act1), 0, kWords * 8, 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc2 = __builtin_amdgcn_make_buffer_rsrc(const_cast<ll_t *>(act2), 0, kWords * 8, 0x00020000);
    v4u_t v1[kMaxChunks], v2[kMaxChunks];
    unsigned need1 = 0, need2 = 0;
#pragma unroll
    for (int i = 0; i < kMaxChunks; ++i) {
        v1[i] = v2[i] = v4u_t{0u, 0u, 0u, 0u};
        const int w0 = 2 * (c0 + i * cstep);
        if ((w0 % (kBMax * GW)) / GW < B) need1 |= 1u << i;
    }
    const unsigned mine = need1;
    need2 = need1;
    long long spins = 0;
    const int pre_sleep = pre_sleep_units >= 0 ? pre_sleep_units : A.pre_sleep;
    for (int i = 0; i < pre_sleep; ++i) __builtin_amdgcn_s_sleep(4);
    while (__any((need1 | need2) != 0)) {
#pragma unroll
        for (int i = 0; i < kMaxChunks; ++i) {
            if (need1 & (1u << i)) v1[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc1, (c0 + i * cstep) * 16, 0, kAuxAgent);
            if (need2 & (1u << i)) v2[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc2, (c0 + i * cstep) * 16, 0, kAuxAgent);
        }
#pragma unroll
        for (int i = 0; i < kMaxChunks; ++i) {
            if ((need1 & (1u << i)) && v1[i][1] == tag && v1[i][3] == tag) {
                const int w0 = 2 * (c0 + i * cstep);
                const int b0 = (w0 % (kBMax * GW)) / GW, k0 = 2 * ((w0 / (kBMax * GW)) * GW + w0 % GW);
                *reinterpret_cast<uint2 *>(act_s + (size_t)b0 * lda + k0) = make_uint2(v1[i][0], v1[i][2]);
                need1 &= ~(1u << i);
            }
            if ((need2 & (1u << i)) && v2[i][1] == tag && v2[i][3] == tag) need2 &= ~(1u << i);
        }
        if (++spins > A.spin_limit || ((spins & 255) == 0 && ll_load(A.bar + 8) != 0)) { fail = 1; break; }
    }
    if (kWaveLocal) wave_sync_lds(); else __syncthreads();
    const bool has_w = l16 < R, has_a = l16 < B;
    constexpr int kw = KS * 32;
    const bf16_t *arow = act_s + (size_t)l16 * lda + wave * kw + 8 * g;
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
    f32x4_t acc = f32x4_t{0.f, 0.f, 0.f, 0.f};
    {
        const bf16_t *wrow = w1_s + (size_t)l16 * ldw + wave * kw + 8 * g;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            Frag a, b;
            a.u = has_w ? lds_load16(wrow + s * 32) : zero;
            b.u = has_a ? lds_load16(arow + s * 32) : zero;
            acc = mfma16(a, b, acc);
        }
    }
    if (kWaveLocal) wave_sync_lds(); else __syncthreads();   // the first vector's rows have been read
#pragma unroll
    for (int i = 0; i < kMaxChunks; ++i)
        if (mine & (1u << i)) {
            const int w0 = 2 * (c0 + i * cstep);
            const int b0 = (w0 % (kBMax * GW)) / GW, k0 = 2 * ((w0 / (kBMax * GW)) * GW + w0 % GW);
            *reinterpret_cast<uint2 *>(act_s + (size_t)b0 * lda + k0) = make_uint2(v2[i][0], v2[i][2]);
        }
    if (kWaveLocal) wave_sync_lds(); else __syncthreads();
    {
        const bf16_t *wrow = w2_s + (size_t)l16 * ldw + wave * kw + 8 * g;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            Frag a, b;
            a.u = has_w ? lds_load16(wrow + s * 32) : zero;
            b.u = has_a ? lds_load16(arow + s * 32) : zero;
            acc = mfma16(a, b, acc);
        }
    }
    float *r = red + ((size_t)wave * kRMax + 4 * g) * kBMax + l16;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i * kBMax] = acc[i];
}

// The product half of wg_gemv_ll alone: rows of an LDS-resident weight slice times activation rows that are already
// staged in LDS as bf16 rows act_s[b][lda] (the caller has synchronised).  The per-wavefront 16 x 16 tiles land in
// red[wave][row][b]; with SS the sum of squares of the staged rows goes to ss_s[wave][b].
template <int KS, bool SS = false>
__device__ __forceinline__ void wg_product_staged(const bf16_t *w_s, int ldw, int R, int B, float *red, const bf16_t *act_s, int lda,
                                                  float *ss_s = nullptr)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, g = lane >> 4;
    const bool has_w = l16 < R, has_a = l16 < B;
    constexpr int kw = KS * 32;
    const bf16_t *wrow = w_s + (size_t)l16 * ldw + wave * kw + 8 * g;
    const bf16_t *arow = act_s + (size_t)l16 * lda + wave * kw + 8 * g;
    f32x4_t acc = f32x4_t{0.f, 0.f, 0.f, 0.f};
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
    float ssp[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        Frag a, b;
        a.u = has_w ? lds_load16(wrow + s * 32) : zero;
        b.u = has_a ? lds_load16(arow + s * 32) : zero;
        acc = mfma16(a, b, acc);
        if (SS) {   // four independent partial sums: one chain of 16 KS dependent multiply-adds is as long as the product
            const unsigned w4[4] = {b.u.x, b.u.y, b.u.z, b.u.w};
#pragma unroll
            for (int h = 0; h < 4; ++h) {   // lo lo + hi hi + sum in one instruction (v_dot2c_f32_bf16)
                const bf16x2_t pr = __builtin_bit_cast(bf16x2_t, w4[h]);
                ssp[h] = __builtin_amdgcn_fdot2_f32_bf16(pr, pr, ssp[h], false);
            }
        }
    }
    if (SS) {
        float ss = (ssp[0] + ssp[1]) + (ssp[2] + ssp[3]);
        ss += xor16(ss);
        ss += xor32(ss);
        if (g == 0) ss_s[wave * kBMax + l16] = ss;
    }
    float *r = red + ((size_t)wave * kRMax + 4 * g) * kBMax + l16;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i * kBMax] = acc[i];
}

__device__ __forceinline__ float red_sum(const float *red, int row, int b)
{
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < kPW; ++w) v += red[((size_t)w * kRMax + row) * kBMax + b];
    return v;
}

// rows [row0, row0+nrows), columns [col0, col0+K) of a row-major matrix with leading dimension src_ld
// If `gain` is given the columns are scaled by it (W diag(g), rounded to bf16 once): the RMS gain of a
// product's input is folded into the stationary weights, so the exchanged vectors carry no gain.
__device__ __forceinline__ void copy_rows_to_lds(bf16_t *dst, int ldw, const bf16_t *src, int src_ld, int col0, int K, int row0,
                                                 int nrows, const bf16_t *gain = nullptr)
{
    const int per_row = K / 8;  // 16-byte pieces
    for (int idx = threadIdx.x; idx < nrows * per_row; idx += kPThreads) {
        const int r = idx / per_row, c = idx - r * per_row;
        uint4 w = *reinterpret_cast<const uint4 *>(src + (size_t)(row0 + r) * src_ld + col0 + c * 8);
        if (gain) {
            float gg[8], ww[8];
            load8(gain + col0 + c * 8, gg);
            load8(reinterpret_cast<const bf16_t *>(&w), ww);
            w.x = (unsigned)f32_to_bf16(ww[0] * gg[0]) | ((unsigned)f32_to_bf16(ww[1] * gg[1]) << 16);
            w.y = (unsigned)f32_to_bf16(ww[2] * gg[2]) | ((unsigned)f32_to_bf16(ww[3] * gg[3]) << 16);
            w.z = (unsigned)f32_to_bf16(ww[4] * gg[4]) | ((unsigned)f32_to_bf16(ww[5] * gg[5]) << 16);
            w.w = (unsigned)f32_to_bf16(ww[6] * gg[6]) | ((unsigned)f32_to_bf16(ww[7] * gg[7]) << 16);
        }
        *reinterpret_cast<uint4 *>(dst + (size_t)r * ldw + c * 8) = w;
    }
}

// A copy of weight rows (PER 16-byte pieces each) into LDS in two halves, so that all of a thread's pieces are in flight
// at once and the wavefront can do something else meanwhile: rows_issue requests this thread's NB pieces (src(r): first
// element of row r, or null), rows_commit stores them to LDS rows ldw elements apart, multiplied by gain(r) (an LDS
// row of gains, or null).  NB * kPThreads >= nrows * PER.
template <int NB, int PER, typename SRC>
__device__ __forceinline__ void rows_issue(uint4 (&w)[NB], int nrows, SRC src)
{
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int idx = j * kPThreads + (int)threadIdx.x;
        w[j] = make_uint4(0u, 0u, 0u, 0u);
        if (idx < nrows * PER) {
            const int r = idx / PER, c = idx - r * PER;
            const bf16_t *row = src(r);
            if (row) w[j] = global_load16(row + c * 8);
        }
    }
}
template <int NB, int PER, typename GAIN>
__device__ __forceinline__ void rows_commit(const uint4 (&w)[NB], bf16_t *dst, int ldw, int nrows, GAIN gain)
{
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int idx = j * kPThreads + (int)threadIdx.x;
        if (idx >= nrows * PER) continue;
        const int r = idx / PER, c = idx - r * PER;
        uint4 v = w[j];
        const bf16_t *g = gain(r);
        if (g) {
            const uint4 gq = lds_load16(g + c * 8);
            float gg[8], ww[8];
            load8(reinterpret_cast<const bf16_t *>(&gq), gg);
            load8(reinterpret_cast<const bf16_t *>(&v), ww);
            v.x = pack_bf16(ww[0] * gg[0], ww[1] * gg[1]);
            v.y = pack_bf16(ww[2] * gg[2], ww[3] * gg[3]);
            v.z = pack_bf16(ww[4] * gg[4], ww[5] * gg[5]);
            v.w = pack_bf16(ww[6] * gg[6], ww[7] * gg[7]);
        }
        *reinterpret_cast<uint4 *>(dst + (size_t)r * ldw + c * 8) = v;
    }
}

// Bounded poll of NW words per lane.  Every round re-issues all words that are still stale together and checks
// them together, so a round costs one trip to memory however many words are late (re-polling them one after the
// other cost one trip per late word: measured 2.3 us for the two words of a new key-value pair).
template <int NW, typename ARGS>
__device__ __forceinline__ void ll_wait_n(const ll_t *const (&p)[NW], const bool (&active)[NW], unsigned tag,
                                          const ARGS &A, ll_t (&w)[NW], int &fail)
{
    bool bad[NW];
    bool any_bad = false;
#pragma unroll
    for (int i = 0; i < NW; ++i) w[i] = active[i] ? ll_load(p[i]) : 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        bad[i] = active[i] && !ll_ok(w[i], tag);
        any_bad |= bad[i];
    }
    long long spins = 0;
    while (__any(any_bad)) {
#pragma unroll
        for (int i = 0; i < NW; ++i)
            if (bad[i]) w[i] = ll_load(p[i]);
        any_bad = false;
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            if (bad[i]) bad[i] = !ll_ok(w[i], tag);
            any_bad |= bad[i];
        }
        if (++spins > A.spin_limit || ((spins & 255) == 0 && ll_load(A.bar + 8) != 0)) { fail = 1; break; }
    }
}

}  // namespace rt
