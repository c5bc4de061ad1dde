// C ABI of the RT layer library: context, validation, and the host-side schedule driver
// (Appendix C, Algorithm 1) that enqueues every phase on one HIP stream.
#include "../../include/rt.h"
#include "rt_common.h"
#include "rt_persistent.h"
#include "rt_decode_persistent.h"
#include "rt_backward.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

using namespace rt;

struct rt_ctx {
    rt_config cfg;
    LayerDims base;      // B, N, kv_cap filled per call
    Scratch S;
    void *slab = nullptr;
    size_t slab_bytes = 0;
    hipStream_t stream = nullptr;
    bool use_mfma = false;
    bool broken = false;
    int last_B = 0, last_N = 0;   // shape of the last prefill (what the scratch holds)
    // K and V of one batch chunk, [max_seq][chunk][d] each: a batch beyond the single-launch engine's rows runs as
    // chunks of that many rows, whose pairs are copied into the caller's position-major cache afterwards
    void *kv_chunk = nullptr;
    size_t kv_chunk_bytes = 0;
    bool last_hp = false;         // that prefill formed high-precision logits (scratch holds unrounded queries and key remainders)
    std::string err;
    std::string engine;
    PersistentState persist;
    DecodeCoopState dec;             // single-launch decoding step
    // layer-wavefront engine: one scratch set per layer and the device copy of the layer descriptors
    void *stack_slab = nullptr;
    size_t stack_bytes = 0;
    int stack_L = 0, stack_chunk = 0;
    std::vector<Scratch> stack_S;
    WaveLayer *stack_dev = nullptr;
    WaveStreams wave_streams = {};   // st[1..], ev[..] created on first use
    void *par_slab = nullptr;        // activations of the loop-free evaluations (rt_layer_recompute, rt_transformer_layer)
    size_t par_bytes = 0;
    void *bw_slab = nullptr;         // scratch of rt_layer_backward
    BwpState bw_loop;                // its single-launch reverse loop
    size_t bw_bytes = 0;
    // cached HIP graph of one stepwise prefill
    hipGraphExec_t graph_exec = nullptr;
    hipStream_t capture_stream = nullptr;  // the legacy default stream cannot be captured
    struct GraphKey {
        const void *x, *y, *K, *V;
        rt_layer_weights w;
        int B, N, kv_cap;
    } graph_key;
};

static const char *kNoCtx = "no context";

static rt_status fail(rt_ctx *c, rt_status s, const char *fmt, const char *detail = "")
{
    if (c) {
        char buf[512];
        snprintf(buf, sizeof(buf), fmt, detail);
        c->err = buf;
    }
    return s;
}
static rt_status fail_hip(rt_ctx *c, hipError_t e, const char *where)
{
    if (c) {
        c->err = std::string(where) + ": " + hipGetErrorString(e);
        c->broken = true;
    }
    return RT_ERR_HIP;
}

// RT_FLAG_DEBUG_POISON: every partial softmax state (m, l, o) of a scratch set becomes NaN before a call, so that a state
// that is read before the call has written it shows up in the outputs.
__global__ __launch_bounds__(256) void poison_f32_kernel(float *__restrict__ p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = __uint_as_float(0x7FC00000u);
}
static void poison_partials(const rt_ctx *c, const Scratch &S)
{
    if (!(c->cfg.flags & RT_FLAG_DEBUG_POISON) || !S.pm) return;
    const size_t np = (size_t)S.levels * S.slots * c->cfg.max_batch * c->cfg.n_heads;
    auto grid = [](size_t n) { return dim3((unsigned)((n + 255) / 256 < 2048 ? (n + 255) / 256 : 2048)); };
    hipLaunchKernelGGL(poison_f32_kernel, grid(np), dim3(256), 0, c->stream, S.pm, np);
    hipLaunchKernelGGL(poison_f32_kernel, grid(np), dim3(256), 0, c->stream, S.pl, np);
    hipLaunchKernelGGL(poison_f32_kernel, grid(np * kHeadDim), dim3(256), 0, c->stream, S.po, np * kHeadDim);
}

static int ilog2(int v)
{
    int l = 0;
    while ((1 << (l + 1)) <= v) ++l;
    return l;
}
static bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }
static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Lays one scratch set out from `base` (may be null: sizes only) and returns its size in bytes.
static size_t layout_scratch(Scratch &S, char *base, size_t Bm, size_t Nm, size_t d, size_t F, size_t H, size_t E, bool mfma,
                             int levels, int slots, bool packed_weights = false)
{
    memset(&S, 0, sizeof(S));
    S.levels = levels;
    S.slots = slots;
    S.vt_stride = (int)align_up(Nm, 64);
    size_t off = 0;
    auto carve = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    const size_t oQ = carve(Nm * Bm * d * E), oKt = carve(Nm * Bm * d * E), oVt = carve(Nm * Bm * d * E);
    const size_t oVT = mfma ? carve(Bm * H * kHeadDim * (size_t)S.vt_stride * 2) : 0;
    const size_t oQf = mfma ? carve(Nm * Bm * d * 4) : 0, oKtf = mfma ? carve(Nm * Bm * d * 4) : 0;
    const size_t oKlo = mfma ? carve(Nm * Bm * d * 2) : 0;
    const size_t oKh = mfma ? carve(Nm * Bm * d * 2) : 0;
    const size_t np = (size_t)levels * slots * Bm * H;
    const size_t opm = carve(np * 4), opl = carve(np * 4), opo = carve(np * kHeadDim * 4);
    const size_t orinv = carve(Bm * Nm * 4);
    const size_t ocat = carve(Bm * d * 4), oh = carve(Bm * d * 4), ou = carve(Bm * F * 4), oz = carve(Bm * d * 4);
    const size_t okv = carve(Bm * 2 * d * 4), oqkv = carve(Bm * 3 * d * 4);
    const size_t oopa = carve(2 * Bm * d * 2), ooph = carve(2 * Bm * d * 2), oopz = carve(2 * Bm * d * 2);
    const size_t oopu = carve(2 * Bm * F * 2);
    const size_t osh = carve(Bm * (d / 16 + 1) * 4), osz = carve(Bm * (d / 16 + 1) * 4);
    const size_t oopx = carve(2 * Bm * d * 2), osx = carve(Bm * (d / 16 + 1) * 4);
    const size_t owg = mfma ? carve(3 * d * d * 2) : 0;
    const size_t owo = packed_weights ? carve(d * d * 2) : 0, ow1 = packed_weights ? carve(F * d * 2) : 0;
    const size_t ow2 = packed_weights ? carve(d * F * 2) : 0, owkv = packed_weights ? carve(2 * d * d * 2) : 0;
    if (base) {
        char *p = base;
        S.Q = p + oQ; S.Kt = p + oKt; S.Vt = p + oVt;
        S.VT = mfma ? (bf16_t *)(p + oVT) : nullptr;
        S.Qf = mfma ? (float *)(p + oQf) : nullptr;
        S.Ktf = mfma ? (float *)(p + oKtf) : nullptr;
        S.Klo = mfma ? (bf16_t *)(p + oKlo) : nullptr;
        S.Kh = mfma ? (uint16_t *)(p + oKh) : nullptr;
        S.pm = (float *)(p + opm); S.pl = (float *)(p + opl); S.po = (float *)(p + opo);
        S.rinv = (float *)(p + orinv);
        S.attn_cat = (float *)(p + ocat); S.h = (float *)(p + oh); S.u = (float *)(p + ou); S.z = (float *)(p + oz);
        S.kv_raw = (float *)(p + okv);
        S.qkv_raw = (float *)(p + oqkv);
        S.op_a = (bf16_t *)(p + oopa); S.op_h = (bf16_t *)(p + ooph); S.op_z = (bf16_t *)(p + oopz);
        S.op_u = (bf16_t *)(p + oopu);
        S.ssq_h = (float *)(p + osh); S.ssq_z = (float *)(p + osz);
        S.op_x = (bf16_t *)(p + oopx); S.ssq_x = (float *)(p + osx);
        S.wg_qkv = mfma ? (bf16_t *)(p + owg) : nullptr;
        if (packed_weights) {
            S.wp_o = (bf16_t *)(p + owo); S.wp_1 = (bf16_t *)(p + ow1); S.wp_2 = (bf16_t *)(p + ow2);
            S.wp_kv = (bf16_t *)(p + owkv);
        }
    }
    return off;
}

// Checks every field of a configuration that does not need the device; p_min and the kernel family it selects are returned.
static rt_status validate_config(const rt_config *cfg, int *p_min_out, bool *mfma_out)
{
    if (cfg->d_model <= 0 || cfg->n_heads <= 0 || cfg->head_dim <= 0 || cfg->d_hidden <= 0 || cfg->max_batch <= 0 ||
        cfg->max_seq <= 0 || (int64_t)cfg->n_heads * cfg->head_dim != cfg->d_model)
        return RT_ERR_INVALID_ARG;
    if (cfg->dtype != RT_F32 && cfg->dtype != RT_BF16) return RT_ERR_INVALID_ARG;
    if (cfg->head_dim != kHeadDim || cfg->d_hidden % 8 != 0) return RT_ERR_UNSUPPORTED;
    if (cfg->max_seq > (1 << 20) || cfg->max_batch > 1024) return RT_ERR_UNSUPPORTED;
    if ((cfg->flags & RT_FLAG_ENGINE_STEPWISE) && (cfg->flags & RT_FLAG_ENGINE_PERSISTENT)) return RT_ERR_INVALID_ARG;
    const bool mfma = cfg->dtype == RT_BF16 && !(cfg->flags & RT_FLAG_NO_MFMA);
    const int p_min = cfg->p_min == 0 ? 32 : cfg->p_min;
    if (!is_pow2(p_min) || p_min > 1024 || (mfma && p_min < 32)) return RT_ERR_INVALID_ARG;
    if (!(cfg->rms_eps >= 0.f) || !(cfg->attn_scale == cfg->attn_scale) || !(cfg->resid_scale == cfg->resid_scale))
        return RT_ERR_INVALID_ARG;
    if (!(cfg->alibi_max_bias >= 0.f) || !(cfg->alibi_max_bias <= 1024.f)) return RT_ERR_INVALID_ARG;
    *p_min_out = p_min;
    *mfma_out = mfma;
    return RT_OK;
}

static void fill_dims(LayerDims &D, const rt_config &cfg, int p_min)
{
    D.B = 0; D.N = 0; D.kv_cap = 0;
    D.d = cfg.d_model; D.H = cfg.n_heads; D.F = cfg.d_hidden;
    D.p_min = p_min; D.log2_pmin = ilog2(p_min);
    D.alpha = cfg.resid_scale; D.scale = cfg.attn_scale; D.eps = cfg.rms_eps;
    D.norm_free = (cfg.flags & RT_FLAG_NORM_FREE) ? 1 : 0;
    D.alibi = cfg.alibi_max_bias;
}

static rt_status stack_workspace(rt_ctx *c, int L, int chunk);
// rt_layer_prefill: from this many sequences on a position of all sequences at once, with batched matrix products, is faster
// than chunks of 16 rows on the single-launch engine (MI355X, d = 1024, 512 positions: 5 chunks take 39.3 ms, 6 take 47.1;
// the batched steps 40.8 ms at B = 80, 41.3 at B = 96, 42.4 at B = 128)
constexpr int kBatchedFrom = 81;
// ... and between these batch sizes the layer-wavefront engine with a single layer (its small-M products on the matrix cores, a
// batch tile of 16 rows per workgroup) is faster than both (same shapes, ms per call at B = 48 / 56 / 64 / 80 / 128 / 160: chunks
// 23.6 / 30.7 / 31.4 / 39.3 / - / -, batched steps 35.4 / 37.5 / 39.8 / 40.5 / 41.7 / 48.4, this engine 28.5 / 28.3 / 29.2 / 30.9 /
// 33.2 / 49.2)
constexpr int kWaveFrom = 49, kWaveTo = 128;

// Scratch of the loop-free evaluations / of the backward pass for max_batch x max_seq positions: allocated once, at
// rt_create when rt_config.reserve asks for it, else by the first call that needs it.
static rt_status ensure_loop_free_scratch(rt_ctx *c)
{
    if (c->par_slab) return RT_OK;
    const size_t Mmax = (size_t)c->cfg.max_batch * c->cfg.max_seq;
    LayerDims D = c->base;
    const bool fast = c->cfg.dtype == RT_BF16 && parallel_supported(D, c->use_mfma);
    const size_t need = fast ? parallel_scratch_bytes(Mmax, c->cfg.d_model, c->cfg.d_hidden)
                             : Launch<float>::loop_free_scratch_bytes(Mmax, c->cfg.d_model, c->cfg.d_hidden);
    hipError_t e = hipMalloc(&c->par_slab, need);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        c->par_slab = nullptr;
        return fail(c, e == hipErrorOutOfMemory ? RT_ERR_OOM : RT_ERR_HIP, "activation scratch: %s", hipGetErrorString(e));
    }
    c->par_bytes = need;
    return RT_OK;
}
static rt_status ensure_backward_scratch(rt_ctx *c)
{
    if (c->bw_slab) return RT_OK;
    const size_t E = c->cfg.dtype == RT_BF16 ? 2 : 4;
    const size_t need = backward_scratch_bytes((size_t)c->cfg.max_batch, (size_t)c->cfg.max_seq, (size_t)c->cfg.d_model,
                                               (size_t)c->cfg.d_hidden, (size_t)c->cfg.n_heads, E);
    hipError_t e = hipMalloc(&c->bw_slab, need);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        c->bw_slab = nullptr;
        return fail(c, e == hipErrorOutOfMemory ? RT_ERR_OOM : RT_ERR_HIP, "backward scratch: %s", hipGetErrorString(e));
    }
    c->bw_bytes = need;
    size_t xo = 0, xb = 0;
    backward_exchange_region((size_t)c->cfg.max_batch, (size_t)c->cfg.max_seq, (size_t)c->cfg.d_model, (size_t)c->cfg.d_hidden,
                             (size_t)c->cfg.n_heads, E, &xo, &xb);
    if (xb > 0) {
        e = hipMemset((char *)c->bw_slab + xo, 0, xb);
        if (e != hipSuccess) return fail_hip(c, e, "backward scratch");
        (void)bwp_create(c->bw_loop, c->cfg.device, c->cfg.d_model, c->cfg.d_hidden, c->cfg.n_heads, c->cfg.max_batch,
                         c->use_mfma && !(c->cfg.flags & RT_FLAG_ENGINE_STEPWISE));
    }
    return RT_OK;
}

extern "C" {

int32_t rt_version(void) { return 100; }

const char *rt_status_string(rt_status s)
{
    switch (s) {
    case RT_OK: return "RT_OK";
    case RT_ERR_INVALID_ARG: return "RT_ERR_INVALID_ARG";
    case RT_ERR_UNSUPPORTED: return "RT_ERR_UNSUPPORTED";
    case RT_ERR_OOM: return "RT_ERR_OOM";
    case RT_ERR_HIP: return "RT_ERR_HIP";
    case RT_ERR_STATE: return "RT_ERR_STATE";
    }
    return "RT_ERR_?";
}

int32_t rt_schedule_events(int32_t N, int32_t p_min, int32_t *out, int32_t cap)
{
    if (N < 1 || !is_pow2(p_min)) return -1;
    int32_t n = 0;
    for (int32_t t = 1; t < N; ++t) {
        const int32_t P = t & -t;
        if (P < p_min) continue;
        if (out && n < cap) {
            int32_t *r = out + 5 * (size_t)n;
            r[0] = t; r[1] = P; r[2] = t + 1; r[3] = (t + P < N) ? t + P : N; r[4] = t - P + 1;
        }
        ++n;
    }
    return n;
}

int32_t rt_schedule_events_shifted(int32_t N, int32_t p_min, int32_t *out, int32_t cap)
{
    if (N < 1 || !is_pow2(p_min)) return -1;
    int32_t n = 0;
    // 0-based position t of the engine's loop: block of keys [t-P, t) serves queries c = t .. t+nq-1 (rows c+1)
    for (int32_t t = p_min; t < N - 1; ++t) {
        const int32_t P = t & -t;
        if (P < p_min) continue;
        const int32_t nq = (P < N - 1 - t) ? P : N - 1 - t;
        if (out && n < cap) {
            int32_t *r = out + 5 * (size_t)n;
            r[0] = t; r[1] = P; r[2] = t + 2; r[3] = t + 1 + nq; r[4] = t - P + 1;
        }
        ++n;
    }
    return n;
}

int32_t rt_schedule_events_chunked(int32_t N, int32_t p_min, int32_t chunk, int32_t *out, int32_t cap)
{
    if (N < 1 || !is_pow2(p_min) || !is_pow2(chunk) || chunk < p_min) return -1;
    int32_t n = 0;
    for (int32_t t = 1; t < N; ++t) {
        int32_t P = t & -t;
        int32_t v = (t + P < N) ? t + P : N, s = t - P + 1;
        if (P >= chunk) { v = (t + chunk < N) ? t + chunk : N; s = 1; P = t; }   // far tile: every key so far
        else if (P < p_min) continue;
        if (out && n < cap) {
            int32_t *r = out + 5 * (size_t)n;
            r[0] = t; r[1] = P; r[2] = t + 1; r[3] = v; r[4] = s;
        }
        ++n;
    }
    return n;
}

int64_t rt_partial_slot(int32_t level, int32_t query)
{
    if (level < 0 || level > 30 || query < 1) return -1;
    const int i0 = query - 1;
    if (!((i0 >> level) & 1)) return -1;
    return partial_slot(level, i0);
}

rt_status rt_create(const rt_config *cfg, rt_ctx **out)
{
    if (out) *out = nullptr;
    if (!cfg || !out) return RT_ERR_INVALID_ARG;
    int p_min = 0;
    bool mfma = false;
    const rt_status vs = validate_config(cfg, &p_min, &mfma);
    if (vs != RT_OK) return vs;

    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || cfg->device < 0 || cfg->device >= ndev) return RT_ERR_HIP;
    if (hipSetDevice(cfg->device) != hipSuccess) return RT_ERR_HIP;

    rt_ctx *c = new (std::nothrow) rt_ctx();
    if (!c) return RT_ERR_OOM;
    c->cfg = *cfg;
    c->cfg.p_min = p_min;
    c->stream = (hipStream_t)cfg->stream;
    c->use_mfma = mfma;
    LayerDims &D = c->base;
    fill_dims(D, c->cfg, p_min);

    const size_t E = cfg->dtype == RT_BF16 ? 2 : 4;
    const size_t Bm = cfg->max_batch, Nm = cfg->max_seq, d = cfg->d_model, F = cfg->d_hidden, H = cfg->n_heads;
    Scratch &S = c->S;
    const int lvmax = Nm >= 2 ? ilog2((int)Nm - 1) : 0;
    int levels = lvmax - D.log2_pmin + 1;
    if (levels < 1) levels = 1;
    int slots = (int)((Nm + 1) / 2);
    if (slots < 64) slots = 64;
    c->slab_bytes = layout_scratch(S, nullptr, Bm, Nm, d, F, H, E, mfma, levels, slots);
    hipError_t e = hipMalloc(&c->slab, c->slab_bytes);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        delete c;
        return e == hipErrorOutOfMemory ? RT_ERR_OOM : RT_ERR_HIP;
    }
    layout_scratch(S, (char *)c->slab, Bm, Nm, d, F, H, E, mfma, levels, slots);
    if (S.VT) {   // tiles read whole 64-position chunks of the transposed values: positions never written must hold finite values
        e = hipMemset(S.VT, 0, Bm * H * kHeadDim * (size_t)S.vt_stride * 2);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            (void)hipFree(c->slab);
            delete c;
            return RT_ERR_HIP;
        }
    }

    rt_status ps = persistent_create(c->persist, c->cfg, D);
    if (ps != RT_OK && (cfg->flags & RT_FLAG_ENGINE_PERSISTENT)) {
        (void)hipFree(c->slab);
        delete c;
        return ps;
    }
    if (c->persist.available && c->cfg.max_batch > c->persist.max_batch) {
        const size_t two = 2 * Nm * (size_t)c->persist.max_batch * d * E;
        if (hipMalloc(&c->kv_chunk, two) == hipSuccess) c->kv_chunk_bytes = two;
        else { (void)hipGetLastError(); c->kv_chunk = nullptr; }   // such batches then never run in chunks
    }
    (void)decode_coop_create(c->dec, c->cfg, D);   // shapes it does not cover keep the multi-launch step
    // scratch of the other entry points, when the caller wants no allocation inside a later call
    rt_status rs = RT_OK;
    if (cfg->reserve_stack_layers > 0) {
        const int chunk = cfg->reserve_stack_chunk == 0 ? 64 : cfg->reserve_stack_chunk;
        const int chunk_min = mfma ? 64 : p_min;
        if (cfg->reserve_stack_layers > 4096 || !is_pow2(chunk) || chunk < chunk_min || chunk < p_min || chunk > (1 << 20))
            rs = RT_ERR_INVALID_ARG;
        else
            rs = stack_workspace(c, cfg->reserve_stack_layers, chunk);
    }
    const bool batched_prefill = cfg->max_batch >= kBatchedFrom && cfg->dtype == RT_BF16 && !(cfg->flags & RT_FLAG_ENGINE_STEPWISE) &&
                                 !(cfg->flags & RT_FLAG_ENGINE_PERSISTENT) && parallel_supported(D, c->use_mfma);
    if (rs == RT_OK && (cfg->reserve & RT_RESERVE_LOOP_FREE)) rs = ensure_loop_free_scratch(c);
    if (rs == RT_OK && batched_prefill && ensure_loop_free_scratch(c) != RT_OK) c->err.clear();   // such batches then run in chunks
    const bool wave_prefill = cfg->max_batch >= kWaveFrom && cfg->dtype == RT_BF16 && !(cfg->flags & RT_FLAG_ENGINE_STEPWISE) &&
                              !(cfg->flags & RT_FLAG_ENGINE_PERSISTENT) && p_min <= 64 &&
                              wavefront_uses_matrix_cores(cfg->d_model, cfg->d_hidden, c->use_mfma);
    if (rs == RT_OK && wave_prefill && !c->stack_slab && stack_workspace(c, 1, 64) != RT_OK) c->err.clear();
    if (rs == RT_OK && (cfg->reserve & RT_RESERVE_BACKWARD)) rs = ensure_backward_scratch(c);
    if (rs != RT_OK) {
        (void)rt_destroy(c);
        return rs;
    }
    *out = c;
    return RT_OK;
}

rt_status rt_destroy(rt_ctx *c)
{
    if (!c) return RT_OK;
    (void)hipSetDevice(c->cfg.device);
    if (c->graph_exec) (void)hipGraphExecDestroy(c->graph_exec);
    if (c->capture_stream) (void)hipStreamDestroy(c->capture_stream);
    persistent_destroy(c->persist);
    decode_coop_destroy(c->dec);
    if (c->kv_chunk) (void)hipFree(c->kv_chunk);
    if (c->stack_slab) (void)hipFree(c->stack_slab);
    if (c->stack_dev) (void)hipFree(c->stack_dev);
    if (c->par_slab) (void)hipFree(c->par_slab);
    if (c->bw_slab) (void)hipFree(c->bw_slab);
    for (int g = 0; g < kMaxWaveStreams; ++g) {
        if (g > 0 && c->wave_streams.st[g]) (void)hipStreamDestroy(c->wave_streams.st[g]);
        if (c->wave_streams.ev[g]) (void)hipEventDestroy(c->wave_streams.ev[g]);
    }
    hipError_t e = hipFree(c->slab);
    delete c;
    return e == hipSuccess ? RT_OK : RT_ERR_HIP;
}

static const char *static_last_error();
const char *rt_last_error(const rt_ctx *c) { return c ? c->err.c_str() : static_last_error(); }
uint64_t rt_workspace_bytes(const rt_ctx *c)
{
    return c ? (uint64_t)c->slab_bytes + c->kv_chunk_bytes + persistent_bytes(c->persist) + decode_coop_bytes(c->dec) + c->stack_bytes +
                   c->par_bytes + c->bw_bytes
             : 0;
}
const char *rt_engine_name(const rt_ctx *c) { return c ? c->engine.c_str() : ""; }

int32_t rt_device_wait_expired(rt_ctx *c)
{
    if (!c) return 0;
    const int v = persistent_wait_expired(c->persist);
    if (v) {
        c->broken = true;
        c->err = "a bounded device-side wait expired in the persistent engine";
        return v;
    }
    const int w = decode_coop_wait_expired(c->dec);
    if (w) {
        c->broken = true;
        c->err = "a bounded device-side wait expired in the single-launch decoding step";
        return w;
    }
    if (c->bw_slab && c->bw_loop.available) {   // abort word of the backward pass's single-launch loop (word 8 of its exchange area)
        unsigned long long a = 0;
        if (hipMemcpy(&a, (char *)c->bw_slab + 64, sizeof(a), hipMemcpyDeviceToHost) != hipSuccess) return -1;
        if (a != 0) {
            c->broken = true;
            c->err = "a bounded device-side wait expired in the reverse loop of the backward pass";
            return 1;
        }
    }
    return 0;
}

int32_t rt_phase_trace(rt_ctx *c, uint64_t *out, int32_t rows)
{
    if (!c || !out || rows < 1) return 0;
    return persistent_read_trace(c->persist, (unsigned long long *)out, rows);
}

int32_t rt_decode_phase_trace(rt_ctx *c, uint64_t *out, int32_t workgroups)
{
    if (!c || !out || workgroups < 1) return 0;
    return decode_coop_read_trace(c->dec, (unsigned long long *)out, workgroups);
}

}  // extern "C"

static bool ranges_overlap(const void *a, size_t na, const void *b, size_t nb)
{
    const char *pa = (const char *)a, *pb = (const char *)b;
    return pa < pb + nb && pb < pa + na;
}

static rt_status check_weights(rt_ctx *c, const rt_layer_weights *w)
{
    if (!w || !w->Wq || !w->Wk || !w->Wv || !w->Wo || !w->W1 || !w->W2)
        return fail(c, RT_ERR_INVALID_ARG, "null weight pointer%s");
    return RT_OK;
}

static Weights to_weights(const rt_layer_weights *w)
{
    Weights W;
    W.Wq = w->Wq; W.Wk = w->Wk; W.Wv = w->Wv; W.Wo = w->Wo; W.W1 = w->W1; W.W2 = w->W2;
    W.g_attn = w->g_attn; W.g_mlp = w->g_mlp; W.g_kv = w->g_kv ? w->g_kv : w->g_attn; W.g_q = w->g_q; W.g_k = w->g_k;
    return W;
}

#define RT_TRY(expr, where)                                   \
    do {                                                      \
        hipError_t _e = (expr);                               \
        if (_e != hipSuccess) return fail_hip(c, _e, where);  \
    } while (0)

// One position of the sequential loop as separate launches (base case of Algorithm 1).
template <typename T>
static rt_status enqueue_position(rt_ctx *c, const LayerDims &D, const Weights &W, const void *x_t, size_t x_stride_b,
                                  void *y_t, size_t y_stride_b, void *K, void *V, int t, int q_row, int n_splits,
                                  bool write_vt)
{
    hipStream_t st = c->stream;
    RT_TRY(Launch<T>::merge(D, c->S, K, V, t, q_row, n_splits, st), "merge");
    RT_TRY(Launch<T>::gemv_wo(D, W, c->S, x_t, x_stride_b, st), "gemv_wo");
    RT_TRY(Launch<T>::gemv_w1(D, W, c->S, st), "gemv_w1");
    RT_TRY(Launch<T>::gemv_w2(D, W, c->S, y_t, y_stride_b, st), "gemv_w2");
    RT_TRY(Launch<T>::gemv_kv(D, W, c->S, st), "gemv_kv");
    RT_TRY(Launch<T>::finalize_kv(D, W, c->S, K, V, t, write_vt, st), "finalize_kv");
    return RT_OK;
}

template <typename T>
static rt_status enqueue_prefill_stepwise(rt_ctx *c, const LayerDims &D, const Weights &W, const void *x, void *y, void *K,
                                          void *V)
{
    hipStream_t st = c->stream;
    const size_t E = sizeof(T);
    RT_TRY(Launch<T>::prepass(D, W, c->S, x, D.B, D.N, c->use_mfma, st), "prepass");
    for (int t = 0; t < D.N; ++t) {
        rt_status s = enqueue_position<T>(c, D, W, (const char *)x + (size_t)t * D.d * E, (size_t)D.N * D.d,
                                          (char *)y + (size_t)t * D.d * E, (size_t)D.N * D.d, K, V, t, t, -1, c->use_mfma);
        if (s != RT_OK) return s;
        const int t1 = t + 1;
        const int P = t1 & -t1;
        if (P >= D.p_min && t1 < D.N) {
            const int nq = (P < D.N - t1) ? P : D.N - t1;
            RT_TRY(Launch<T>::cross(D, c->S, K, V, t1, P, nq, c->use_mfma, st), "cross");
        }
    }
    return RT_OK;
}

template <typename T>
static rt_status prefill_stepwise(rt_ctx *c, const LayerDims &D, const rt_layer_weights *w, const void *x, void *y, void *K,
                                  void *V)
{
    const Weights W = to_weights(w);
    if (!(c->cfg.flags & RT_FLAG_HIP_GRAPH)) {
        c->engine = "stepwise";
        return enqueue_prefill_stepwise<T>(c, D, W, x, y, K, V);
    }
    c->engine = "stepwise+graph";
    rt_ctx::GraphKey key;
    memset(&key, 0, sizeof(key));
    key.x = x; key.y = y; key.K = K; key.V = V; key.w = *w; key.B = D.B; key.N = D.N; key.kv_cap = D.kv_cap;
    if (!c->graph_exec || memcmp(&key, &c->graph_key, sizeof(key)) != 0) {
        if (c->graph_exec) { (void)hipGraphExecDestroy(c->graph_exec); c->graph_exec = nullptr; }
        // Record on a private stream (default priority), replay on the caller's stream.
        if (!c->capture_stream)
            RT_TRY(hipStreamCreateWithFlags(&c->capture_stream, hipStreamNonBlocking), "hipStreamCreateWithFlags");
        hipStream_t user = c->stream;
        c->stream = c->capture_stream;
        hipError_t e = hipStreamBeginCapture(c->capture_stream, hipStreamCaptureModeThreadLocal);
        if (e != hipSuccess) { c->stream = user; return fail_hip(c, e, "hipStreamBeginCapture"); }
        rt_status s = enqueue_prefill_stepwise<T>(c, D, W, x, y, K, V);
        c->stream = user;
        hipGraph_t g = nullptr;
        e = hipStreamEndCapture(c->capture_stream, &g);
        if (s != RT_OK) { if (g) (void)hipGraphDestroy(g); return s; }
        if (e != hipSuccess) return fail_hip(c, e, "hipStreamEndCapture");
        e = hipGraphInstantiate(&c->graph_exec, g, nullptr, nullptr, 0);
        (void)hipGraphDestroy(g);
        if (e != hipSuccess) { c->graph_exec = nullptr; return fail_hip(c, e, "hipGraphInstantiate"); }
        c->graph_key = key;
    }
    RT_TRY(hipGraphLaunch(c->graph_exec, c->stream), "hipGraphLaunch");
    return RT_OK;
}

extern "C" rt_status rt_layer_prefill(rt_ctx *c, const rt_layer_weights *w, const void *x, int32_t B, int32_t N, void *y,
                                      void *K, void *V, int32_t kv_cap)
{
    if (!c) return RT_ERR_INVALID_ARG;
    if (c->broken) return fail(c, RT_ERR_STATE, "context is unusable after an earlier failure%s");
    rt_status s = check_weights(c, w);
    if (s != RT_OK) return s;
    if (!x || !y || !K || !V) return fail(c, RT_ERR_INVALID_ARG, "null tensor pointer%s");
    if (B < 1 || B > c->cfg.max_batch) return fail(c, RT_ERR_INVALID_ARG, "B out of range [1, max_batch]%s");
    if (N < 1 || N > c->cfg.max_seq) return fail(c, RT_ERR_INVALID_ARG, "N out of range [1, max_seq]%s");
    if (kv_cap < N) return fail(c, RT_ERR_INVALID_ARG, "kv_cap < N%s");
    const size_t E = c->cfg.dtype == RT_BF16 ? 2 : 4;
    const size_t xb = (size_t)B * N * c->cfg.d_model * E, kvb = (size_t)kv_cap * B * c->cfg.d_model * E;
    if (ranges_overlap(x, xb, y, xb)) return fail(c, RT_ERR_INVALID_ARG, "x and y overlap%s");
    if (ranges_overlap(K, kvb, V, kvb) || ranges_overlap(K, kvb, y, xb) || ranges_overlap(V, kvb, y, xb) ||
        ranges_overlap(K, kvb, x, xb) || ranges_overlap(V, kvb, x, xb))
        return fail(c, RT_ERR_INVALID_ARG, "K, V, x, y must not overlap%s");
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, RT_ERR_HIP, "hipSetDevice failed%s");

    LayerDims D = c->base;
    D.B = B; D.N = N; D.kv_cap = kv_cap;
    c->last_B = B; c->last_N = N;
    c->last_hp = false;
    poison_partials(c, c->S);
    const bool want_stepwise = (c->cfg.flags & RT_FLAG_ENGINE_STEPWISE) != 0;
    if (!want_stepwise && persistent_supported(c->persist, D)) {
        c->engine = "persistent";
        c->last_hp = true;
        const Weights W = to_weights(w);
        hipError_t e;
        if (c->cfg.dtype == RT_BF16) e = Launch<bf16_t>::prepass(D, W, c->S, x, B, N, c->use_mfma, c->stream);
        else e = Launch<float>::prepass(D, W, c->S, x, B, N, false, c->stream);
        if (e != hipSuccess) return fail_hip(c, e, "prepass");
        std::string perr;
        s = persistent_prefill(c->persist, D, W, c->S, x, y, K, V, c->stream, perr);
        if (s != RT_OK) { c->err = perr; if (s == RT_ERR_HIP) c->broken = true; }
        return s;
    }
    if (!want_stepwise && !(c->cfg.flags & RT_FLAG_ENGINE_PERSISTENT) && B >= kWaveFrom && B <= kWaveTo && c->cfg.dtype == RT_BF16 &&
        c->stack_slab && c->stack_chunk == 64 && c->base.p_min <= 64 &&
        wavefront_uses_matrix_cores(c->cfg.d_model, c->cfg.d_hidden, c->use_mfma)) {
        // a stack of one layer on the layer-wavefront engine (workspace reserved at rt_create for such contexts)
        void *y1 = y, *K1 = K, *V1 = V;
        c->last_B = 0;   // the engine keeps its state in the stack workspace: no stand-alone tile on the context's scratch
        return rt_stack_prefill(c, w, 1, x, B, N, &y1, &K1, &V1, kv_cap, 64);
    }
    if (!want_stepwise && !(c->cfg.flags & RT_FLAG_ENGINE_PERSISTENT) && B >= kBatchedFrom && c->cfg.dtype == RT_BF16 &&
        parallel_supported(D, c->use_mfma) && c->par_slab) {
        // many sequences: one position of all of them per step, the base-case products as batched matrix products over the
        // B rows (the blocked recurrence with blocks of one position, which is this layer); its scratch was reserved at rt_create
        c->engine = "position-batched";
        c->last_hp = true;
        hipError_t e = blocked_layer(D, to_weights(w), c->S, x, 1, y, K, V, c->par_slab, c->stream);
        if (e != hipSuccess) return fail_hip(c, e, "blocked_layer");
        return RT_OK;
    }
    LayerDims Dc = D;
    Dc.B = c->persist.max_batch;
    if (!want_stepwise && c->kv_chunk && B > c->persist.max_batch && persistent_supported(c->persist, Dc)) {
        // batch rows are independent: chunks of the engine's rows, one after the other on the stream; x and y of a chunk are
        // contiguous slices, its pairs go through the chunk buffers (the cache is position-major over the whole batch)
        c->engine = "persistent";
        c->last_hp = true;
        c->last_B = 0;   // the scratch holds the last chunk only: no stand-alone tile on it
        const Weights W = to_weights(w);
        const size_t d = (size_t)c->cfg.d_model, row = d * E;
        char *Kc = (char *)c->kv_chunk, *Vc = Kc + c->kv_chunk_bytes / 2;
        for (int b0 = 0; b0 < B; b0 += c->persist.max_batch) {
            const int nb = B - b0 < c->persist.max_batch ? B - b0 : c->persist.max_batch;
            Dc.B = nb; Dc.kv_cap = N;
            const char *xc = (const char *)x + (size_t)b0 * N * row;
            char *yc = (char *)y + (size_t)b0 * N * row;
            if (b0 > 0) poison_partials(c, c->S);
            hipError_t e = Launch<bf16_t>::prepass(Dc, W, c->S, xc, nb, N, c->use_mfma, c->stream);
            if (e != hipSuccess) return fail_hip(c, e, "prepass");
            std::string perr;
            s = persistent_prefill(c->persist, Dc, W, c->S, xc, yc, Kc, Vc, c->stream, perr);
            if (s != RT_OK) { c->err = perr; if (s == RT_ERR_HIP) c->broken = true; return s; }
            RT_TRY(hipMemcpy2DAsync((char *)K + (size_t)b0 * row, (size_t)B * row, Kc, (size_t)nb * row, (size_t)nb * row, (size_t)N,
                                    hipMemcpyDeviceToDevice, c->stream), "hipMemcpy2DAsync");
            RT_TRY(hipMemcpy2DAsync((char *)V + (size_t)b0 * row, (size_t)B * row, Vc, (size_t)nb * row, (size_t)nb * row, (size_t)N,
                                    hipMemcpyDeviceToDevice, c->stream), "hipMemcpy2DAsync");
        }
        return RT_OK;
    }
    if (c->cfg.flags & RT_FLAG_ENGINE_PERSISTENT)
        return fail(c, RT_ERR_UNSUPPORTED, "the persistent engine does not cover this shape%s");
    if (c->cfg.dtype == RT_BF16) return prefill_stepwise<bf16_t>(c, D, w, x, y, K, V);
    return prefill_stepwise<float>(c, D, w, x, y, K, V);
}

template <typename T>
static rt_status decode_impl(rt_ctx *c, const LayerDims &D, const rt_layer_weights *w, const void *x_t, int t, void *y_t,
                             void *K, void *V)
{
    const Weights W = to_weights(w);
    hipStream_t st = c->stream;
    // up to three times the rows the single launch takes: one launch per chunk of those rows (batch rows are independent;
    // MI355X, d = 1024, t = 511: B = 32 takes 63 us in two chunks against 85 us as eight launches, B = 64 126 against 121)
    if (sizeof(T) == 2 && c->dec.available && D.B > c->dec.max_batch && D.B <= 3 * c->dec.max_batch) {
        c->engine = "decode-single-launch";
        const size_t row = (size_t)D.d * sizeof(T);
        for (int b0 = 0; b0 < D.B; b0 += c->dec.max_batch) {
            LayerDims Dc = D;
            Dc.B = D.B - b0 < c->dec.max_batch ? D.B - b0 : c->dec.max_batch;
            std::string derr;
            const rt_status ds = decode_coop_step(c->dec, Dc, W, (const char *)x_t + b0 * row, t, (char *)y_t + b0 * row,
                                                  (char *)K + b0 * row, (char *)V + b0 * row, st, derr, (size_t)D.B * D.d);
            if (ds != RT_OK) { c->err = derr; if (ds == RT_ERR_HIP) c->broken = true; return ds; }
        }
        return RT_OK;
    }
    if (sizeof(T) == 2 && decode_coop_supported(c->dec, D)) {   // the whole step as one cooperative launch
        c->engine = "decode-single-launch";
        std::string derr;
        const rt_status ds = decode_coop_step(c->dec, D, W, x_t, t, y_t, K, V, st, derr);
        if (ds != RT_OK) { c->err = derr; if (ds == RT_ERR_HIP) c->broken = true; }
        return ds;
    }
    // bf16 with d and F multiples of 256: the products run on the matrix cores
    const bool mm = sizeof(T) == 2 && step_mm_supported(D, c->use_mfma);
    RT_TRY(Launch<T>::prepass_one(D, W, c->S, x_t, (size_t)D.d, st, mm), "prepass_one");
    const int chunk = 64;   // keys per wavefront: t / 64 wavefronts per (b, h) keep the whole chip reading the cache
    const int nsplit = (t + chunk - 1) / chunk;
    if (nsplit > 0) RT_TRY(Launch<T>::decode_split(D, c->S, K, V, t, chunk, nsplit, st), "decode_split");
    if (!mm) return enqueue_position<T>(c, D, W, x_t, (size_t)D.d, y_t, (size_t)D.d, K, V, t, 0, nsplit, false);
    RT_TRY(Launch<T>::merge(D, c->S, K, V, t, 0, nsplit, st, true), "merge");
    const size_t row = (size_t)t * D.B * D.d * sizeof(T);
    RT_TRY(step_base_case_mm(D, W, c->S, x_t, y_t, (char *)K + row, (char *)V + row, st), "step_base_case_mm");
    return RT_OK;
}

// Host-side argument checks of a decoding step (both entry points); msg receives the reason.
static rt_status check_decode_args(const rt_config &cfg, const rt_layer_weights *w, const void *x_t, int32_t B, int32_t t,
                                   const void *y_t, const void *K, const void *V, int32_t kv_cap, const char **msg)
{
    *msg = "";
    if (!w || !w->Wq || !w->Wk || !w->Wv || !w->Wo || !w->W1 || !w->W2) { *msg = "null weight pointer"; return RT_ERR_INVALID_ARG; }
    if (!x_t || !y_t || !K || !V) { *msg = "null tensor pointer"; return RT_ERR_INVALID_ARG; }
    if (B < 1 || B > cfg.max_batch) { *msg = "B out of range [1, max_batch]"; return RT_ERR_INVALID_ARG; }
    if (t < 0 || t >= kv_cap) { *msg = "t out of range [0, kv_cap)"; return RT_ERR_INVALID_ARG; }
    if (t >= cfg.max_seq) { *msg = "t out of range [0, max_seq)"; return RT_ERR_INVALID_ARG; }
    const size_t E = cfg.dtype == RT_BF16 ? 2 : 4;
    const size_t xb = (size_t)B * cfg.d_model * E, kvb = (size_t)kv_cap * B * cfg.d_model * E;
    if (ranges_overlap(x_t, xb, y_t, xb)) { *msg = "x_t and y_t overlap"; return RT_ERR_INVALID_ARG; }
    if (ranges_overlap(K, kvb, V, kvb) || ranges_overlap(K, kvb, y_t, xb) || ranges_overlap(V, kvb, y_t, xb) ||
        ranges_overlap(K, kvb, x_t, xb) || ranges_overlap(V, kvb, x_t, xb)) {
        *msg = "K, V, x_t, y_t must not overlap";
        return RT_ERR_INVALID_ARG;
    }
    return RT_OK;
}

extern "C" rt_status rt_decode_step(rt_ctx *c, const rt_layer_weights *w, const void *x_t, int32_t B, int32_t t, void *y_t,
                                    void *K, void *V, int32_t kv_cap)
{
    if (!c) return RT_ERR_INVALID_ARG;
    if (c->broken) return fail(c, RT_ERR_STATE, "context is unusable after an earlier failure%s");
    const char *msg;
    rt_status s = check_decode_args(c->cfg, w, x_t, B, t, y_t, K, V, kv_cap, &msg);
    if (s != RT_OK) return fail(c, s, "%s", msg);
    if ((t + 63) / 64 > c->S.slots) return fail(c, RT_ERR_INVALID_ARG, "t too large for this context's max_seq%s");
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, RT_ERR_HIP, "hipSetDevice failed%s");
    LayerDims D = c->base;
    D.B = B; D.N = 1; D.kv_cap = kv_cap;
    c->engine = "stepwise";
    if (c->cfg.dtype == RT_BF16) return decode_impl<bf16_t>(c, D, w, x_t, t, y_t, K, V);
    return decode_impl<float>(c, D, w, x_t, t, y_t, K, V);
}

// ------------------------------------------------------------------------------------------------------------
// The decoding step for callers that cannot allocate (rt_decode_step_static): no context, no hipMalloc.  Its
// scratch - the position's q and temporary pair, the split-attention partial states, the vectors between the base
// case's products - lives in this file-scope device array; each device holds its own copy at its own address,
// looked up once per device and kept.  The array's name is only a host-side handle: host code passes the looked-up
// address, never the name.
// ------------------------------------------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes = RT_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kStaticMaxDevices = 64;
static std::mutex g_static_mu;
static void *g_static_ptr[kStaticMaxDevices];   // device address of `scratch` on device i, or null before its first use
static thread_local char g_static_err[256];      // reason of the last failed context-free call on this thread

// Device address of the static scratch on `device` (made current by the caller).
static rt_status static_scratch_address(int device, void **out)
{
    if (device < 0 || device >= kStaticMaxDevices) return RT_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[device]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            snprintf(g_static_err, sizeof(g_static_err), "hipGetSymbolAddress: %s", hipGetErrorString(e));
            return RT_ERR_HIP;
        }
        g_static_ptr[device] = p;
    }
    *out = g_static_ptr[device];
    return RT_OK;
}

static const char *static_last_error() { return g_static_err[0] ? g_static_err : kNoCtx; }

static rt_status static_fail(rt_status s, const char *msg)
{
    snprintf(g_static_err, sizeof(g_static_err), "%s", msg);
    return s;
}

extern "C" rt_status rt_decode_step_static(const rt_config *cfg, const rt_layer_weights *w, const void *x_t, int32_t B,
                                           int32_t t, void *y_t, void *K, void *V, int32_t kv_cap)
{
    g_static_err[0] = 0;
    if (!cfg) return static_fail(RT_ERR_INVALID_ARG, "null configuration");
    int p_min = 0;
    bool mfma = false;
    rt_status s = validate_config(cfg, &p_min, &mfma);
    if (s != RT_OK) return static_fail(s, "invalid or unsupported configuration");
    const char *msg;
    s = check_decode_args(*cfg, w, x_t, B, t, y_t, K, V, kv_cap, &msg);
    if (s != RT_OK) return static_fail(s, msg);
    // the scratch of this call: one position's rows for B sequences and one partial state per split of 64 keys
    const size_t E = cfg->dtype == RT_BF16 ? 2 : 4;
    const int nsplit = (t + 63) / 64;
    Scratch S;
    const size_t need = layout_scratch(S, nullptr, (size_t)B, 1, (size_t)cfg->d_model, (size_t)cfg->d_hidden, (size_t)cfg->n_heads, E,
                                       false, 1, nsplit > 0 ? nsplit : 1);
    if (need > kStaticScratchBytes) {
        snprintf(g_static_err, sizeof(g_static_err),
                 "B, t, d_model, d_hidden need %zu bytes of scratch, the static scratch holds %zu", need, kStaticScratchBytes);
        return RT_ERR_INVALID_ARG;
    }
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || cfg->device < 0 || cfg->device >= ndev)
        return static_fail(RT_ERR_HIP, "no such device");
    if (hipSetDevice(cfg->device) != hipSuccess) return static_fail(RT_ERR_HIP, "hipSetDevice failed");
    void *base = nullptr;
    s = static_scratch_address(cfg->device, &base);
    if (s != RT_OK) return s;
    rt_ctx tmp;   // a context on the stack: configuration, stream and the scratch pointers, nothing owned
    tmp.cfg = *cfg;
    tmp.cfg.p_min = p_min;
    tmp.stream = (hipStream_t)cfg->stream;
    tmp.use_mfma = mfma;
    fill_dims(tmp.base, tmp.cfg, p_min);
    layout_scratch(tmp.S, (char *)base, (size_t)B, 1, (size_t)cfg->d_model, (size_t)cfg->d_hidden, (size_t)cfg->n_heads, E, false, 1,
                   nsplit > 0 ? nsplit : 1);
    LayerDims D = tmp.base;
    D.B = B; D.N = 1; D.kv_cap = kv_cap;
    s = cfg->dtype == RT_BF16 ? decode_impl<bf16_t>(&tmp, D, w, x_t, t, y_t, K, V) : decode_impl<float>(&tmp, D, w, x_t, t, y_t, K, V);
    if (s != RT_OK) snprintf(g_static_err, sizeof(g_static_err), "%s", tmp.err.c_str());
    return s;
}

extern "C" rt_status rt_embed_rows(rt_ctx *c, const void *table, int32_t vocab, const int32_t *ids, int64_t ids_stride,
                                   int32_t first, int32_t B, int32_t N, void *x)
{
    if (!c) return RT_ERR_INVALID_ARG;
    if (c->broken) return fail(c, RT_ERR_STATE, "context is unusable after an earlier failure%s");
    if (!table || !ids || !x) return fail(c, RT_ERR_INVALID_ARG, "null pointer%s");
    if (vocab < 1 || B < 1 || N < 1 || first < 0 || ids_stride < (int64_t)first + N)
        return fail(c, RT_ERR_INVALID_ARG, "vocab, B, N >= 1 and first + N <= ids_stride are required%s");
    if ((int64_t)B * N > (int64_t)1 << 31) return fail(c, RT_ERR_INVALID_ARG, "B * N too large%s");
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, RT_ERR_HIP, "hipSetDevice failed%s");
    hipError_t e;
    if (c->cfg.dtype == RT_BF16)
        e = embed_rows_launch<bf16_t>(table, ids, x, B, N, c->cfg.d_model, vocab, ids_stride, first, c->stream);
    else
        e = embed_rows_launch<float>(table, ids, x, B, N, c->cfg.d_model, vocab, ids_stride, first, c->stream);
    if (e != hipSuccess) return fail_hip(c, e, "embed_rows");
    return RT_OK;
}

extern "C" rt_status rt_lm_head(rt_ctx *c, const void *W_lm, const void *g_final, int32_t vocab, const void *z,
                                int64_t z_stride, int32_t B, float *logits)
{
    if (!c) return RT_ERR_INVALID_ARG;
    if (c->broken) return fail(c, RT_ERR_STATE, "context is unusable after an earlier failure%s");
    if (!W_lm || !z || !logits) return fail(c, RT_ERR_INVALID_ARG, "null pointer%s");
    if (vocab < 1 || B < 1 || B > c->cfg.max_batch || z_stride < c->cfg.d_model)
        return fail(c, RT_ERR_INVALID_ARG, "vocab >= 1, 1 <= B <= max_batch and z_stride >= d_model are required%s");
    if (c->cfg.d_model > 12288) return fail(c, RT_ERR_UNSUPPORTED, "rt_lm_head covers d_model <= 12288%s");
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, RT_ERR_HIP, "hipSetDevice failed%s");
    const int nf = (c->cfg.flags & RT_FLAG_NORM_FREE) ? 1 : 0;
    hipError_t e;
    if (c->cfg.dtype == RT_BF16)
        e = lm_head_launch<bf16_t>(W_lm, g_final, z, z_stride, logits, B, c->cfg.d_model, vocab, c->cfg.rms_eps, nf, c->stream);
    else
        e = lm_head_launch<float>(W_lm, g_final, z, z_stride, logits, B, c->cfg.d_model, vocab, c->cfg.rms_eps, nf, c->stream);
    if (e != hipSuccess) return fail_hip(c, e, "lm_head");
    return RT_OK;
}

extern "C" rt_status rt_cross_block_event(rt_ctx *c, const void *K, const void *V, int32_t B, int32_t t1, int32_t P, int32_t nq)
{
    if (!c) return RT_ERR_INVALID_ARG;
    if (c->broken) return fail(c, RT_ERR_STATE, "context is unusable after an earlier failure%s");
    if (!K || !V) return fail(c, RT_ERR_INVALID_ARG, "null tensor pointer%s");
    if (c->last_N == 0 || B != c->last_B) return fail(c, RT_ERR_STATE, "no prefill of this batch size has run on this context%s");
    if (!is_pow2(P) || P < c->cfg.p_min || t1 < P || t1 % P != 0 || nq < 1 || nq > P || (int64_t)t1 + nq > c->last_N)
        return fail(c, RT_ERR_INVALID_ARG, "need P a power of two >= p_min, t1 a positive multiple of P, 1 <= nq <= P, t1 + nq <= N%s");
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, RT_ERR_HIP, "hipSetDevice failed%s");
    LayerDims D = c->base;
    D.B = B; D.N = c->last_N; D.kv_cap = c->last_N;
    hipError_t e;
    // the tile in the form the engine of that prefill uses: after the persistent engine with high-precision logits
    if (c->cfg.dtype == RT_BF16 && c->use_mfma && c->last_hp) e = cross_mfma_launch(D, c->S, K, t1, P, nq, true, c->stream);
    else if (c->cfg.dtype == RT_BF16) e = Launch<bf16_t>::cross(D, c->S, K, V, t1, P, nq, c->use_mfma, c->stream);
    else e = Launch<float>::cross(D, c->S, K, V, t1, P, nq, false, c->stream);
    if (e != hipSuccess) return fail_hip(c, e, "cross");
    return RT_OK;
}

// Scratch of the layer-wavefront engine: one set per layer, sized for max_batch x max_seq; kept until the
// context is destroyed and reused by later calls with the same chunk and at most as many layers.
static rt_status stack_workspace(rt_ctx *c, int L, int chunk)
{
    if (c->stack_slab && c->stack_L >= L && c->stack_chunk == chunk) return RT_OK;
    // a different shape: wait for whatever still uses the old sets before they go
    if (c->stack_slab || c->stack_dev) {
        if (hipStreamSynchronize(c->stream) != hipSuccess) return fail(c, RT_ERR_HIP, "hipStreamSynchronize failed%s");
        if (c->stack_slab) (void)hipFree(c->stack_slab);
        if (c->stack_dev) (void)hipFree(c->stack_dev);
        c->stack_slab = nullptr; c->stack_dev = nullptr; c->stack_bytes = 0; c->stack_L = 0;
    }
    const rt_config &cfg = c->cfg;
    const size_t E = cfg.dtype == RT_BF16 ? 2 : 4;
    // partial states: the levels inside a chunk, then one far state per query (slots 0..N-1 of the next level on)
    int slots = (cfg.max_seq + 1) / 2;
    if (slots < 64) slots = 64;
    const int levels = ilog2(chunk) - c->base.log2_pmin + (cfg.max_seq + slots - 1) / slots;
    Scratch tmp;
    const bool packed = wavefront_uses_matrix_cores(cfg.d_model, cfg.d_hidden, c->use_mfma);
    const size_t one = align_up(layout_scratch(tmp, nullptr, cfg.max_batch, cfg.max_seq, cfg.d_model, cfg.d_hidden, cfg.n_heads, E,
                                               c->use_mfma, levels, slots, packed), 256);
    hipError_t e = hipMalloc(&c->stack_slab, one * L);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        c->stack_slab = nullptr;
        return fail(c, e == hipErrorOutOfMemory ? RT_ERR_OOM : RT_ERR_HIP, "scratch of the layer stack: %s", hipGetErrorString(e));
    }
    // the engine reads whole 32-position groups of the transposed values and gives the positions not written yet the
    // weight 0: they must hold finite numbers
    e = hipMemsetAsync(c->stack_slab, 0, one * L, c->stream);
    if (e != hipSuccess) {
        (void)hipFree(c->stack_slab);
        c->stack_slab = nullptr;
        return fail(c, RT_ERR_HIP, "clearing the scratch of the layer stack: %s", hipGetErrorString(e));
    }
    e = hipMalloc((void **)&c->stack_dev, sizeof(WaveLayer) * L);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(c->stack_slab);
        c->stack_slab = nullptr; c->stack_dev = nullptr;
        return fail(c, RT_ERR_OOM, "layer descriptors: %s", hipGetErrorString(e));
    }
    c->stack_S.resize(L);
    for (int l = 0; l < L; ++l)
        layout_scratch(c->stack_S[l], (char *)c->stack_slab + one * l, cfg.max_batch, cfg.max_seq, cfg.d_model, cfg.d_hidden,
                       cfg.n_heads, E, c->use_mfma, levels, slots, packed);
    c->stack_bytes = one * L + sizeof(WaveLayer) * L;
    c->stack_L = L;
    c->stack_chunk = chunk;
    return RT_OK;
}

extern "C" rt_status rt_stack_prefill(rt_ctx *c, const rt_layer_weights *layers, int32_t L, const void *x, int32_t B, int32_t N,
                                      void *const *y, void *const *K, void *const *V, int32_t kv_cap, int32_t chunk)
{
    if (!c) return RT_ERR_INVALID_ARG;
    if (c->broken) return fail(c, RT_ERR_STATE, "context is unusable after an earlier failure%s");
    if (!layers || !x || !y || !K || !V) return fail(c, RT_ERR_INVALID_ARG, "null pointer%s");
    if (L < 1 || L > 4096) return fail(c, RT_ERR_INVALID_ARG, "L out of range [1, 4096]%s");
    if (B < 1 || B > c->cfg.max_batch) return fail(c, RT_ERR_INVALID_ARG, "B out of range [1, max_batch]%s");
    if (N < 1 || N > c->cfg.max_seq) return fail(c, RT_ERR_INVALID_ARG, "N out of range [1, max_seq]%s");
    if (kv_cap < N) return fail(c, RT_ERR_INVALID_ARG, "kv_cap < N%s");
    if (chunk == 0) chunk = 64;
    const int chunk_min = c->use_mfma ? 64 : c->cfg.p_min;
    if (!is_pow2(chunk) || chunk < chunk_min || chunk < c->cfg.p_min || chunk > (1 << 20))
        return fail(c, RT_ERR_INVALID_ARG, "chunk must be a power of two, at least p_min (and 64 with the MFMA kernels)%s");
    const size_t E = c->cfg.dtype == RT_BF16 ? 2 : 4;
    const size_t xb = (size_t)B * N * c->cfg.d_model * E, kvb = (size_t)kv_cap * B * c->cfg.d_model * E;
    for (int l = 0; l < L; ++l) {
        rt_status s = check_weights(c, &layers[l]);
        if (s != RT_OK) return s;
        if (!y[l] || !K[l] || !V[l]) return fail(c, RT_ERR_INVALID_ARG, "null tensor pointer%s");
        const void *in = l == 0 ? x : y[l - 1];
        if (ranges_overlap(in, xb, y[l], xb) || ranges_overlap(K[l], kvb, V[l], kvb) || ranges_overlap(K[l], kvb, y[l], xb) ||
            ranges_overlap(V[l], kvb, y[l], xb) || ranges_overlap(K[l], kvb, in, xb) || ranges_overlap(V[l], kvb, in, xb))
            return fail(c, RT_ERR_INVALID_ARG, "a layer's input, output, K and V must not overlap%s");
        for (int m = 0; m < l; ++m)
            if (ranges_overlap(y[m], xb, y[l], xb) || ranges_overlap(K[m], kvb, K[l], kvb) || ranges_overlap(V[m], kvb, V[l], kvb) ||
                ranges_overlap(K[m], kvb, V[l], kvb) || ranges_overlap(V[m], kvb, K[l], kvb))
                return fail(c, RT_ERR_INVALID_ARG, "tensors of different layers must not overlap%s");
    }
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, RT_ERR_HIP, "hipSetDevice failed%s");
    rt_status s = stack_workspace(c, L, chunk);
    if (s != RT_OK) return s;

    std::vector<WaveLayer> host(L);
    for (int l = 0; l < L; ++l) {
        host[l].W = to_weights(&layers[l]);
        host[l].S = c->stack_S[l];
        host[l].x = l == 0 ? x : y[l - 1];
        host[l].y = y[l]; host[l].K = K[l]; host[l].V = V[l];
        poison_partials(c, c->stack_S[l]);
    }
    // pageable source: the copy has been staged when the call returns, `host` may go out of scope
    RT_TRY(hipMemcpyAsync(c->stack_dev, host.data(), sizeof(WaveLayer) * L, hipMemcpyHostToDevice, c->stream), "descriptor copy");
    LayerDims D = c->base;
    D.B = B; D.N = N; D.kv_cap = kv_cap;
    c->engine = "wavefront";
    // groups of layers on streams of their own (RT_WAVE_STREAMS = 1..4 overrides the default of 3: cfg5, 12 layers, takes 302 ms
    // with two groups, 294-295 ms with three, twice as long with four - the process has four hardware queues)
    WaveStreams &WS = c->wave_streams;
    int want = 3;
    if (const char *ev = getenv("RT_WAVE_STREAMS")) want = atoi(ev);
    if (want < 1) want = 1;
    if (want > kMaxWaveStreams) want = kMaxWaveStreams;
    WS.st[0] = c->stream;
    for (int g = 0; g < want; ++g) {
        if (g > 0 && !WS.st[g]) RT_TRY(hipStreamCreateWithFlags(&WS.st[g], hipStreamNonBlocking), "hipStreamCreateWithFlags");
        if (!WS.ev[g]) RT_TRY(hipEventCreateWithFlags(&WS.ev[g], hipEventDisableTiming), "hipEventCreateWithFlags");
    }
    WS.n = want;
    hipError_t e;
    if (c->cfg.dtype == RT_BF16) e = wavefront_prefill<bf16_t>(D, c->stack_dev, host.data(), L, chunk, c->use_mfma, WS);
    else e = wavefront_prefill<float>(D, c->stack_dev, host.data(), L, chunk, false, WS);
    if (e != hipSuccess) return fail_hip(c, e, "wavefront_prefill");
    return RT_OK;
}

// Loop-free evaluation of a whole sequence (rt_parallel.hip); pairs_src = z (recompute) or x (Transformer layer).
// block > 0: blocked recurrence over blocks of that many positions instead (pairs_src = x).
static rt_status parallel_entry(rt_ctx *c, const rt_layer_weights *w, const void *x, const void *pairs_src, bool transformer,
                                int32_t B, int32_t N, void *y, void *K, void *V, int32_t kv_cap, int32_t block = 0)
{
    if (!c) return RT_ERR_INVALID_ARG;
    if (c->broken) return fail(c, RT_ERR_STATE, "context is unusable after an earlier failure%s");
    rt_status s = check_weights(c, w);
    if (s != RT_OK) return s;
    if (!x || !pairs_src || !y || !K || !V) return fail(c, RT_ERR_INVALID_ARG, "null tensor pointer%s");
    if (B < 1 || B > c->cfg.max_batch) return fail(c, RT_ERR_INVALID_ARG, "B out of range [1, max_batch]%s");
    if (N < 1 || N > c->cfg.max_seq) return fail(c, RT_ERR_INVALID_ARG, "N out of range [1, max_seq]%s");
    if (kv_cap < N) return fail(c, RT_ERR_INVALID_ARG, "kv_cap < N%s");
    if (block != 0 && (!is_pow2(block) || block > c->cfg.p_min))
        return fail(c, RT_ERR_INVALID_ARG, "block must be a power of two, at most p_min%s");
    const size_t E = c->cfg.dtype == RT_BF16 ? 2 : 4;
    const size_t xb = (size_t)B * N * c->cfg.d_model * E, kvb = (size_t)kv_cap * B * c->cfg.d_model * E;
    if (ranges_overlap(x, xb, y, xb) || (pairs_src != x && ranges_overlap(pairs_src, xb, y, xb)))
        return fail(c, RT_ERR_INVALID_ARG, "the output must not overlap an input%s");
    if (ranges_overlap(K, kvb, V, kvb) || ranges_overlap(K, kvb, y, xb) || ranges_overlap(V, kvb, y, xb) ||
        ranges_overlap(K, kvb, x, xb) || ranges_overlap(V, kvb, x, xb) || ranges_overlap(K, kvb, pairs_src, xb) ||
        ranges_overlap(V, kvb, pairs_src, xb))
        return fail(c, RT_ERR_INVALID_ARG, "K, V and the other tensors must not overlap%s");
    LayerDims D = c->base;
    D.B = B; D.N = N; D.kv_cap = kv_cap;
    // bf16 with the matrix-core kernels: GEMMs and one masked attention pass; anything else (fp32 storage, no MFMA, odd
    // hidden width): the plain-ALU kernels
    const bool fast = c->cfg.dtype == RT_BF16 && parallel_supported(D, c->use_mfma);
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, RT_ERR_HIP, "hipSetDevice failed%s");
    poison_partials(c, c->S);
    s = ensure_loop_free_scratch(c);
    if (s != RT_OK) return s;
    if (!fast) {
        c->last_B = B; c->last_N = N;
        c->last_hp = false;
        c->engine = block ? "blocked" : (transformer ? "transformer" : "recompute");
        const Weights Wg = to_weights(w);
        hipError_t e;
        if (block)
            e = c->cfg.dtype == RT_BF16 ? Launch<bf16_t>::blocked_generic(D, Wg, c->S, x, block, y, K, V, c->par_slab, c->stream)
                                        : Launch<float>::blocked_generic(D, Wg, c->S, x, block, y, K, V, c->par_slab, c->stream);
        else
            e = c->cfg.dtype == RT_BF16
                    ? Launch<bf16_t>::loop_free(D, Wg, c->S, x, pairs_src, transformer, y, K, V, c->par_slab, c->stream)
                    : Launch<float>::loop_free(D, Wg, c->S, x, pairs_src, transformer, y, K, V, c->par_slab, c->stream);
        if (e != hipSuccess) return fail_hip(c, e, "loop_free");
        return RT_OK;
    }
    c->last_B = B; c->last_N = N;
    c->last_hp = true;
    c->engine = block ? "blocked" : (transformer ? "transformer" : "recompute");
    const Weights W = to_weights(w);
    hipError_t e = block ? blocked_layer(D, W, c->S, x, block, y, K, V, c->par_slab, c->stream)
                         : parallel_layer(D, W, c->S, x, pairs_src, transformer, y, K, V, c->par_slab, c->stream);
    if (e != hipSuccess) return fail_hip(c, e, "parallel_layer");
    return RT_OK;
}

extern "C" rt_status rt_layer_prefill_blocked(rt_ctx *c, const rt_layer_weights *w, const void *x, int32_t B, int32_t N,
                                              int32_t block, void *y, void *K, void *V, int32_t kv_cap)
{
    if (block < 1) return c ? fail(c, RT_ERR_INVALID_ARG, "block must be a power of two, at most p_min%s") : RT_ERR_INVALID_ARG;
    return parallel_entry(c, w, x, x, true, B, N, y, K, V, kv_cap, block);
}

extern "C" rt_status rt_layer_recompute(rt_ctx *c, const rt_layer_weights *w, const void *x, const void *z, int32_t B, int32_t N,
                                        void *y, void *K, void *V, int32_t kv_cap)
{
    return parallel_entry(c, w, x, z, false, B, N, y, K, V, kv_cap);
}

extern "C" rt_status rt_transformer_layer(rt_ctx *c, const rt_layer_weights *w, const void *x, int32_t B, int32_t N, void *y,
                                          void *K, void *V, int32_t kv_cap)
{
    return parallel_entry(c, w, x, x, true, B, N, y, K, V, kv_cap);
}

// Backward pass of one layer (rt_backward.hip).
extern "C" rt_status rt_layer_backward(rt_ctx *c, const rt_layer_weights *w, const void *x, const void *z, const void *gy,
                                       const void *gK, const void *gV, int32_t B, int32_t N, float *dx, const rt_layer_grads *grads)
{
    if (!c) return RT_ERR_INVALID_ARG;
    if (c->broken) return fail(c, RT_ERR_STATE, "context is unusable after an earlier failure%s");
    rt_status s = check_weights(c, w);
    if (s != RT_OK) return s;
    if (!x || !z || !gy || !dx || !grads) return fail(c, RT_ERR_INVALID_ARG, "null tensor pointer%s");
    if (B < 1 || B > c->cfg.max_batch) return fail(c, RT_ERR_INVALID_ARG, "B out of range [1, max_batch]%s");
    if (N < 1 || N > c->cfg.max_seq) return fail(c, RT_ERR_INVALID_ARG, "N out of range [1, max_seq]%s");
    if (N > 65535) return fail(c, RT_ERR_UNSUPPORTED, "rt_layer_backward covers sequences of at most 65535 positions%s");
    const size_t E = c->cfg.dtype == RT_BF16 ? 2 : 4;
    const size_t d = (size_t)c->cfg.d_model, F = (size_t)c->cfg.d_hidden;
    const size_t xb = (size_t)B * N * d * E, dxb = (size_t)B * N * d * 4;
    if (ranges_overlap(dx, dxb, x, xb) || ranges_overlap(dx, dxb, z, xb) || ranges_overlap(dx, dxb, gy, xb) ||
        (gK && ranges_overlap(dx, dxb, gK, xb)) || (gV && ranges_overlap(dx, dxb, gV, xb)))
        return fail(c, RT_ERR_INVALID_ARG, "dx must not overlap an input%s");
    {   // no gradient tensor may overlap dx or another gradient tensor
        const float *gp[11] = {grads->Wq, grads->Wk, grads->Wv, grads->Wo, grads->W1, grads->W2,
                               grads->g_attn, grads->g_mlp, grads->g_kv, grads->g_q, grads->g_k};
        const size_t gb[11] = {d * d * 4, d * d * 4, d * d * 4, d * d * 4, F * d * 4, F * d * 4, d * 4, d * 4, d * 4, d * 4, d * 4};
        for (int i = 0; i < 11; ++i) {
            if (!gp[i]) continue;
            if (ranges_overlap(gp[i], gb[i], dx, dxb)) return fail(c, RT_ERR_INVALID_ARG, "a gradient tensor overlaps dx%s");
            for (int j = i + 1; j < 11; ++j)
                if (gp[j] && ranges_overlap(gp[i], gb[i], gp[j], gb[j]))
                    return fail(c, RT_ERR_INVALID_ARG, "two gradient tensors overlap%s");
        }
    }
    if (hipSetDevice(c->cfg.device) != hipSuccess) return fail(c, RT_ERR_HIP, "hipSetDevice failed%s");
    s = ensure_backward_scratch(c);
    if (s != RT_OK) return s;
    LayerDims D = c->base;
    D.B = B; D.N = N; D.kv_cap = N;
    Weights W = to_weights(w);
    W.g_kv = w->g_kv;   // null = RMS(z) shares g_attn: that share of the gradient goes into grads->g_attn
    BwGrads G = {grads->Wq, grads->Wk, grads->Wv, grads->Wo, grads->W1, grads->W2,
                 grads->g_attn, grads->g_mlp, grads->g_kv, grads->g_q, grads->g_k};
    c->engine = "backward";
    hipError_t e = c->cfg.dtype == RT_BF16 ? backward_layer<bf16_t>(D, W, x, z, gy, gK, gV, dx, G, c->bw_slab, c->use_mfma, c->stream, &c->bw_loop)
                                           : backward_layer<float>(D, W, x, z, gy, gK, gV, dx, G, c->bw_slab, false, c->stream);
    if (e != hipSuccess) return fail_hip(c, e, "backward_layer");
    return RT_OK;
}
