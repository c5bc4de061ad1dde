/*
 * CPU oracle for the Recurrent Transformer (RT) layer -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain fp64, token by token, no tiling and no online softmax in the main entry
 * points: each function is the paper's definition written out.  Nothing here is
 * shared with the HIP library; only tests, the smoke check and the benchmark's
 * CPU-baseline leg may link or call this file.
 *
 *   rto_layer_prefill      Sec. 2.2 "The Recurrent Transformer layer": temporary pair from x_i,
 *                          a_i over persistent pairs j < i plus the temporary pair, z_i, and
 *                          the persistent pair from z_i (eqs. persistentK / persistentV);
 *                          multi-head + output projection per the Notation paragraph of Sec. 2.
 *   rto_decode_step        one iteration of the same recurrence over a caller-held KV cache (Sec. 7.3).
 *   rto_transformer_layer  Sec. 2.1 "The Transformer layer" (used only to check the emulation theorem).
 *   rto_layer_prefill_tiled  Appendix C, Algorithms 1 and 2 taken literally (running (m, l, o) per
 *                          query, read-modify-write); exists to check the exactness claim.
 *   rto_update_tile        Appendix C, Algorithm 2 on one (query tile, KV tile).
 *   rto_schedule           the (t, P, u, v, s, e) events of Algorithm 1.
 *   rto_layer_prefill_blocked  the blocked-recurrence extension of Sec. 8 (reading stated at the function).
 *
 * Readings taken where the paper is silent (all configurable, see rto_params):
 *   RMS(x) = g * x / sqrt(mean(x^2) + eps)   (paper: sqrt(D) x / |x|, i.e. eps = 0, g = 1)
 *   qkRMS  = the same normalisation applied to each head's slice of width dh
 *   MLP(u) = W2 * gelu(W1 * u), exact (erf) GELU, no biases, unless a callback is given
 *   logits = attn_scale * <k, q>   (paper: attn_scale = 1)
 *   residual scale alpha = 1/sqrt(L):  h = x + alpha a,  z = h + alpha MLP(RMS(h))
 *   norm_free != 0 turns every RMS and qkRMS into the identity (Appendix A).
 *   alibi_max_bias = beta > 0 adds the linear positional bias the paper's trained models use (Appendix D,
 *   experimental details: ALiBi with maximum bias 8.0): logit(i, j) -= m_h (i - j) for a persistent key of position
 *   j < i, with head slopes m_h = 2^(-beta (h + 1) / H), h = 0..H-1; the temporary pair sits at distance 0.
 *
 * Layouts: x, y [B][N][d];  K, V [kv_cap][B][H][dh] (position first);  weights row-major [out][in].
 * Pinned by tests/test_oracle_pins.py (closed forms, invariants, Appendix A construction,
 * Theorem 4.1, brute-force prefix re-evaluation, fixed-point recompute).
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef void (*rto_mlp_fn)(const double *in, double *out, int d, void *user);

typedef struct {
    int32_t d, H, dh, F;
    double alpha, attn_scale, eps;
    int32_t norm_free;
    int32_t threads;              /* <=0: all available */
    const double *Wq, *Wk, *Wv;   /* [d][d] */
    const double *Wo;             /* [d][d] or NULL = identity */
    const double *W1;             /* [F][d] (ignored when mlp != NULL) */
    const double *W2;             /* [d][F] */
    const double *g_attn, *g_mlp, *g_kv, *g_q, *g_k; /* [d] or NULL = ones */
    rto_mlp_fn mlp;               /* optional replacement for the whole MLP block */
    void *mlp_user;
    double alibi_max_bias;        /* 0 = no positional bias */
} rto_params;

static double alibi_slope(const rto_params *p, int h)
{
    return p->alibi_max_bias > 0.0 ? pow(2.0, -p->alibi_max_bias * (double)(h + 1) / (double)p->H) : 0.0;
}

#if defined(__x86_64__) && defined(__GNUC__) && !defined(__clang__)
#define RTO_CLONES __attribute__((target_clones("avx2", "default")))
#else
#define RTO_CLONES
#endif

/* out[o] = sum_i W[o][i] x[i] for o in [lo, hi), summed in increasing i for every o.
 * Wt is the transposed copy [n_in][n_out] so that the inner loop runs over o. */
RTO_CLONES static void matvec_range(const double *Wt, int n_in, int n_out, const double *x,
                                    double *out, int lo, int hi)
{
    for (int o = lo; o < hi; ++o) out[o] = 0.0;
    for (int i = 0; i < n_in; ++i) {
        const double xi = x[i];
        const double *w = Wt + (size_t)i * n_out;
        for (int o = lo; o < hi; ++o) out[o] += w[o] * xi;
    }
}

static void matvec(const double *Wt, int n_in, int n_out, const double *x, double *out, int par)
{
    if (!par) { matvec_range(Wt, n_in, n_out, x, out, 0, n_out); return; }
#pragma omp parallel
    {
#ifdef _OPENMP
        int nt = omp_get_num_threads(), id = omp_get_thread_num();
#else
        int nt = 1, id = 0;
#endif
        int chunk = (n_out + nt - 1) / nt;
        int lo = id * chunk, hi = lo + chunk;
        if (hi > n_out) hi = n_out;
        if (lo < hi) matvec_range(Wt, n_in, n_out, x, out, lo, hi);
    }
}

static double *transpose_copy(const double *W, int n_out, int n_in)
{
    double *t = (double *)malloc(sizeof(double) * (size_t)n_out * n_in);
    if (!t) return NULL;
    for (int o = 0; o < n_out; ++o)
        for (int i = 0; i < n_in; ++i) t[(size_t)i * n_out + o] = W[(size_t)o * n_in + i];
    return t;
}

/* RMS normalisation of a length-n vector with gain g (NULL = ones). */
static void rms_norm(const double *x, const double *g, int n, double eps, int norm_free, double *out)
{
    if (norm_free) { for (int i = 0; i < n; ++i) out[i] = x[i]; return; }
    double ss = 0.0;
    for (int i = 0; i < n; ++i) ss += x[i] * x[i];
    const double r = 1.0 / sqrt(ss / (double)n + eps);
    for (int i = 0; i < n; ++i) out[i] = x[i] * r * (g ? g[i] : 1.0);
}

static double gelu_erf(double u) { return 0.5 * u * (1.0 + erf(u * 0.70710678118654752440)); }

RTO_CLONES static double dot(const double *a, const double *b, int n)
{
    double s = 0.0;
    for (int i = 0; i < n; ++i) s += a[i] * b[i];
    return s;
}

typedef struct {
    double *Wq_t, *Wk_t, *Wv_t, *Wo_t, *W1_t, *W2_t; /* transposed copies */
} rto_tw;

static void free_tw(rto_tw *w)
{
    free(w->Wq_t); free(w->Wk_t); free(w->Wv_t); free(w->Wo_t); free(w->W1_t); free(w->W2_t);
}

static int make_tw(const rto_params *p, rto_tw *w)
{
    memset(w, 0, sizeof(*w));
    const int d = p->d, F = p->F;
    w->Wq_t = transpose_copy(p->Wq, d, d);
    w->Wk_t = transpose_copy(p->Wk, d, d);
    w->Wv_t = transpose_copy(p->Wv, d, d);
    if (p->Wo) w->Wo_t = transpose_copy(p->Wo, d, d);
    if (!p->mlp) {
        w->W1_t = transpose_copy(p->W1, F, d);
        w->W2_t = transpose_copy(p->W2, d, F);
    }
    if (!w->Wq_t || !w->Wk_t || !w->Wv_t || (p->Wo && !w->Wo_t) || (!p->mlp && (!w->W1_t || !w->W2_t))) {
        free_tw(w);
        return -1;
    }
    return 0;
}

/* per-row scratch */
typedef struct {
    double *n, *q, *kt, *vt, *cat, *a, *h, *u, *hid, *mo, *r, *logit;
    int maxpos;
} rto_ws;

static int make_ws(rto_ws *s, int d, int F, int maxpos, int H)
{
    /* one logit row per head, so that the heads of a position can be evaluated by different threads */
    size_t tot = (size_t)d * 9 + (size_t)F + (size_t)d + (size_t)maxpos * (size_t)H + 8;
    double *base = (double *)calloc(tot, sizeof(double));
    if (!base) return -1;
    s->n = base; s->q = s->n + d; s->kt = s->q + d; s->vt = s->kt + d; s->cat = s->vt + d;
    s->a = s->cat + d; s->h = s->a + d; s->u = s->h + d; s->mo = s->u + d; s->r = s->mo + d;
    s->hid = s->r + d; s->logit = s->hid + F;
    s->maxpos = maxpos;
    return 0;
}
static void free_ws(rto_ws *s) { free(s->n); }

/* q, temporary k and temporary v of one input row (Sec. 2.2, first display). */
static void project_qkv(const rto_params *p, const rto_tw *w, const double *x, rto_ws *s, int par)
{
    const int d = p->d, H = p->H, dh = p->dh;
    rms_norm(x, p->g_attn, d, p->eps, p->norm_free, s->n);
    matvec(w->Wq_t, d, d, s->n, s->u, par);
    matvec(w->Wk_t, d, d, s->n, s->mo, par);
    matvec(w->Wv_t, d, d, s->n, s->vt, par);
    for (int h = 0; h < H; ++h) {
        rms_norm(s->u + h * dh, p->g_q ? p->g_q + h * dh : NULL, dh, p->eps, p->norm_free, s->q + h * dh);
        rms_norm(s->mo + h * dh, p->g_k ? p->g_k + h * dh : NULL, dh, p->eps, p->norm_free, s->kt + h * dh);
    }
}

/* From the concatenated head outputs in s->cat: a, h, z (into y) and the persistent pair
 * of this position (into k_out, v_out).  Sec. 2.2, displays for z_i, k_i, v_i. */
static void finish_position(const rto_params *p, const rto_tw *w, const double *x, rto_ws *s,
                            double *y, double *k_out, double *v_out, int par)
{
    const int d = p->d, H = p->H, dh = p->dh, F = p->F;
    if (w->Wo_t) matvec(w->Wo_t, d, d, s->cat, s->a, par);
    else for (int i = 0; i < d; ++i) s->a[i] = s->cat[i];
    for (int i = 0; i < d; ++i) s->h[i] = x[i] + p->alpha * s->a[i];
    rms_norm(s->h, p->g_mlp, d, p->eps, p->norm_free, s->u);
    if (p->mlp) {
        p->mlp(s->u, s->mo, d, p->mlp_user);
    } else {
        matvec(w->W1_t, d, F, s->u, s->hid, par);
        for (int j = 0; j < F; ++j) s->hid[j] = gelu_erf(s->hid[j]);
        matvec(w->W2_t, F, d, s->hid, s->mo, par);
    }
    for (int i = 0; i < d; ++i) y[i] = s->h[i] + p->alpha * s->mo[i];
    rms_norm(y, p->g_kv, d, p->eps, p->norm_free, s->r);
    matvec(w->Wk_t, d, d, s->r, s->u, par);
    matvec(w->Wv_t, d, d, s->r, v_out, par);
    for (int h = 0; h < H; ++h)
        rms_norm(s->u + h * dh, p->g_k ? p->g_k + h * dh : NULL, dh, p->eps, p->norm_free, k_out + h * dh);
}

/* Attention of one position: persistent rows 0..t-1 of (K, V) for batch row b plus the
 * temporary pair (s->kt, s->vt); direct two-pass softmax.  attw (optional) gets [H][t+1] weights. */
static void attend(const rto_params *p, rto_ws *s, const double *K, const double *V, int B, int b, int t,
                   double *attw, int attw_stride, int par)
{
    const int H = p->H, dh = p->dh;
    /* heads are independent (Sec. 2, Notation); with par != 0 they are spread over the threads, each with its own
     * logit row, in the same arithmetic order as the serial loop */
#pragma omp parallel for schedule(static) if (par && t >= 64)
    for (int h = 0; h < H; ++h) {
        const double *q = s->q + h * dh;
        double *logit = s->logit + (size_t)h * s->maxpos;
        const double slope = alibi_slope(p, h);
        double mx = -INFINITY;
        for (int j = 0; j < t; ++j) {
            const double *kj = K + (((size_t)j * B + b) * H + h) * dh;
            logit[j] = p->attn_scale * dot(kj, q, dh) - slope * (double)(t - j);
            if (logit[j] > mx) mx = logit[j];
        }
        logit[t] = p->attn_scale * dot(s->kt + h * dh, q, dh);
        if (logit[t] > mx) mx = logit[t];
        double den = 0.0;
        for (int j = 0; j <= t; ++j) { logit[j] = exp(logit[j] - mx); den += logit[j]; }
        double *o = s->cat + h * dh;
        for (int c = 0; c < dh; ++c) o[c] = 0.0;
        for (int j = 0; j < t; ++j) {
            const double wj = logit[j] / den;
            const double *vj = V + (((size_t)j * B + b) * H + h) * dh;
            for (int c = 0; c < dh; ++c) o[c] += wj * vj[c];
            if (attw) attw[(size_t)h * attw_stride + j] = wj;
        }
        const double wt = logit[t] / den;
        for (int c = 0; c < dh; ++c) o[c] += wt * s->vt[h * dh + c];
        if (attw) attw[(size_t)h * attw_stride + t] = wt;
    }
}

static int pick_threads(const rto_params *p)
{
#ifdef _OPENMP
    int nt = p->threads > 0 ? p->threads : omp_get_max_threads();
    if (p->mlp) nt = 1; /* callbacks may not be re-entrant */
    return nt;
#else
    (void)p; return 1;
#endif
}

static int check_params(const rto_params *p)
{
    if (!p || p->d <= 0 || p->H <= 0 || p->dh <= 0 || p->H * p->dh != p->d) return -1;
    if (!p->Wq || !p->Wk || !p->Wv) return -1;
    if (!p->mlp && (!p->W1 || !p->W2 || p->F <= 0)) return -1;
    return 0;
}

/* One position t (0-based) of batch row b given persistent rows 0..t-1; writes y, K[t], V[t]. */
static void position(const rto_params *p, const rto_tw *w, rto_ws *s, const double *x_row, int B, int b, int t,
                     double *y_row, double *K, double *V, double *attw, int attw_stride, int par)
{
    const int H = p->H, dh = p->dh;
    project_qkv(p, w, x_row, s, par);
    attend(p, s, K, V, B, b, t, attw, attw_stride, par);
    double *k_out = K + (((size_t)t * B + b) * H) * dh;
    double *v_out = V + (((size_t)t * B + b) * H) * dh;
    finish_position(p, w, x_row, s, y_row, k_out, v_out, par);
}

/* attw: optional [B][H][N][N] attention weights (row i holds weights over j <= i, the last being
 * the temporary pair's). */
int rto_layer_prefill(const rto_params *p, const double *x, int B, int N, double *y, double *K, double *V,
                      int kv_cap, double *attw)
{
    if (check_params(p) || B <= 0 || N <= 0 || kv_cap < N) return -1;
    rto_tw w;
    if (make_tw(p, &w)) return -2;
    const int d = p->d, H = p->H;
    const int nt = pick_threads(p);
    const int outer = B >= 2 && nt > 1;              /* batch rows in parallel (one thread per sequence) */
    const int inner = !outer && nt > 1 && d >= 256;  /* else split matrix rows */
    rto_ws *ws = (rto_ws *)calloc((size_t)B, sizeof(rto_ws));
    int err = ws ? 0 : -2;
    for (int b = 0; b < B && !err; ++b) if (make_ws(&ws[b], d, p->F > 0 ? p->F : 1, N + 1, H)) err = -2;
    if (!err) {
#ifdef _OPENMP
        omp_set_num_threads(nt);
#endif
        for (int t = 0; t < N; ++t) {
#pragma omp parallel for schedule(static) if (outer)
            for (int b = 0; b < B; ++b) {
                double *aw = attw ? attw + (((size_t)b * H) * N + t) * N : NULL;
                position(p, &w, &ws[b], x + ((size_t)b * N + t) * d, B, b, t, y + ((size_t)b * N + t) * d,
                         K, V, aw, N * N, inner);
            }
        }
    }
    if (ws) { for (int b = 0; b < B; ++b) if (ws[b].n) free_ws(&ws[b]); free(ws); }
    free_tw(&w);
    return err;
}

/* Blocked recurrence (Sec. 8, Discussion: "recurrence executed over blocks of steps", given as an extension in
 * one sentence).  Reading: the positions are cut into blocks of S; a position attends the PERSISTENT pairs of all
 * positions in earlier blocks, and the TEMPORARY pairs (from the layer input) of the positions of its own block up to
 * and including itself - inside a block the layer is the Transformer layer of Sec. 2.1, across blocks the RT layer of
 * Sec. 2.2, so the outputs of a block do not depend on each other and the recurrent depth is ceil(N / S).  S = 1 is
 * the RT layer, S >= N the Transformer layer.  K, V receive the persistent pairs.  Serial (a test oracle). */
int rto_layer_prefill_blocked(const rto_params *p, const double *x, int B, int N, int S, double *y, double *K, double *V,
                              int kv_cap)
{
    if (check_params(p) || B <= 0 || N <= 0 || kv_cap < N || S <= 0) return -1;
    rto_tw w;
    if (make_tw(p, &w)) return -2;
    const int d = p->d, H = p->H, dh = p->dh;
    rto_ws s;
    if (make_ws(&s, d, p->F > 0 ? p->F : 1, N + 1, H)) { free_tw(&w); return -2; }
    const int Sb = S < N ? S : N;
    double *Kp = (double *)malloc(sizeof(double) * (size_t)Sb * d), *Vp = (double *)malloc(sizeof(double) * (size_t)Sb * d);
    int err = (Kp && Vp) ? 0 : -2;
    for (int b = 0; b < B && !err; ++b) {
        for (int t0 = 0; t0 < N; t0 += S) {
            const int t1 = t0 + S < N ? t0 + S : N;
            /* rows t0..t1-1 of K, V hold the temporary pairs while the block is evaluated */
            for (int t = t0; t < t1; ++t) {
                project_qkv(p, &w, x + ((size_t)b * N + t) * d, &s, 0);
                memcpy(K + (((size_t)t * B + b) * H) * dh, s.kt, sizeof(double) * d);
                memcpy(V + (((size_t)t * B + b) * H) * dh, s.vt, sizeof(double) * d);
            }
            for (int t = t0; t < t1; ++t) {
                const double *xr = x + ((size_t)b * N + t) * d;
                project_qkv(p, &w, xr, &s, 0);
                attend(p, &s, K, V, B, b, t, NULL, 0, 0); /* rows < t0 persistent, rows t0..t-1 temporary, own pair */
                finish_position(p, &w, xr, &s, y + ((size_t)b * N + t) * d, Kp + (size_t)(t - t0) * d,
                                Vp + (size_t)(t - t0) * d, 0);
            }
            for (int t = t0; t < t1; ++t) {
                memcpy(K + (((size_t)t * B + b) * H) * dh, Kp + (size_t)(t - t0) * d, sizeof(double) * d);
                memcpy(V + (((size_t)t * B + b) * H) * dh, Vp + (size_t)(t - t0) * d, sizeof(double) * d);
            }
        }
    }
    free(Kp); free(Vp);
    free_ws(&s);
    free_tw(&w);
    return err;
}

int rto_decode_step(const rto_params *p, const double *x_t, int B, int t, double *y_t, double *K, double *V,
                    int kv_cap)
{
    if (check_params(p) || B <= 0 || t < 0 || t >= kv_cap) return -1;
    rto_tw w;
    if (make_tw(p, &w)) return -2;
    rto_ws s;
    if (make_ws(&s, p->d, p->F > 0 ? p->F : 1, t + 1, p->H)) { free_tw(&w); return -2; }
    for (int b = 0; b < B; ++b)
        position(p, &w, &s, x_t + (size_t)b * p->d, B, b, t, y_t + (size_t)b * p->d, K, V, NULL, 0, 0);
    free_ws(&s);
    free_tw(&w);
    return 0;
}

/* Standard causal layer of Sec. 2.1: keys/values from the layer input at every position.
 * K, V receive those pairs (same layout); attw as in rto_layer_prefill. */
int rto_transformer_layer(const rto_params *p, const double *x, int B, int N, double *y, double *K, double *V,
                          int kv_cap, double *attw)
{
    if (check_params(p) || B <= 0 || N <= 0 || kv_cap < N) return -1;
    rto_tw w;
    if (make_tw(p, &w)) return -2;
    const int d = p->d, H = p->H, dh = p->dh, F = p->F;
    rto_ws s;
    if (make_ws(&s, d, F > 0 ? F : 1, N + 1, p->H)) { free_tw(&w); return -2; }
    for (int b = 0; b < B; ++b) {
        for (int t = 0; t < N; ++t) {
            const double *xr = x + ((size_t)b * N + t) * d;
            double *yr = y + ((size_t)b * N + t) * d;
            project_qkv(p, &w, xr, &s, 0);
            /* own pair is stored first, then attention runs over rows 0..t inclusive */
            double *k_row = K + (((size_t)t * B + b) * H) * dh;
            double *v_row = V + (((size_t)t * B + b) * H) * dh;
            for (int i = 0; i < d; ++i) { k_row[i] = s.kt[i]; v_row[i] = s.vt[i]; }
            double *aw = attw ? attw + (((size_t)b * H) * N + t) * N : NULL;
            attend(p, &s, K, V, B, b, t, aw, N * N, 0); /* rows < t persistent + (kt, vt) == row t */
            if (w.Wo_t) matvec(w.Wo_t, d, d, s.cat, s.a, 0);
            else for (int i = 0; i < d; ++i) s.a[i] = s.cat[i];
            for (int i = 0; i < d; ++i) s.h[i] = xr[i] + p->alpha * s.a[i];
            rms_norm(s.h, p->g_mlp, d, p->eps, p->norm_free, s.u);
            if (p->mlp) p->mlp(s.u, s.mo, d, p->mlp_user);
            else {
                matvec(w.W1_t, d, F, s.u, s.hid, 0);
                for (int j = 0; j < F; ++j) s.hid[j] = gelu_erf(s.hid[j]);
                matvec(w.W2_t, F, d, s.hid, s.mo, 0);
            }
            for (int i = 0; i < d; ++i) yr[i] = s.h[i] + p->alpha * s.mo[i];
        }
    }
    free_ws(&s);
    free_tw(&w);
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Appendix C taken literally.
 * ------------------------------------------------------------------------------------------ */

/* Algorithm 2: fold KV rows (k[j], v[j]), j in [0, nkv), into the running (m, l, o) of nq queries.
 * q, k, v rows have `stride` doubles between consecutive positions; o rows are dense [nq][dh].
 * Positional bias: query i of the tile is dist0 + i - j positions after key j, logit -= slope * that. */
void rto_update_tile(const double *q, int nq, int q_stride, const double *k, const double *v, int nkv,
                     int kv_stride, int dh, double scale, double *m, double *l, double *o, double slope, int dist0)
{
    double *logit = (double *)malloc(sizeof(double) * (size_t)(nkv > 0 ? nkv : 1));
    for (int i = 0; i < nq; ++i) {
        const double *qi = q + (size_t)i * q_stride;
        double m_tile = -INFINITY;
        for (int j = 0; j < nkv; ++j) {
            logit[j] = scale * dot(k + (size_t)j * kv_stride, qi, dh) - slope * (double)(dist0 + i - j);
            if (logit[j] > m_tile) m_tile = logit[j];
        }
        const double m_new = m[i] > m_tile ? m[i] : m_tile;
        const double resc = exp(m[i] - m_new); /* exp(-inf) = 0 on first touch */
        for (int c = 0; c < dh; ++c) o[(size_t)i * dh + c] *= resc;
        l[i] *= resc;
        for (int j = 0; j < nkv; ++j) {
            const double e = exp(logit[j] - m_new);
            const double *vj = v + (size_t)j * kv_stride;
            for (int c = 0; c < dh; ++c) o[(size_t)i * dh + c] += vj[c] * e;
            l[i] += e;
        }
        m[i] = m_new;
    }
    free(logit);
}

/* Events of Algorithm 1 for a sequence of length N, 1-based inclusive ranges:
 * out[6*e + 0..5] = t, P, u, v, s, e.  Returns the number of events (<= cap is the caller's job:
 * there are at most N-1). */
int rto_schedule(int N, int32_t *out, int cap)
{
    int n = 0;
    for (int t = 1; t <= N; ++t) {
        int P = 1;
        while (t % (2 * P) == 0) P *= 2;
        const int u = t + 1, v = (t + P < N) ? t + P : N;
        if (u <= v) {
            if (n < cap && out) {
                int32_t *r = out + 6 * (size_t)n;
                r[0] = t; r[1] = P; r[2] = u; r[3] = v; r[4] = t - P + 1; r[5] = t;
            }
            ++n;
        }
    }
    return n;
}

/* Algorithm 1 with Algorithm 2 as its update primitive; single batch loop, read-modify-write
 * running statistics initialised to (-inf, 0, 0).
 * chunk = 0: the schedule as printed.  chunk = C > 0 (a power of two): the variant for a layer that knows its
 * queries only one chunk of C positions ahead - the blocks P < C are served as printed (their queries lie in the
 * block's own chunk), the blocks P >= C are not; instead, when position t = cC is finished, ONE UpdateTile folds
 * all keys 1..t into the queries t+1..min(t+C, N).  Every (query, earlier key) pair is still covered exactly once,
 * and UpdateTile is exact for any partition of the keys (Appendix C, online softmax), so the result is the same. */
int rto_layer_prefill_tiled(const rto_params *p, const double *x, int B, int N, double *y, double *K, double *V,
                            int kv_cap, int chunk)
{
    if (check_params(p) || B <= 0 || N <= 0 || kv_cap < N || chunk < 0 || (chunk & (chunk - 1))) return -1;
    rto_tw w;
    if (make_tw(p, &w)) return -2;
    const int d = p->d, H = p->H, dh = p->dh;
    rto_ws s;
    if (make_ws(&s, d, p->F > 0 ? p->F : 1, N + 1, p->H)) { free_tw(&w); return -2; }
    double *Q = (double *)malloc(sizeof(double) * (size_t)N * d);
    double *m = (double *)malloc(sizeof(double) * (size_t)N * H);
    double *l = (double *)malloc(sizeof(double) * (size_t)N * H);
    double *o = (double *)malloc(sizeof(double) * (size_t)N * d); /* [H][N][dh] */
    int err = (Q && m && l && o) ? 0 : -2;
    const int kvs = B * H * dh; /* doubles between consecutive positions of K, V */
    for (int b = 0; b < B && !err; ++b) {
        for (int i = 0; i < N; ++i) { /* line 1: all queries up front */
            project_qkv(p, &w, x + ((size_t)b * N + i) * d, &s, 0);
            memcpy(Q + (size_t)i * d, s.q, sizeof(double) * d);
        }
        for (size_t i = 0; i < (size_t)N * H; ++i) { m[i] = -INFINITY; l[i] = 0.0; }
        memset(o, 0, sizeof(double) * (size_t)N * d);
        for (int t = 1; t <= N; ++t) {
            const double *xr = x + ((size_t)b * N + (t - 1)) * d;
            project_qkv(p, &w, xr, &s, 0); /* temporary pair of position t */
            for (int h = 0; h < H; ++h) {
                double *mh = m + (size_t)h * N, *lh = l + (size_t)h * N, *oh = o + (size_t)h * N * dh;
                rto_update_tile(Q + (size_t)(t - 1) * d + h * dh, 1, d, s.kt + h * dh, s.vt + h * dh, 1, 0, dh,
                                p->attn_scale, mh + (t - 1), lh + (t - 1), oh + (size_t)(t - 1) * dh, 0.0, 0);
                for (int c = 0; c < dh; ++c) s.cat[h * dh + c] = oh[(size_t)(t - 1) * dh + c] / lh[t - 1];
            }
            double *k_out = K + (((size_t)(t - 1) * B + b) * H) * dh;
            double *v_out = V + (((size_t)(t - 1) * B + b) * H) * dh;
            finish_position(p, &w, xr, &s, y + ((size_t)b * N + (t - 1)) * d, k_out, v_out, 0);
            int P = 1;
            while (t % (2 * P) == 0) P *= 2;
            int u = t + 1, v = (t + P < N) ? t + P : N;
            int s0 = t - P + 1;
            if (chunk > 0 && P >= chunk) { /* chunked variant: every key so far against the next chunk's queries */
                v = (t + chunk < N) ? t + chunk : N;
                s0 = 1;
                P = t;
            }
            if (u <= v) {
                for (int h = 0; h < H; ++h) {
                    double *mh = m + (size_t)h * N, *lh = l + (size_t)h * N, *oh = o + (size_t)h * N * dh;
                    rto_update_tile(Q + (size_t)(u - 1) * d + h * dh, v - u + 1, d,
                                    K + (((size_t)(s0 - 1) * B + b) * H + h) * dh,
                                    V + (((size_t)(s0 - 1) * B + b) * H + h) * dh, P, kvs, dh, p->attn_scale,
                                    mh + (u - 1), lh + (u - 1), oh + (size_t)(u - 1) * dh, alibi_slope(p, h), u - s0);
                }
            }
        }
    }
    free(Q); free(m); free(l); free(o);
    free_ws(&s);
    free_tw(&w);
    return err;
}

int rto_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
