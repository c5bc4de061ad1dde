/*
 * rt.h -- C ABI of the MI355X (gfx950) Recurrent Transformer layer library (librt_hip.so).
 *
 * One RT layer: forward (prefill, decoding step) and backward (rt_layer_backward).  Per position i (paper Sec. 2.2, "The Recurrent Transformer layer"):
 *
 *     n_i      = RMS(x_i; g_attn)
 *     q_i      = qkRMS(Wq n_i; g_q)     k_i^tmp = qkRMS(Wk n_i; g_k)     v_i^tmp = Wv n_i
 *     a_i      = Wo * concat_heads Attn((k_1,v_1) ... (k_{i-1},v_{i-1}), (k_i^tmp,v_i^tmp); q_i)
 *     h_i      = x_i + alpha a_i
 *     z_i      = h_i + alpha W2 gelu(W1 RMS(h_i; g_mlp))                 (layer output, y)
 *     k_i      = qkRMS(Wk RMS(z_i; g_kv); g_k)     v_i = Wv RMS(z_i; g_kv)       (persistent pair)
 *
 * with Attn the softmax-weighted sum over logits attn_scale*<k,q> (Sec. 2, Notation; the paper's
 * logits are unscaled, attn_scale = 1; optionally minus an ALiBi bias, rt_config.alibi_max_bias), RMS(u) = g * u / sqrt(mean(u^2) + eps), qkRMS the same
 * normalisation on each head's slice, exact (erf) GELU, no biases, alpha the 1/sqrt(L) residual
 * scale of Sec. 2.  Persistent pairs of positions j < i only, plus position i's own temporary
 * pair: that is the whole causal mask.
 *
 * rt_layer_prefill evaluates all N positions with the exact tiled schedule of Appendix C
 * (Algorithms 1 and 2): when position t is finished and P is the largest power of two dividing t,
 * the KV block [t-P+1, t] is folded into the softmax state of queries [t+1, min(t+P, N)].  Blocks
 * smaller than the context's p_min are instead attended directly when each query is finished
 * (Algorithm 1's free "query tile size" parameter); results do not depend on p_min beyond rounding.
 *
 * All pointers named "device" are device (HBM) addresses valid on rt_config.device.  The calls return
 * without synchronising, and their work is ordered on rt_config.stream: it starts after everything
 * enqueued there before the call, and whatever is enqueued there after the call sees its outputs.
 * Every entry point enqueues on that stream alone except rt_stack_prefill, which puts two of its three
 * groups of layers on streams the context owns, forked from and joined back into rt_config.stream by
 * events inside the call (see there).  The caller owns x, y, K, V and the weights; the context owns
 * only scratch memory.  No exceptions cross this boundary.
 */
#ifndef RT_H_
#define RT_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rt_ctx rt_ctx; /* opaque */

typedef enum {
    RT_OK = 0,
    RT_ERR_INVALID_ARG = 1, /* null pointer, size out of range, overlapping x / y, t >= kv_cap ... */
    RT_ERR_UNSUPPORTED = 2, /* shape or dtype the kernels do not cover (head_dim != 64, ...) */
    RT_ERR_OOM = 3,         /* scratch allocation failed */
    RT_ERR_HIP = 4,         /* a HIP runtime call failed; see rt_last_error */
    RT_ERR_STATE = 5        /* context unusable (earlier failure, or a bounded device-side wait expired) */
} rt_status;

typedef enum { RT_F32 = 0, RT_BF16 = 1 } rt_dtype; /* storage type of x, y, K, V, weights and gains */

/* rt_config.flags */
#define RT_FLAG_NORM_FREE 0x1u       /* every RMS / qkRMS is the identity (Appendix A's norm-free layer) */
#define RT_FLAG_ENGINE_STEPWISE 0x2u /* drive the sequential loop as one set of kernel launches per position */
#define RT_FLAG_ENGINE_PERSISTENT 0x4u /* require the single persistent weight-stationary kernel (error if it cannot run) */
#define RT_FLAG_NO_MFMA 0x8u         /* use the plain-ALU kernels also for bf16 storage (cross-checks) */
#define RT_FLAG_HIP_GRAPH 0x10u      /* stepwise engine: capture the launches of a prefill in a HIP graph and replay it */
#define RT_FLAG_DEBUG_POISON 0x20u   /* debugging: before every prefill (any engine, stacks, blocked recurrence) all stored
                                        partial softmax states are set to NaN, so that a state read before this call has
                                        written it - a slip in one of the schedules - reaches the outputs as NaN */

typedef struct {
    int32_t d_model, n_heads, head_dim, d_hidden; /* n_heads * head_dim == d_model; head_dim must be 64 */
    int32_t max_batch, max_seq;                   /* sizes the scratch (queries, temporary pairs, partial states) */
    int32_t dtype;                                /* rt_dtype */
    int32_t p_min;                                /* smallest KV block handled by the cross-block kernel; power of
                                                     two, at most 1024, at least 32 when the MFMA kernels are in use
                                                     (bf16 without RT_FLAG_NO_MFMA), else at least 1; 0 = default (32) */
    float resid_scale;                            /* alpha = 1/sqrt(L) (Sec. 2); 1 for a single layer */
    float attn_scale;                             /* multiplies the logits; paper-literal 1 */
    float rms_eps;                                /* paper-literal 0; 1e-6 is the usual choice */
    uint32_t flags;
    int32_t device;                               /* HIP device ordinal */
    void *stream;                                 /* hipStream_t; NULL = the default stream */
    float alibi_max_bias;                         /* beta >= 0: linear positional bias (ALiBi) as in the paper's trained
                                                     models (Appendix D: maximum bias 8.0): the logit of query i and the
                                                     persistent key of position j < i is lowered by m_h (i - j), head
                                                     slopes m_h = 2^(-beta (h + 1) / H), h = 0..H-1; the temporary pair is
                                                     at distance 0.  0 = none (Sec. 2.2 as it stands) */
    /* Scratch that would otherwise be allocated by the first call that needs it; reserved at rt_create instead, so that
     * no later call allocates (all zero = allocate on first use): */
    int32_t reserve_stack_layers;                 /* rt_stack_prefill: scratch sets for this many layers ... */
    int32_t reserve_stack_chunk;                  /* ... at this chunk (0 = 64); a call with more layers or another chunk
                                                     still reallocates */
    uint32_t reserve;                             /* RT_RESERVE_* bits */
} rt_config;
#define RT_RESERVE_LOOP_FREE 0x1u /* rt_layer_recompute, rt_transformer_layer, rt_layer_prefill_blocked */
#define RT_RESERVE_BACKWARD 0x2u  /* rt_layer_backward */

/* Device pointers, caller-owned, read-only.  Matrices are row-major [out, in] (y = W u).
 * Gains: NULL = ones.  g_kv NULL = use g_attn.  g_q, g_k are [d_model] = [n_heads, head_dim]. */
typedef struct {
    const void *Wq, *Wk, *Wv, *Wo; /* [d, d] */
    const void *W1;                /* [F, d] */
    const void *W2;                /* [d, F] */
    const void *g_attn, *g_mlp, *g_kv;
    const void *g_q, *g_k;
} rt_layer_weights;

/* Create a context: validates cfg, allocates scratch on cfg->device.  *out is NULL on failure. */
rt_status rt_create(const rt_config *cfg, rt_ctx **out);

/* Whole-sequence forward of one layer (Appendix C, Algorithm 1: inputs x_{1:N}, outputs z_{1:N} and
 * the persistent pairs (k_{1:N}, v_{1:N})).
 *   x [B, N, d]  device, read-only, must not overlap y
 *   y [B, N, d]  device, written
 *   K, V [kv_cap, B, H, head_dim] device, position first (Sec. 6.3); rows 0..N-1 are written in place
 *   1 <= B <= max_batch, 1 <= N <= max_seq, N <= kv_cap.
 * Batch rows are independent; where the single-launch engine applies (bf16) it stages at most 16 of them, and a larger
 * batch runs as chunks of 16 rows one after the other on the stream, each chunk's pairs copied into K, V from a
 * buffer of 2 * max_seq * 16 * d elements that rt_create allocates when max_batch > 16.  With bf16 and the matrix-core
 * kernels, 49 to 128 rows run as a stack of one layer on rt_stack_prefill's engine, and more rows step through the
 * positions with all rows at once, the base-case products as batched matrix products; rt_create reserves the workspace
 * of the former when max_batch >= 49 and the scratch of the loop-free entry points, which the latter uses, when
 * max_batch >= 81 (where a reservation fails the call falls back to the chunks).
 * Host-detectable errors are returned before anything is enqueued and leave the outputs untouched. */
rt_status rt_layer_prefill(rt_ctx *ctx, const rt_layer_weights *w, const void *x, int32_t B, int32_t N, void *y,
                           void *K, void *V, int32_t kv_cap);

/* One position of the same recurrence over a caller-held cache (Sec. 7.3: decoding attends over the
 * cached persistent pairs like a Transformer).
 *   x_t [B, d] device; t is 0-based: rows 0..t-1 of K, V are valid, row t is written; y_t [B, d].
 *   0 <= t < kv_cap, t < max_seq.  N successive decode steps equal one prefill of length N.
 *   x_t, y_t, K and V must not overlap one another (RT_ERR_INVALID_ARG, nothing enqueued).
 * bf16 storage with the MFMA kernels, d_model in {256, 512, 768, 1024}, d_hidden = 4 d_model, B n_heads <= 256, on a
 * device with 256 compute units: the whole step is ONE kernel launch of one workgroup per compute unit (engine name
 * "decode-single-launch"): the cache rows and the rows of all six matrices are requested at its start, the base case
 * runs on weight slices held in LDS, and the workgroups exchange the vectors between the products through memory.  The
 * workgroups wait for one another, so two such steps must not run at the same time on one device (two contexts on two
 * streams): each could hold part of the chip and wait for the rest; their bounded waits would then expire
 * (rt_device_wait_expired) instead of hanging.  Steps on one stream are ordered and safe.  A batch of up to three times
 * the rows one launch takes (min(16, 256 / n_heads)) runs as one such launch per chunk of rows, one after the other.  Any
 * other shape, dtype or batch size, and contexts created with RT_FLAG_ENGINE_STEPWISE, take eight launches per step instead. */
rt_status rt_decode_step(rt_ctx *ctx, const rt_layer_weights *w, const void *x_t, int32_t B, int32_t t, void *y_t,
                         void *K, void *V, int32_t kv_cap);

/* rt_decode_step for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  No context is needed and nothing is allocated or freed, on the device or through any
 * allocating library routine: the step's scratch (the position's query and temporary pair, one partial softmax state per
 * 64 cached keys, the vectors between the base case's products) is a static device array of RT_STATIC_SCRATCH_BYTES that
 * every device the library runs on holds until the process ends.  Same arguments as rt_decode_step; the step runs as
 * eight launches - the kernels, and bit for bit the results, of rt_decode_step on a context created from *cfg with
 * RT_FLAG_ENGINE_STEPWISE (cfg->max_batch and cfg->max_seq still bound B and t; cfg->stream is the stream the step is
 * enqueued on).
 *   Limit: the scratch of the call, about B (66 n_heads ceil(t / 64) + 11 d_model + 3 d_hidden) 4 bytes, must fit the
 *   array (d_model 1024, d_hidden 4096, B = 8: t < 16000); a larger call returns RT_ERR_INVALID_ARG and enqueues
 *   nothing.  rt_last_error(NULL) gives the reason of the calling thread's last failed call.
 *   All calls on one device share the one array, which keeps the previous call's contents (every word a step reads it
 *   has written before, so nothing is cleared): two steps that overlap in time on one device - different streams,
 *   different threads - race.  Steps enqueued on one stream are ordered and safe. */
#define RT_STATIC_SCRATCH_BYTES (8u << 20)
rt_status rt_decode_step_static(const rt_config *cfg, const rt_layer_weights *w, const void *x_t, int32_t B, int32_t t,
                                void *y_t, void *K, void *V, int32_t kv_cap);

/* Whole-sequence forward of a stack of L layers, layer l + 1 reading layer l's output (Sec. 2: the layers of a
 * model are stacked; Sec. 2.2: each RT layer has its own persistent key-value memory).  Same results as L
 * successive rt_layer_prefill calls up to rounding, but the layers run concurrently, layer l working `chunk`
 * positions behind layer l - 1 (the queries of a layer depend only on its input, Sec. 5, so a layer can start a
 * chunk as soon as the layer below has finished it).  Inside a chunk the schedule is Appendix C, Algorithm 1;
 * the keys before the chunk are folded into the chunk's queries by one UpdateTile (Algorithm 2) when the layer
 * enters the chunk.
 *   layers [L] host array of weight structs (device pointers inside); x [B, N, d] device, input of layer 0;
 *   y, K, V: host arrays of L device pointers: y[l] [B, N, d] output of layer l (all L are written: y[l] is layer
 *   l + 1's input), K[l], V[l] [kv_cap, B, H, head_dim] rows 0..N-1 written.  No two of these tensors may overlap.
 *   chunk: power of two >= p_min (>= 64 with the MFMA kernels); 0 = 64.
 * Unless rt_config.reserve_stack_layers reserved them at rt_create, the first call allocates one scratch set per layer
 * (RT_ERR_OOM if that fails); it is kept until rt_destroy and
 * reused by later calls with the same chunk and at most as many layers (another shape synchronises the stream
 * and reallocates).  The layers run as three groups: the first on rt_config.stream, the others on two streams that
 * the context owns (default priority; they start after the work already enqueued on rt_config.stream and that
 * stream continues after them; the environment variable RT_WAVE_STREAMS = 1..4 sets the number of layer groups /
 * streams, default 3).
 * rt_decode_step continues from the caches layer by layer. */
rt_status rt_stack_prefill(rt_ctx *ctx, const rt_layer_weights *layers, int32_t L, const void *x, int32_t B, int32_t N,
                           void *const *y, void *const *K, void *const *V, int32_t kv_cap, int32_t chunk);

/* The same layer evaluated without the sequential loop, given its output (Sec. 6.1, "Activation checkpointing": with
 * z known, all persistent pairs k_i, v_i = proj(RMS(z_i)) can be rebuilt at once and every intermediate recomputed in
 * parallel): K, V rows 0..N-1 are written from z, then y_i = the layer's output at position i computed from x_i, the
 * temporary pair of i and the persistent pairs of positions < i - one masked causal attention over all positions
 * (a single flash-style pass; Algorithm 1's blocks are not needed once every pair is known) and three GEMMs.  If z is the layer's true output for x, y reproduces it up to rounding (by induction over
 * the positions z is the only fixed point).  This is the forward half of a training step's recompute; rt_layer_backward
 * does its own recompute.
 *   x, z [B, N, d] device, read-only; y [B, N, d] written; K, V [kv_cap, B, H, head_dim] rows 0..N-1 written.
 *   bf16 storage with the MFMA kernels and d_hidden a multiple of 64: matrix-core GEMMs and one masked attention pass.
 *   Any other context (fp32 storage, RT_FLAG_NO_MFMA, another hidden width): the same results from the plain-ALU
 *   kernels (one wavefront per (b, h, position) for the attention, the products in tiles of eight rows) - for checking
 *   at fp32 tolerance, not for speed.
 * The first call allocates activation scratch for max_batch x max_seq rows (kept until rt_destroy) unless
 * RT_RESERVE_LOOP_FREE reserved it at rt_create. */
rt_status rt_layer_recompute(rt_ctx *ctx, const rt_layer_weights *w, const void *x, const void *z, int32_t B, int32_t N,
                             void *y, void *K, void *V, int32_t kv_cap);

/* The standard Transformer layer of Sec. 2.1 on the same kernels (the comparison layer of the paper's Figure 4): keys
 * and values of every position come from the layer input, k_i = qkRMS(Wk RMS(x_i)), v_i = Wv RMS(x_i), attention over
 * positions <= i, then the same output projection, residuals and MLP.  Same arguments and limits as
 * rt_layer_recompute (K, V receive the pairs). */
rt_status rt_transformer_layer(rt_ctx *ctx, const rt_layer_weights *w, const void *x, int32_t B, int32_t N, void *y,
                               void *K, void *V, int32_t kv_cap);

/* Blocked recurrence, the extension the paper's Discussion (Sec. 8) names in one sentence: the recurrence advances by
 * blocks of positions instead of single positions, so that the block length trades depth in time for speed.  Reading taken: the
 * positions are cut into blocks of `block`; position i attends the persistent pairs k_j, v_j = proj(RMS(z_j)) of the
 * positions j in EARLIER blocks and the temporary pairs (from the layer input) of the positions of its OWN block up
 * to and including itself.  Inside a block this is the Transformer layer of Sec. 2.1, across blocks the RT layer of
 * Sec. 2.2; the sequential loop runs over ceil(N / block) blocks whose `block` x B rows go through the matrix
 * products together.  block = 1 is rt_layer_prefill's layer (a different, slower evaluation of it), block >= N would
 * be rt_transformer_layer's.  K, V receive the persistent pairs.
 *   block: power of two, 1 <= block <= p_min.  Other arguments and the two kernel paths as rt_layer_recompute. */
rt_status rt_layer_prefill_blocked(rt_ctx *ctx, const rt_layer_weights *w, const void *x, int32_t B, int32_t N, int32_t block,
                                   void *y, void *K, void *V, int32_t kv_cap);

/* Where rt_layer_backward writes the gradients of the parameters: device, fp32, same shapes as the parameters
 * (matrices [out, in] row-major, gains [d_model]); written, not accumulated.  A null pointer skips that tensor. */
typedef struct {
    float *Wq, *Wk, *Wv, *Wo; /* [d, d] */
    float *W1;                /* [F, d] */
    float *W2;                /* [d, F] */
    float *g_attn, *g_mlp, *g_kv;
    float *g_q, *g_k;
} rt_layer_grads;

/* Backward pass of one RT layer (Sec. 6.4, "The backward pass"), with the forward intermediates recomputed from the
 * layer's input and output (Sec. 6.1, "Activation checkpointing": given z, all persistent pairs are rebuilt at once and
 * the remaining intermediates follow in parallel).  For the map (x, parameters) -> (y, K, V) of rt_layer_prefill and
 *     L = <gy, y> + <gK, K> + <gV, V>
 * it returns dL/dx and dL/d(parameter).  As Sec. 6.4 lays out, only the gradients of the persistent pairs are carried
 * through the reverse loop over positions (position i needs the complete gradient of its z_i, which depends on k_i, v_i,
 * before its attention can pass gradient to earlier pairs); the gradients of x, q, the temporary pairs and every parameter
 * are batched products after the loop.  Earlier pairs are reached in Algorithm 1's blocks run backwards (Appendix C).
 *   x, z [B, N, d] device, storage dtype, read-only: z must be the layer's output for x (from rt_layer_prefill).
 *   gy [B, N, d] storage dtype: gradient arriving at y.  gK, gV [N, B, H, head_dim] storage dtype or NULL (zero):
 *   gradients arriving at the returned persistent pairs (e.g. from decoding steps that read the cache).
 *   dx [B, N, d] fp32, written.  grads: see rt_layer_grads.  When rt_layer_weights.g_kv is NULL (RMS(z) shares g_attn)
 *   that share is added into grads->g_attn and grads->g_kv, if given, is zero-filled; gradients are also produced for
 *   gains that were passed as NULL (implicit ones).  With RT_FLAG_NORM_FREE the gain gradients are zero.
 *   1 <= B <= max_batch, 1 <= N <= min(max_seq, 65535).  dx and the gradient tensors must not overlap anything else.
 * All arithmetic is fp32 whatever the storage dtype.  The first call allocates scratch for max_batch x max_seq positions
 * (about (33 d + 3 F) 4 bytes per position; RT_ERR_OOM if that fails), kept until rt_destroy, unless RT_RESERVE_BACKWARD
 * reserved it at rt_create. */
rt_status rt_layer_backward(rt_ctx *ctx, const rt_layer_weights *w, const void *x, const void *z, const void *gy,
                            const void *gK, const void *gV, int32_t B, int32_t N, float *dx, const rt_layer_grads *grads);

/* Input of the first layer of a stack (Sec. 2: a sequence of token embeddings enters the first layer):
 *   x[b, n, :] = table[ids[b * ids_stride + first + n], :]   for 0 <= b < B, 0 <= n < N.
 *   table [vocab, d] device, storage dtype; ids device int32; x [B, N, d] device, written.
 * An id outside [0, vocab) is clamped into the table.  B, N >= 1 (not limited by max_batch / max_seq:
 * no scratch is used). */
rt_status rt_embed_rows(rt_ctx *ctx, const void *table, int32_t vocab, const int32_t *ids, int64_t ids_stride, int32_t first,
                        int32_t B, int32_t N, void *x);

/* Read-out of a stack: logits[b, v] = < W_lm[v, :], RMS(z_b; g_final) >, the final normalisation being
 * the same RMS as inside the layers (Sec. 2, Notation) and W_lm an untied [vocab, d] matrix.
 *   z: B rows of d elements, row b at z + b * z_stride elements (so the last position of a [B, N, d]
 *   tensor can be passed without a copy); g_final [d] or NULL = ones; logits [B, vocab] fp32 device, written.
 *   1 <= B <= max_batch. */
rt_status rt_lm_head(rt_ctx *ctx, const void *W_lm, const void *g_final, int32_t vocab, const void *z, int64_t z_stride,
                     int32_t B, float *logits);

/* Waits for nothing: the caller synchronises the stream first.  Frees scratch.  NULL is allowed. */
rt_status rt_destroy(rt_ctx *ctx);

/* Text of the last error on this context (owned by the context).  ctx == NULL: the reason of the calling thread's last
 * failed rt_decode_step_static call, or a static string if there was none. */
const char *rt_last_error(const rt_ctx *ctx);

const char *rt_status_string(rt_status s);

/* Bytes of device scratch the context holds. */
uint64_t rt_workspace_bytes(const rt_ctx *ctx);

/* After the stream has been synchronised: 0 if every bounded device-side wait of the last call on
 * this context completed, non-zero if one expired (the call's outputs are then invalid). */
int32_t rt_device_wait_expired(rt_ctx *ctx);

/* Name of the engine the last prefill call on this context used: "stepwise", "stepwise+graph",
 * "persistent", "wavefront" (rt_stack_prefill), "recompute", "transformer", "blocked", "backward", or "" before the first call. */
const char *rt_engine_name(const rt_ctx *ctx);

/* Diagnostics of the persistent engine, after the stream has been synchronised: when the environment
 * variable RT_PERSIST_TRACE was set at rt_create, copies for each of the first `rows` positions sixteen
 * 100 MHz clock stamps of workgroup 0 (slot 0 start, 1..6 end of phases M, cross-block items, O, 1, 2, KV,
 * 7..13 points inside the phases, 14 and 15 the end of the first grid barrier and of the tile work of a cross-block event) into out[rows][16] (host memory).  Returns the number of rows written, 0 if tracing is off. */
int32_t rt_phase_trace(rt_ctx *ctx, uint64_t *out, int32_t rows);

/* Diagnostics of the single-launch decoding step, after the stream has been synchronised: when the environment variable
 * RT_DECODE_TRACE was set at rt_create, copies for each of the first `workgroups` workgroups of the last step thirteen
 * 100 MHz clock stamps (0 start, 1 input rows and [Wq; Wk; Wv] rows staged, 2 raw q, k, v sent, 3 the other weight
 * slices staged, 4 this workgroup's cache chunks folded, 5 its wavefronts' states combined, 6 partial state or attention
 * output sent, 7..11 end of the base case's products Wo, W1, W2 (partial), W2 (sum), [Wk; Wv], 12 end) into
 * out[workgroups][16] (host memory).  Returns the number of rows written, 0 if tracing is off. */
int32_t rt_decode_phase_trace(rt_ctx *ctx, uint64_t *out, int32_t workgroups);

/* Diagnostics / measurement: run one cross-block UpdateTile (Appendix C, Algorithm 2) again, by itself, on the
 * state the last rt_layer_prefill of this context left behind (its queries and transposed values in scratch, the
 * caller's K, V): queries t1+1 .. t1+nq (1-based) against the keys t1-P+1 .. t1.  Rewrites those queries' partial
 * states of level log2(P) with the values the stand-alone kernel computes; outputs of the prefill are not touched.
 * The tile runs in the form that prefill's engine uses: after the persistent engine (and the loop-free layers) with
 * logits from the unrounded queries and keys (each rounded once to fp16, one product per logit tile; blocks of 32 keys:
 * bf16 head + remainder, three products), else with plain bf16 ones.
 *   B = batch of that prefill; P a power of two >= p_min; t1 a positive multiple of P; 1 <= nq <= P; t1 + nq <= N.
 * Used by the benchmark to time the cross-block kernel alone. */
rt_status rt_cross_block_event(rt_ctx *ctx, const void *K, const void *V, int32_t B, int32_t t1, int32_t P, int32_t nq);

/* Host-only: the cross-block events the driver issues for a sequence of length N with threshold
 * p_min (Appendix C, Algorithm 1, lines "P <- 2^nu2(t)" to the second UpdateTile call, restricted to
 * P >= p_min).  Event e: out[5e+0..4] = t, P, first query u, last query v, first key s (1-based,
 * inclusive; last key = t).  Pairs not covered by an event are covered by the direct window of
 * query i, keys [ (i-1) - ((i-1) mod p_min) + 1, i-1 ].  Returns the number of events; writes at most
 * cap of them (out may be NULL when cap == 0). */
int32_t rt_schedule_events(int32_t N, int32_t p_min, int32_t *out, int32_t cap);

/* Host-only: the events of the persistent engine, whose block decomposition is shifted by one key:
 * query i takes key i-1 directly, and keys 1..i-2 are split by the bits of c = i-2 (1-based keys; c is
 * the number of keys before the newest one).  Event e: out[5e+0..4] = t, P, first query u, last query v,
 * first key s, all 1-based inclusive, where t = last key of the block (a multiple of P >= p_min), the
 * queries are t+2 .. min(t+P+1, N), and the partial of query i is stored in the slot of (log2 P, query i-1).
 * The direct window of query i is keys [c - (c mod p_min) + 1, c] with c = i-2, plus key i-1. */
int32_t rt_schedule_events_shifted(int32_t N, int32_t p_min, int32_t *out, int32_t cap);

/* Host-only: the events rt_stack_prefill issues for each layer (positions of that layer, 1-based as above): the events
 * of rt_schedule_events with p_min <= P < chunk unchanged, and for every t that is a multiple of chunk one event with
 * P = t, s = 1 (every key so far) and queries t+1 .. min(t+chunk, N), whose partial states are stored one per query
 * beside the levels of the blocks.  All queries of an event lie in one chunk of `chunk` positions, the one a layer has
 * just entered when the event is issued.  chunk: power of two >= p_min. */
int32_t rt_schedule_events_chunked(int32_t N, int32_t p_min, int32_t chunk, int32_t *out, int32_t cap);

/* Host-only: index of the partial-state slot of (level, query), or -1 if that query takes no tile at
 * that level.  level = log2(P); query is 1-based.  Slots of one level are dense in [0, ceil(N/2)). */
int64_t rt_partial_slot(int32_t level, int32_t query);

/* Library version: major*10000 + minor*100 + patch. */
int32_t rt_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RT_H_ */
