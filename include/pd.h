/*
 * pd.h -- C ABI of the pipelined-decoder library for AMD MI355X (gfx950).
 *
 * The library implements the decode hot path of the pipelined decoder (paper
 * Section 3): Algorithm 1 driven one time-step at a time, where every time-step
 * feeds the newest token of each open subsequence through a decoder-only
 * transformer (Eq. 3) under the dependency rule of Section 3.2 and selects the
 * most probable next token for each of them (Eq. 4).
 *
 * Conventions
 *   - "device" pointers are HIP device memory on the current device, "host"
 *     pointers are ordinary host memory.  The library never allocates or frees
 *     device memory: weights and the workspace are allocated by the caller (for
 *     example as PyTorch tensors) and must outlive the pd_ctx.
 *   - All matrices are row-major [out][in].  dtype 0: fp32 weights, fp32 KV cache.
 *     dtype 1: bf16 weights (raw 16-bit patterns), 16-bit KV cache (IEEE half: the same
 *     two bytes per element as bf16 with an 11-bit significand; values beyond +-65504
 *     saturate), fp32 accumulation and fp32 residual stream.  Norm gains/biases are
 *     always fp32.
 *   - Every function returns PD_OK (0) or a negative PD_E* code; on error no output
 *     argument is written and pd_last_error() describes the failure.  Nothing
 *     throws or aborts across this boundary.
 *   - A pd_ctx is not re-entrant: one thread and one stream at a time.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 */
#ifndef PD_H
#define PD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PD_OK      0
#define PD_EINVAL -1   /* bad argument: NULL, shape out of range, L > max_ctx, ...      */
#define PD_ESTATE -2   /* call out of order: decode step before prefill                 */
#define PD_ENOMEM -3   /* workspace too small                                            */
#define PD_EHIP   -4   /* a HIP runtime call failed                                      */

typedef struct pd_ctx pd_ctx;   /* opaque; owned by the library between create and destroy */

/* Model shape and capacity.  The paper only says "stacked transformer decoder";
 * the block is pre-norm, without linear biases:
 *   x0 = E_tok[token] (+ E_pos[p]);  h = x + Wo Attn(N1(x));  x' = h + FFN(N2(h));
 *   logits = W_lm N_f(x_last). */
typedef struct {
  int32_t n_layer, d_model, n_head, head_dim, d_ff, vocab;  /* n_head*head_dim == d_model */
  int32_t ffn_kind;    /* 0: W2 gelu_erf(W1 u);  1: W2 (silu(W1 u) * (W_up u))  (SwiGLU)   */
  int32_t norm_kind;   /* 0: LayerNorm(gain, bias);  1: RMSNorm(gain)                      */
  int32_t pos_kind;    /* 0: learned absolute table [max_pos][d];  1: rotary, rotate-half  */
  float   rope_base, norm_eps;
  int32_t dtype;       /* 0: fp32;  1: bf16 weights + 16-bit (half) KV, fp32 accumulate     */
  int32_t bos_id, eos_id;   /* eos_id < 0 disables end-of-sequence termination             */
  int32_t max_batch, max_ctx, max_sub, max_sub_tokens;   /* capacity (workspace sizing)    */
  int32_t max_pos;     /* rows of the learned position table (ignored for rotary)          */
  int32_t kv_pair_layers;   /* dtype 1: the first kv_pair_layers layers keep every key and value as
                             * a pair of halves (value = high + low, about 22 significant bits; twice
                             * the cache bytes and attention traffic of those layers).  0: none.
                             * -1: chosen by the library from the shape: 1 when d_model >= 4096, else 0.
                             * Reason: the first layer's attention output is most of the residual
                             * stream behind it, so its cache rounding reaches the logits undiluted,
                             * and the error grows with the score scale, i.e. with the width: measured
                             * with weights N(0, 0.02) it is 6e-4 of logit error at width 2048 (24
                             * layers) and 2e-2 - 3e-2 at width 4096 (32 layers); one pair layer brings
                             * the latter to 1.3e-3 for under 1 % of the step time.  Ignored for
                             * dtype 0.  pd_get_info reports the number in use.                    */
} pd_config;

/* Device pointers to the weights; per-layer entries are HOST arrays of n_layer
 * device pointers.  Read-only to the library. */
typedef struct {
  const void *tok_emb;        /* [vocab][d]                                  */
  const void *pos_emb;        /* [max_pos][d], NULL for rotary               */
  const void *lm_head;        /* [vocab][d] (not tied to tok_emb)            */
  const float *final_norm_g, *final_norm_b;   /* [d]; bias NULL for RMSNorm  */
  const void *const *wqkv;    /* [3d][d]: rows 0..d-1 = Q, d..2d-1 = K, 2d..3d-1 = V; head h = rows h*hd.. */
  const void *const *wo;      /* [d][d]                                      */
  const void *const *w1;      /* [ff][d]  (GELU: up;  SwiGLU: gate)          */
  const void *const *w_up;    /* [ff][d]  SwiGLU only, else NULL             */
  const void *const *w2;      /* [d][ff]                                     */
  const float *const *norm1_g, *const *norm1_b, *const *norm2_g, *const *norm2_b;   /* [d] */
} pd_weights;

/* Bytes of device workspace pd_create needs for this configuration (KV caches in
 * the library's own layout, re-packed weights for the bf16 path, activations,
 * schedule state).  Returns 0 if the configuration is invalid. */
size_t pd_workspace_bytes(const pd_config *cfg);

/* Creates a context on the current device.  `dev_workspace` (device, 256-byte
 * aligned, >= pd_workspace_bytes) is cleared and, for dtype 1, receives a
 * re-packed copy of every matrix; this runs on `hip_stream` and is complete when
 * the call returns. */
int pd_create(const pd_config *cfg, const pd_weights *w, void *dev_workspace, size_t bytes,
              void *hip_stream, pd_ctx **out);
int pd_destroy(pd_ctx *ctx);

/* Encodes B contexts of L tokens each (the role of Eq. 1: the input is encoded
 * once; here as the causal prefix of a decoder-only model, context token j at
 * position j) into the context KV cache, fixes the decode parameters of Algorithm 1
 * and resets time to t = 0.
 *   ctx_tokens  host int32 [B][L], ids in [0, vocab)
 *   n_sub       sub^max >= 1,  delta_t >= 1,  time_max >= 0
 *   max_sub_tokens  M >= 1: a subsequence also ends after M generated tokens
 * Asynchronous on hip_stream except for the copy of ctx_tokens. */
int pd_prefill_context(pd_ctx *ctx, const int32_t *ctx_tokens, int B, int L, int n_sub,
                       int delta_t, int max_sub_tokens, int time_max, void *hip_stream);

/* Advances Algorithm 1 by exactly one time-step t (lines 5-13): opens a new
 * subsequence when (t-1) mod delta_t == 0 and fewer than n_sub exist; feeds the
 * newest token of every subsequence that has one (position p = L + (t-1) + (i-1));
 * each row attends to all L context tokens plus the generated-side tokens of
 * subsequences i' <= i fed so far, including this step's (Section 3.2); appends
 * argmax(logits) (lowest index on ties, Eq. 4) to every unfinished subsequence;
 * marks requests whose opened subsequences have all finished.
 *   force_tokens  host int32 [B][n_sub] or NULL: where >= 0 the value replaces the
 *                 argmax result of that subsequence (teacher forcing)
 *   out_tokens    host int32 [B][n_sub] or NULL: token appended this step, -1 if none
 *   out_logits    DEVICE fp32 [B][n_sub][vocab] or NULL: logits of every row that was
 *                 fed this step (rows not fed are left untouched)
 *   out_all_done  host int32 or NULL: 1 when every request has terminated
 * Host outputs force a stream synchronisation; with all of them NULL the call
 * only enqueues work.  After termination further calls are no-ops. */
int pd_decode_step(pd_ctx *ctx, const int32_t *force_tokens, int32_t *out_tokens,
                   float *out_logits, int32_t *out_all_done, void *hip_stream);

/* pd_prefill_context followed by decode steps until every request has terminated
 * or time_max steps have run (Algorithm 1 as a whole).
 *   out_tokens  host int32 [B][n_sub][M]: the subsequences in index order without
 *               <bos>/<eos>, padded with -1
 *   out_lens    host int32 [B][n_sub]: tokens in each (0 for subsequences never opened)
 *   out_steps   host int32 [B]: time-steps run for each request
 * Synchronises the stream before returning. */
int pd_generate(pd_ctx *ctx, const int32_t *ctx_tokens, int B, int L, int n_sub, int delta_t,
                int max_sub_tokens, int time_max, int32_t *out_tokens, int32_t *out_lens,
                int32_t *out_steps, void *hip_stream);

/* pd_generate for callers that cannot allocate device memory (code under HIP graph capture nearby,
 * tight serving loops, harnesses that forbid hipMalloc): the workspace that pd_create takes from the
 * caller is a device array inside the library (PD_STATIC_WORKSPACE_BYTES, held by every GPU the
 * library runs on until the process ends), the context exists for this call only, and nothing that
 * allocates device or pinned host memory is called.  `cfg` and `w` as for pd_create (cfg's
 * capacities must cover B, L, n_sub and max_sub_tokens); the other arguments and the results are
 * those of pd_generate, bit for bit.  Configurations whose pd_workspace_bytes exceeds the array
 * return PD_ENOMEM.  Every call on a GPU uses that GPU's one array: the part a call needs is
 * cleared and the weights are re-packed into it each time, and calls that overlap on one GPU (other
 * threads, other streams) race.  Synchronises the stream before returning. */
#define PD_STATIC_WORKSPACE_BYTES (64u << 20)
int pd_generate_static(const pd_config *cfg, const pd_weights *w, const int32_t *ctx_tokens, int B,
                       int L, int n_sub, int delta_t, int max_sub_tokens, int time_max,
                       int32_t *out_tokens, int32_t *out_lens, int32_t *out_steps, void *hip_stream);

/* Encoder-decoder form, the form the paper itself runs (Eq. 1: H^E = Encoder(X), computed once per
 * request by a stacked bidirectional encoder; Eq. 3: every decoder layer attends to the generated
 * side under the dependency rule of Section 3.2, then to H^E; Section 4.3: the relative position of
 * two generated-side tokens is the Manhattan distance |t1 - t2| + |i1 - i2| of their grid
 * coordinates).  The backbone is the text-to-text transformer family that Section 4.3 names:
 * pre-norm blocks, RMS norm (gain only), W2 relu(W1 u), no biases in linear layers, scores q.k +
 * bias[head][bucket(relative position)] without a 1/sqrt(head_dim) factor, one bias table per stack
 * shared by its layers, no bias in the attention over H^E, no absolute positions.  bucket(n) for a
 * key n >= 0 positions behind the query: n below buckets/2, then logarithmic up to
 * rel_max_distance, the last bucket beyond; the encoder uses half of the buckets for keys behind or
 * at the query and half for keys ahead.  Readings: the decoder's distance is (t_q - t_k) + (i_q - i_k)
 * (both terms are non-negative on visible pairs); the vocabulary projection is a separate matrix.
 * bf16 weights only (the matrix-core kernels); n_head * head_dim == d_model; head_dim, d_model and
 * d_ff multiples of 32, head_dim <= 128; rel_buckets even; rel_max_distance <= 128;
 * max_ctx at most min(4096, 65536 / n_head) (the encoder runs a request's input as one launch
 * sequence).  Weight pointers as in pd_weights: per-layer entries are HOST arrays of device pointers. */
typedef struct {
  int32_t n_enc_layer, n_dec_layer, d_model, n_head, head_dim, d_ff, vocab;
  int32_t rel_buckets, rel_max_distance;
  float   norm_eps;
  int32_t bos_id, eos_id;
  int32_t max_batch, max_ctx, max_sub, max_sub_tokens;
} pd_encdec_config;

typedef struct {
  const void *tok_emb;            /* [vocab][d], shared by both stacks           */
  const void *lm_head;            /* [vocab][d]                                  */
  const float *enc_rel_bias, *dec_rel_bias;           /* [rel_buckets][n_head]   */
  const float *enc_final_norm_g, *dec_final_norm_g;   /* [d]                     */
  /* encoder layers (n_enc_layer entries each) */
  const void *const *enc_wqkv, *const *enc_wo, *const *enc_w1, *const *enc_w2;   /* as in pd_weights */
  const float *const *enc_norm1_g, *const *enc_norm2_g;
  /* decoder layers (n_dec_layer entries each): self-attention, attention over H^E, feed-forward */
  const void *const *dec_wqkv, *const *dec_wo, *const *dec_w1, *const *dec_w2;
  const void *const *cross_wq;    /* [d][d]                                      */
  const void *const *cross_wkv;   /* [2d][d]: rows 0..d-1 = K, d..2d-1 = V       */
  const void *const *cross_wo;    /* [d][d]                                      */
  const float *const *dec_norm1_g, *const *dec_norm3_g, *const *dec_norm2_g;     /* before self-attention,
                                                                   before the attention over H^E, before the FFN */
} pd_encdec_weights;

/* Workspace size and creation, as pd_workspace_bytes / pd_create.  The context is used through the
 * same calls as a decoder-only one: pd_prefill_context encodes the B inputs (Eq. 1) and fills every
 * decoder layer's keys and values of H^E; pd_decode_step, pd_generate, pd_decode_steps,
 * pd_reset_decode, pd_set_option and pd_get_info behave as described there (a row's position index is
 * its grid coordinate (t-1) + (i-1); there is no context part in the decoder's own cache). */
size_t pd_encdec_workspace_bytes(const pd_encdec_config *cfg);
int pd_encdec_create(const pd_encdec_config *cfg, const pd_encdec_weights *w, void *dev_workspace,
                     size_t bytes, void *hip_stream, pd_ctx **out);

/* Teacher-forced forward of Section 3.3 over the contexts encoded by the last pd_prefill_context (whose
 * n_sub and delta_t fix the grid): every token of the training targets of Eq. 5 is fed at its grid
 * coordinate tau = (i-1) delta_t + 1 + j in ONE pass per request under the matrix of Fig. 3b (a token sees
 * the whole input and the target tokens of subsequences i' <= i at times tau' <= tau), and the loss of
 * Eq. 6 is returned: the sum of -log P(next token) over every token that has a successor in its
 * subsequence.  Reading: the closing token of a subsequence has no term of its own but is a key for later
 * tokens, as Algorithm 1 feeds a finished subsequence's last token once.
 *   target       host int32 [B][n_sub][max_len]: subsequence i of request b as fed, normally <bos>, Y_i,
 *                <eos> (and the terminal <bos>, <eos>), padded with -1; empty subsequences only at the end;
 *                max_len <= max_sub_tokens + 2, and a request's tokens must fit its generated-side cache
 *                (n_sub * (max_sub_tokens + 1)) and one pass of rows
 *   out_logits   DEVICE fp32 [B][rows_cap][vocab]: logits of every target token of request b in
 *                subsequence-major order (row of token j of subsequence i = tokens of the subsequences
 *                before i, plus j); rows behind a request's last token are left untouched
 *   out_row_nll  host fp32 [B][rows_cap] or NULL: the term of every row (0 for rows without a successor)
 *   out_loss     host fp64 [B]: Eq. 6 per request (terms added in row order)
 *   out_rows     host int32 [B] or NULL: rows of each request
 * Both model forms, on the matrix-core kernels only (the encoder-decoder form adds the Manhattan-distance
 * bias of Section 4.3 between every visible pair and the attention over the encoder states).  Uses the
 * generated side of the KV caches and the schedule state as scratch and leaves the context at t = 0, as
 * pd_reset_decode does.  Synchronises. */
int pd_teacher_forced(pd_ctx *ctx, const int32_t *target, int max_len, float *out_logits, int rows_cap,
                      float *out_row_nll, double *out_loss, int32_t *out_rows, void *hip_stream);

/* Runs `n_steps` decode steps (no host inputs or outputs) back to back on the
 * stream; used for timing.  Does not synchronise. */
int pd_decode_steps(pd_ctx *ctx, int n_steps, void *hip_stream);

/* Restarts decoding at t = 0 for the contexts already encoded (keeps the context
 * KV cache, drops everything generated).  Asynchronous. */
int pd_reset_decode(pd_ctx *ctx, void *hip_stream);

/* Tunables and instrumentation.  Keys:
 *   PD_OPT_ATTN_SPLITS   work-groups per (request, head) in the attention kernel (0 = auto)
 *   PD_OPT_USE_GRAPH     1: replay each decode step from a captured HIP graph
 *   PD_OPT_PROFILE       1: bracket the attention kernel of every layer (the kernel that streams the
 *                        keys and values; not the small kernel that merges its partial results) with
 *                        HIP events;  2: bracket the pair of kernels  (adds event overhead to the
 *                        step; for measurement only);  3: no events: every decode step launches that
 *                        kernel one extra time, first, on the cache of the layer half the stack away
 *                        (other bytes of the same size) and into the same outputs, which the real launch
 *                        overwrites -- the time a run of steps gains by it, per launch, is what the kernel
 *                        costs where it runs (results unchanged; not for layers that keep pairs of halves)
 *   PD_OPT_SPLIT_ACT     bf16 path: 1 (default) carries every activation that enters a matrix
 *                        multiply as a pair of bf16 values (about 16 mantissa bits) and runs two
 *                        matrix-core passes per weight / key / value fragment; 0 uses plain bf16
 *                        activations (half the matrix-core work, larger rounding error)
 *   PD_OPT_PREFILL_CHUNK rows of the context pass per launch (0 = default: up to 4096 on the bf16
 *                        path, 128 on the fp32 path; other values are rounded up to a multiple
 *                        of 16 and capped at that default).  Results do not depend on it beyond
 *                        rounding order.
 *   PD_OPT_FUSE_NORM     1 (default): in steps of at most 16 rows (and of up to 128 rows against small
 *                        matrices, where every block works on one row tile) the output projection adds its result
 *                        to the residual stream itself, hands gain * x and per-tile row sums to the
 *                        first FFN projection, and that projection finishes the second norm of the
 *                        layer in its epilogue (one kernel less per layer); 0: a separate norm kernel,
 *                        as in steps with more rows.  Same results up to rounding order.
 *                        2: models without rotary positions also hand over the first norm of the next
 *                        layer the same way (second FFN projection -> QKV projection).  Not the default:
 *                        that projection then cannot be cut along K over blocks, and measured slower.
 *   PD_OPT_STREAM_LOADS  1: decode steps load weights, keys and values with the non-temporal hint; 0: ordinary
 *                        loads.  Chosen at creation from the configuration: 1 when the bytes a step reads at
 *                        full capacity (every weight, every request's keys and values) exceed the 256 MB
 *                        last-level cache, so that nothing of them would be found there a step later (cfg4:
 *                        1.37 -> 1.31 ms per step, cfg5 6.55 -> 6.09); 0 for models the cache serves step after
 *                        step (cfg2: 0.187 ms, 0.202 with the hint).  Same results bit for bit.
 *                        pd_get_info(PD_INFO_STREAM_LOADS) reports the setting.
 *   PD_OPT_CONTEXT_ATTN  attention kernel of the context pass (bf16 path, head_dim 64 or 128, layers without
 *                        pair caches): 1 (default) the kernel with 32 queries per block where a chunk makes
 *                        at least 512 such blocks, else the decode step's kernel (16 queries per block, split
 *                        over the keys); 0 always the decode step's kernel; 2 the 32-query kernel wherever the
 *                        shape allows it.  Same results up to rounding order.
 *   PD_OPT_CONTEXT_SPLIT_ACT  activations of the context pass (pd_prefill_context of a decoder-only context on
 *                        the matrix-core kernels): 1 (default) as pairs of bf16 values (high + low part, what the
 *                        decode step uses), 0 as single bf16 values (half the multiplies of its projections).
 *                        Measured over whole runs against the fp64 oracle: width 1024, 24 layers 4.2e-4 -> 2.6e-3
 *                        of logit error for 0.017 -> 0.014 s; width 2048, 24 layers 4.8e-4 -> 3.4e-3 for 0.047 ->
 *                        0.033 s (8192 context tokens), all tokens with a margin above 0.05 unchanged; width
 *                        4096, 32 layers 9.3e-4 -> 8.6e-2, outside the 2e-2 tolerance: a caller's trade, not the
 *                        library's.  pd_get_info(PD_INFO_CONTEXT_PAIRS) reports the setting in use.  */
#define PD_OPT_ATTN_SPLITS 1
#define PD_OPT_USE_GRAPH   2
#define PD_OPT_PROFILE     3
#define PD_OPT_SPLIT_ACT   4
#define PD_OPT_PREFILL_CHUNK 5
#define PD_OPT_FUSE_NORM 6
#define PD_OPT_CONTEXT_SPLIT_ACT 7
#define PD_OPT_STREAM_LOADS 8
#define PD_OPT_CONTEXT_ATTN 9
int pd_set_option(pd_ctx *ctx, int key, int value);

/* Average time in microseconds between the two events of the brackets recorded since the
 * last call (PD_OPT_PROFILE), and how many brackets there were.  Synchronises. */
int pd_profile_read(pd_ctx *ctx, double *attn_avg_us, int32_t *attn_launches);

/* Measurement aid, independent of any pd_ctx: bandwidth in GB/s (1e9 bytes/s) of a kernel that only
 * reads, the ceiling a memory-bound kernel of this size can reach on this device.  Reads `chunk_bytes`
 * per launch from `dev_buf` (DEVICE, 16-byte aligned, `buf_bytes` long; a different chunk every
 * launch, so make the buffer several times larger than the 256 MB last-level cache), `iters` launches
 * back to back between two HIP events; the time includes the gaps between launches, as it does for
 * the kernels of a decode step.  The last 256 bytes of the buffer may be written.  Synchronises. */
int pd_measure_read_bandwidth(const void *dev_buf, size_t buf_bytes, size_t chunk_bytes, int iters,
                              void *hip_stream, double *gb_per_s);

/* Facts about a context that the caller cannot see from outside.  Keys:
 *   PD_INFO_KERNEL_PATH     1: the bf16 matrix-core kernels run this configuration; 0: the plain
 *                           fp32-activation kernels do (dtype 0, and dtype 1 shapes the matrix-core
 *                           kernels do not cover: head_dim, d_model or d_ff not a multiple of 32, or
 *                           head_dim > 128) -- same results, far slower
 *   PD_INFO_KV_PAIR_LAYERS  layers whose cache holds pairs of halves (kv_pair_layers resolved)
 *   PD_INFO_CONTEXT_PAIRS   1: the context pass carries its activations as bf16 pairs; 0: as single bf16
 *                           values (PD_OPT_CONTEXT_SPLIT_ACT resolved)
 *   PD_INFO_STREAM_LOADS    1: decode steps use the non-temporal hint (PD_OPT_STREAM_LOADS)
 *   PD_INFO_KV_SATURATED    keys and values written since pd_create whose magnitude exceeded the
 *                           largest half (65504) and were stored as +-65504 (dtype 1 only; always
 *                           0 for dtype 0).  Non-zero means the 16-bit cache cannot represent
 *                           this model's keys or values and the logits are not to be trusted.
 *                           Synchronises `hip_stream`.                                           */
#define PD_INFO_KERNEL_PATH    1
#define PD_INFO_KV_PAIR_LAYERS 2
#define PD_INFO_KV_SATURATED   3
#define PD_INFO_CONTEXT_PAIRS  4
#define PD_INFO_STREAM_LOADS   5
int pd_get_info(pd_ctx *ctx, int key, void *hip_stream, int64_t *value);

/* Message for the last error on this thread (static storage, never NULL). */
const char *pd_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PD_H */
