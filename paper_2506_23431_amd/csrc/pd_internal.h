// Internal declarations shared by the HIP sources of libpd.  Not part of the ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>
#include <vector>

#include "pd.h"

typedef uint16_t bf16_t;   // raw bf16 bit pattern

// ---------------------------------------------------------------------------
// error plumbing
// ---------------------------------------------------------------------------
void pd_set_error(const char *fmt, ...);

#define PD_CHECK_HIP(expr)                                                         \
  do {                                                                             \
    hipError_t e_ = (expr);                                                        \
    if (e_ != hipSuccess) {                                                        \
      pd_set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
      return PD_EHIP;                                                              \
    }                                                                              \
  } while (0)

#define PD_REQUIRE(cond, code, ...)                                                \
  do {                                                                             \
    if (!(cond)) {                                                                 \
      pd_set_error(__VA_ARGS__);                                                   \
      return (code);                                                               \
    }                                                                              \
  } while (0)

// ---------------------------------------------------------------------------
// device helpers
// ---------------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even; inputs are finite in this library
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// fp16 bit patterns for the KV cache of dtype 1: same two bytes per element as bf16, 11-bit
// significand.  Values beyond the fp16 range saturate instead of becoming infinite.
typedef _Float16 f16_t;
__device__ __forceinline__ f16_t f32_to_f16_sat(float f) {
  return (f16_t)fminf(fmaxf(f, -65504.f), 65504.f);
}

__device__ __forceinline__ float ld_f32(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float ld_f32(const f16_t *p, size_t i) { return (float)p[i]; }
__device__ __forceinline__ void st_f32(f16_t *p, size_t i, float v) { p[i] = f32_to_f16_sat(v); }
__device__ __forceinline__ float ld_f32(const bf16_t *p, size_t i) { return bf16_to_f32(p[i]); }
__device__ __forceinline__ void st_f32(float *p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void st_f32(bf16_t *p, size_t i, float v) { p[i] = f32_to_bf16(v); }

// ---------------------------------------------------------------------------
// per-row tables written by the schedule tick (decode) or the prefill set-up.
// Row r of a launch belongs to request row_req[r]; invalid rows have flags == 0.
// ---------------------------------------------------------------------------
#define ROW_VALID   1   // the row carries a token this step
#define ROW_PRODUCE 2   // a next token is selected from this row's logits

struct RowTables {
  int32_t *req;    // [R] request index
  int32_t *sub;    // [R] subsequence index (1-based); prefill rows: 0
  int32_t *tok;    // [R] token id fed
  int32_t *pos;    // [R] position index p
  int32_t *slot;   // [R] KV slot (unified index: context j -> j, generated g -> L + g)
  int32_t *lim;    // [R] keys with index < lim are visible unconditionally
  int32_t *flags;  // [R]
  int4 *qinfo;     // [R] {flags, sub, lim, req} again, packed so that one load fetches them
  int4 *kvinfo;    // [R] {flags, req, slot, pos} packed likewise (KV append epilogue)
};

// schedule state of Algorithm 1, one instance per request, all on the device
struct SchedState {
  int32_t *step;      // [B]   iterations started so far (t of the current step)
  int32_t *k_open;    // [B]   subsequences opened
  int32_t *n_tok;     // [B][S] tokens held incl. <bos> (0 = not opened)
  int32_t *n_fed;     // [B][S] tokens already fed to the decoder
  int32_t *fin;       // [B][S] finished flag (1 = by <eos>, 2 = by the length limit)
  int32_t *done;      // [B]   request terminated
  int32_t *steps;     // [B]   iterations run when it terminated
  int32_t *n_gen;     // [B]   generated-side KV slots in use
  int32_t *kv_len;    // [B]   L + n_gen
  int32_t *n_rows;    // [B]   rows this step
  int32_t *grid;      // [B][S][M+1] token grid, index 0 = <bos>
  uint16_t *gen_sub;  // [B][gen_stride] subsequence of each generated-side KV slot; the entry of key slot
                      // j >= L is j - (L & ~7), so that groups of 8 keys are 16-byte aligned
  int32_t *step_tok;  // [B][S] token appended this step (-1 = none)
  int32_t *force;     // [B][S] teacher-forcing input (-1 = none)
  int32_t *all_done;  // [1]   number of requests that have terminated
  int32_t *row_of;    // [B][S] row index of subsequence this step (-1 = none)
};

struct LayerPtrs {
  const void *wqkv, *wo, *w1, *w_up, *w2;          // caller's row-major matrices
  const float *n1g, *n1b, *n2g, *n2b;
  // MFMA path: re-packed copies inside the workspace
  bf16_t *p_wqkv, *p_wo, *p_w1, *p_w2;
  float *c1, *c2;                                  // p_w1 times the second norm's gain / bias, per packed column
  float *cx1;                                      // p_cq times the gain of the norm in front of it
  float *q1, *q2;                                  // p_wqkv times the first norm's gain / bias (layers after the first)
  void *kc, *vc;                                   // KV caches of this layer
  void *kc_lo, *vc_lo;                             // low halves (layers below kv_pair_layers), else NULL
  // encoder-decoder form, decoder layers: attention over the encoder states
  const void *cq, *ckv, *co;                       // caller's [d][d], [2d][d] (keys then values), [d][d]
  const float *n3g;                                // gain of the norm in front of it
  bf16_t *p_cq, *p_ckv, *p_co;
  void *xkc, *xvc;                                 // keys / values of the encoder states, this layer's projection
};

// What pd_encdec_create adds to a context (Eq. 1 as the paper runs it: a stacked encoder, a decoder with
// attention over its states, relative-position biases on bucketed distances, Section 4.3).
struct EncDecState {
  int n_enc_layer, rel_buckets, rel_max_distance;
  std::vector<LayerPtrs> enc;      // encoder layers (kc / vc: one scratch cache shared by all of them)
  const float *enc_fng;            // gain of the encoder's final norm
  const float *enc_rel_bias, *dec_rel_bias;   // caller's [buckets][H] tables (device)
  float *enc_bias, *dec_bias;      // [H][enc_len] / [H][dec_len]: bias by clamped distance, times log2(e)
  int enc_len, dec_len;            // 2 * max_distance + 1 (index: query - key + max_distance), max_distance + 1
  uint16_t *enc_coord;             // [kv_cap] entry j = j: coordinates of the encoder's keys
};

struct pd_ctx {
  pd_config cfg;
  const void *tok_emb, *pos_emb, *lm_head;
  bf16_t *p_lm_head;
  const float *fng, *fnb;
  std::vector<LayerPtrs> layers;
  int impl;                 // 0: fp32-activation kernels; 1: bf16 MFMA kernels
  int pair_layers;          // leading layers whose cache holds pairs of halves (kv_pair_layers resolved)
  int32_t *kv_sat;          // [1] keys / values stored saturated at the largest half since pd_create
  // capacities
  int gen_cap, gen_stride, kv_cap, R_cap, R_pad, vocab_pad, prefill_chunk, prefill_chunk_cap;
  size_t kv_layer_bytes;    // bytes of one K (or V) cache of one layer
  // workspace carve-up
  char *ws; size_t ws_bytes;
  float *x;                 // [R_cap][d] residual stream
  void *xn, *q, *att, *hb;  // activations (type depends on impl)
  float *qkv32;             // simple path: [R_cap][3d]
  float *logits;            // [decode rows][vocab] internal logits (simple path / parity output)
  float *scores;            // simple path attention scratch
  float *att_part;          // split-K partials of the attention kernel
  int part_units;           // records of 16 queries x (head_dim + 2) floats that att_part holds
  float *ypart;             // [4][R_pad][d] split-K partial sums of the O / FFN2 projections
  int pend_parts;           // slices of ypart the next norm kernel has to add to x
  float2 *nstats;           // [16][d/16] per-tile row sums left by the output projection for the next norm
  bool packed;              // this launch sequence keeps activations as packed pairs (at most 8 rows):
                            // high parts in rows 0-7 of a 16-row fragment, low parts in rows 8-15
  bool embed_pending;       // matrix-core path: the next norm kernel gathers x from the embedding tables
  int stream_loads;         // 1: a decode step touches more bytes than the last-level cache holds: weights, keys and
                            // values are loaded with the non-temporal hint (PD_OPT_STREAM_LOADS)
  bool norm_fused;          // the last residual projection left gain * x and per-tile row sums for the next
                            // norm: the projection that follows finishes it, no norm kernel runs
  float *lm_part_val; int32_t *lm_part_idx; int lm_parts;
  int32_t *row_argmax;      // [R_cap] argmax of each row's logits
  float *rope_cs;           // [max_pos][hd/2][2] cos, sin
  int rope_rows;
  RowTables rows;
  SchedState sch;
  int32_t *ctx_tok;         // [B][L] device copy of the context ids
  // decode parameters fixed by prefill
  int B, L, S, dt, M, time_max, A, R;
  // encoder-decoder form: arch == 1; L above is 0 (the decoder's cache holds generated tokens only)
  // and Lx is the length of the encoded input
  int arch, Lx;
  EncDecState ed;
  uint16_t *gen_coord;      // [B][gen_stride] grid coordinate (t - 1) + (i - 1) of each generated-side KV slot
  int4 *qinfo_x;            // [R] row table of the attention over the encoder states
  // teacher-forced forward (Section 3.3)
  float *bias0;             // [H] zeros: the one-entry "no bias" table of the kernels that carry coordinates
  float *nll;               // [R_pad] loss term of each row
  double *loss;             // [B]
  int32_t *tf_target;       // [B][S][M + 2] device copy of the training targets
  bool prefilled;
  int host_steps;           // decode steps enqueued since prefill/reset
  // options
  int opt_splits, opt_graph, opt_profile, opt_split, opt_chunk, opt_fuse_norm, opt_ctx_split, opt_ctx_attn;
  hipGraphExec_t graph_exec; bool graph_ready;
  std::vector<hipEvent_t> ev_pool; size_t ev_used;
  int32_t *h_pinned;        // small host staging buffer (pinned unless stage_pinned is false)
  bool stage_pinned;
};

// ---- launchers (each returns PD_OK or an error code) -----------------------
// schedule / glue (sched.hip)
int launch_reset_state(pd_ctx *c, hipStream_t s);
int launch_tick(pd_ctx *c, hipStream_t s);
int launch_prefill_rows(pd_ctx *c, int b, int p0, int n, hipStream_t s, int L, int bidir, int b_cache);
int launch_embed(pd_ctx *c, int R, hipStream_t s);
int launch_commit(pd_ctx *c, float *out_logits, hipStream_t s);
int launch_teacher_rows(pd_ctx *c, const int32_t *tgt_dev, int b, int ML, hipStream_t s);
int launch_row_nll(pd_ctx *c, const float *logits, int n, double *loss_dev, hipStream_t s);
int launch_rope_table(pd_ctx *c, hipStream_t s);
// fp32-activation path (simple.hip)
int simple_layer(pd_ctx *c, int l, int R, int A, int nreq, int req0, int kv_override, hipStream_t s);
int simple_head(pd_ctx *c, int R, hipStream_t s);
// MFMA path (mfma.hip)
int mfma_pack_weights(pd_ctx *c, hipStream_t s);
int mfma_fold_norms(pd_ctx *c, hipStream_t s);
struct AttnMode;
// mode != NULL: not a context pass (every layer runs to its end) and the attention launch takes the mode
int mfma_layer(pd_ctx *c, int l, int R, int A, int nreq, int req0, int kv_override, hipStream_t s,
               const AttnMode *mode = nullptr);
// logits_to != NULL: the logits of the R rows go there ([R][vocab]) instead of the internal buffer
int mfma_head(pd_ctx *c, int R, bool want_logits, hipStream_t s, float *logits_to = nullptr);
// encoder-decoder form (encdec.hip)
int encdec_pack_weights(pd_ctx *c, hipStream_t s);
int encdec_build_tables(pd_ctx *c, int *scratch, hipStream_t s);
int encdec_encode(pd_ctx *c, int b, hipStream_t s);                   // Eq. 1 for request b, then its cross keys / values
int encdec_decoder_layer(pd_ctx *c, int l, int R, hipStream_t s, int A = 0, int nreq = 0, int req0 = 0, int kv_self = -1);
size_t mfma_packed_weight_bytes(const pd_config *cfg);
