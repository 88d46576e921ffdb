// Launch sequences of the bf16 matrix-core path: one transformer layer and the head.
#include "mfma_common.h"

bf16_t *mfma_lo(pd_ctx *c, void *buf, size_t cols) {
  // every activation buffer is sized for fp32 rows; the low parts live in its second half or, for
  // packed pairs, 8 rows further down the same fragment (64 elements: 8 rows of 8-element granules)
  if (!c->opt_split) return nullptr;
  return c->packed ? (bf16_t *)buf + 64 : (bf16_t *)buf + (size_t)c->R_pad * cols;
}

// fields every projection of a launch sequence shares
void mfma_gemm_base(pd_ctx *c, GemmArgs &a, int R) {
  const pd_config &g = c->cfg;
  memset(&a, 0, sizeof(a));
  a.R = R; a.rt = c->rows; a.d = g.d_model; a.H = g.n_head; a.hd = g.head_dim; a.kv_cap = c->kv_cap;
  a.packed = c->packed;
  a.stream_w = c->stream_loads;
}

// QKV-style projection of the normalised rows in c->xn: queries to c->q, keys and values into the given
// caches at the rows' slots.  `n_tiles` 16-column tiles of W, whose first d columns are section `sec0`
// (0: queries, then keys, then values; 1: keys, then values).
// An output projection (contraction over d_model) can prepare the next norm, and the projection behind
// that norm finish it, when every block of both launches works on one row tile: steps of at most 16 rows,
// and steps of up to 128 rows whose projections are launched with a row tile per block (here: a d x d
// producer and a d x d consumer; wider consumers are checked where they are launched).
bool mfma_can_fuse_norm(pd_ctx *c, int R) {
  if (!c->opt_fuse_norm) return false;
  const int d = c->cfg.d_model;
  return R <= 16 || mfma_gemm_row_tile_blocks(d / 16, d, R, 1);
}
// The second FFN projection has to give up its cut along K over blocks for this, which leaves one block
// per 16 output columns.  With the next layer's QKV projection finishing the norm, a step of the 768 / 3072
// shape measured 0.198 ms against 0.188 ms and one of the 2048 / 8192 shape 1.33-1.34 ms against 1.31 ms
// (the uncut projection loses what the norm kernel took): only on request (value 2 of the option).
static bool ffn2_prepares_norm(pd_ctx *c, int R) {
  return R <= 16 && mfma_can_fuse_norm(c, R) && c->opt_fuse_norm == 2 && c->cfg.pos_kind != 1;
}

int mfma_qkv(pd_ctx *c, GemmArgs &a, const bf16_t *W, int n_tiles, int sec0, void *kc, void *vc, void *kc_lo,
             void *vc_lo, int R, hipStream_t s, const float *c1, const float *c2) {
  const pd_config &g = c->cfg;
  const int d = g.d_model;
  a.W = W; a.xn = (const bf16_t *)c->xn; a.xn_lo = mfma_lo(c, c->xn, d); a.K = d;
  a.n_tiles = n_tiles; a.sec0 = sec0; a.out_bf = (bf16_t *)c->q; a.out_lo = mfma_lo(c, c->q, d);
  a.kc = (f16_t *)kc; a.vc = (f16_t *)vc; a.rope_cs = c->rope_cs;
  a.kc_lo = (f16_t *)kc_lo; a.vc_lo = (f16_t *)vc_lo; a.kv_sat = c->kv_sat;
  if (c1) {
    a.stats_in = c->nstats; a.stats_tiles = d / 16; a.c1 = c1; a.c2 = g.norm_kind == 0 ? c2 : nullptr;
    a.norm_kind = g.norm_kind; a.norm_d = d; a.norm_eps = g.norm_eps;
    int rc = mfma_gemm(EPI_QKV_NORM, a, R, s);
    a.stats_in = nullptr;
    c->norm_fused = false;
    return rc;
  }
  return mfma_gemm(g.pos_kind == 1 ? EPI_QKV_ROPE : EPI_QKV, a, R, s);
}

// output projection of the attention result in c->att, added to the residual stream (as split-K slices
// that the next norm kernel sums)
int mfma_out(pd_ctx *c, GemmArgs &a, const bf16_t *p_wo, int R, hipStream_t s, const float *next_gain) {
  const int d = c->cfg.d_model;
  a.W = p_wo; a.xn = (const bf16_t *)c->att; a.xn_lo = mfma_lo(c, c->att, d); a.K = d; a.n_tiles = d / 16; a.x = c->ypart; a.ld = d;
  a.part_stride = (size_t)c->R_pad * d; a.max_parts = 4; a.parts_out = &c->pend_parts;
  if (next_gain && mfma_can_fuse_norm(c, R)) {
    a.x_res = c->x; a.gain = next_gain; a.stats_out = c->nstats;
    a.out_bf = (bf16_t *)c->xn; a.out_lo = mfma_lo(c, c->xn, d);
    c->norm_fused = true;
    return mfma_gemm(EPI_RESID_NORM, a, R, s);
  }
  return mfma_gemm(EPI_RESID, a, R, s);
}

// output projection + residual, the norm in front of the FFN, the FFN + residual
int mfma_out_ffn(pd_ctx *c, GemmArgs &a, const bf16_t *p_wo, const LayerPtrs &lw, int R, hipStream_t s,
                 const float *next_gain) {
  const pd_config &g = c->cfg;
  int d = g.d_model, ff = g.d_ff, rc;
  a.W = p_wo; a.xn = (const bf16_t *)c->att; a.xn_lo = mfma_lo(c, c->att, d); a.K = d; a.n_tiles = d / 16; a.x = c->ypart; a.ld = d;
  a.part_stride = (size_t)c->R_pad * d; a.max_parts = 4; a.parts_out = &c->pend_parts;
  // At most 16 rows: the projection is not cut along K over blocks, so its epilogue holds the final
  // x + y.  It writes x, gain * x as the activation fragments of the FFN, and per-tile row sums; the
  // first FFN projection finishes the norm in its epilogue and the norm kernel in between is gone.
  const int ffn1_tiles = (g.ffn_kind == 1 ? 2 : 1) * ff / 16;
  const bool fuse = lw.c1 && mfma_can_fuse_norm(c, R) && (R <= 16 || mfma_gemm_row_tile_blocks(ffn1_tiles, d, R, 1));
  if (fuse) {
    a.x_res = c->x; a.gain = lw.n2g; a.stats_out = c->nstats;
    a.out_bf = (bf16_t *)c->xn; a.out_lo = mfma_lo(c, c->xn, d);
    if ((rc = mfma_gemm(EPI_RESID_NORM, a, R, s))) return rc;
    a.stats_in = c->nstats; a.stats_tiles = d / 16; a.c1 = lw.c1; a.c2 = g.norm_kind == 0 ? lw.c2 : nullptr;
    a.norm_kind = g.norm_kind; a.norm_d = d; a.norm_eps = g.norm_eps;
  } else {
    if ((rc = mfma_gemm(EPI_RESID, a, R, s))) return rc;
    if ((rc = mfma_norm(c, lw.n2g, lw.n2b, R, s))) return rc;
  }
  // FFN
  a.xn = (const bf16_t *)c->xn; a.xn_lo = mfma_lo(c, c->xn, d); a.K = d;
  a.out_bf = (bf16_t *)c->hb; a.out_lo = mfma_lo(c, c->hb, ff); a.ld = ff; a.W = lw.p_w1;
  if (g.ffn_kind == 1) {
    a.n_tiles = 2 * ff / 16;
    rc = mfma_gemm(EPI_SWIGLU, a, R, s);
  } else {
    a.n_tiles = ff / 16; a.act = g.ffn_kind == 2 ? 1 : 0;
    rc = mfma_gemm(EPI_GELU, a, R, s);
  }
  if (rc) return rc;
  a.stats_in = nullptr;
  a.W = lw.p_w2; a.xn = (const bf16_t *)c->hb; a.xn_lo = mfma_lo(c, c->hb, ff); a.K = ff; a.n_tiles = d / 16; a.x = c->ypart; a.ld = d;
  if (next_gain && ffn2_prepares_norm(c, R)) {
    // completes x itself and leaves gain * x with the row sums for the next layer's QKV projection
    a.x_res = c->x; a.gain = next_gain; a.stats_out = c->nstats;
    a.out_bf = (bf16_t *)c->xn; a.out_lo = mfma_lo(c, c->xn, d);
    c->norm_fused = true;
    return mfma_gemm(EPI_RESID_NORM, a, R, s);
  }
  return mfma_gemm(EPI_RESID, a, R, s);
}

int mfma_layer(pd_ctx *c, int l, int R, int A, int nreq, int req0, int kv_override, hipStream_t s,
               const AttnMode *mode) {
  const pd_config &g = c->cfg;
  const LayerPtrs &lw = c->layers[l];
  int rc;
  // the previous layer's second FFN projection may have prepared this norm already
  const bool finish = c->norm_fused;
  if (!finish && (rc = mfma_norm(c, lw.n1g, lw.n1b, R, s))) return rc;
  GemmArgs a;
  mfma_gemm_base(c, a, R);
  // QKV projection (+ rotary) + KV append
  if ((rc = mfma_qkv(c, a, lw.p_wqkv, 3 * g.d_model / 16, 0, lw.kc, lw.vc, lw.kc_lo, lw.vc_lo, R, s,
                     finish ? lw.q1 : nullptr, finish ? lw.q2 : nullptr)))
    return rc;
  // context pass, last layer: only its keys and values are ever used (nothing reads the residual
  // stream of a context token after the last layer)
  if (kv_override >= 0 && l == g.n_layer - 1 && !mode) return PD_OK;
  if ((rc = mfma_attention(c, lw, A, nreq, req0, kv_override, s, mode))) return rc;
  const bool decode_step = kv_override < 0 && !mode;
  return mfma_out_ffn(c, a, lw.p_wo, lw, R, s, decode_step && l + 1 < g.n_layer ? c->layers[l + 1].n1g : nullptr);
}

int mfma_head(pd_ctx *c, int R, bool want_logits, hipStream_t s, float *logits_to) {
  const pd_config &g = c->cfg;
  int rc;
  if ((rc = mfma_norm(c, c->fng, c->fnb, R, s))) return rc;
  GemmArgs a;
  memset(&a, 0, sizeof(a));
  a.R = R; a.rt = c->rows; a.W = c->p_lm_head; a.xn = (const bf16_t *)c->xn; a.packed = c->packed;
  a.stream_w = c->stream_loads;
  a.xn_lo = mfma_lo(c, c->xn, g.d_model); a.K = g.d_model;
  a.n_tiles = c->vocab_pad / 16; a.V = g.vocab;
  a.logits = want_logits ? (logits_to ? logits_to : c->logits) : nullptr; a.ld_logits = g.vocab;
  a.part_val = c->lm_part_val; a.part_idx = c->lm_part_idx;
  // leaves one winner per 16-column tile; the commit kernel picks the winner of each row
  return mfma_gemm(EPI_LM, a, R, s);
}
