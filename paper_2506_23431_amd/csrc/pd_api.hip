// Host side of the C ABI: argument validation, workspace carve-up, and the
// launch sequences for prefill / decode step / generate.  No arithmetic of the
// method lives here; every step runs in the kernels of sched/simple/mfma.hip.
#include <stdarg.h>
#include <stdlib.h>

#include <algorithm>
#include <mutex>
#include <new>

#include "mfma_common.h"

static thread_local char g_err[512] = "no error";

void pd_set_error(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

extern "C" const char *pd_last_error(void) { return g_err; }

// ---------------------------------------------------------------------------
// configuration checks and derived capacities
// ---------------------------------------------------------------------------
static int check_config(const pd_config *g) {
  PD_REQUIRE(g != nullptr, PD_EINVAL, "config is NULL");
  PD_REQUIRE(g->n_layer >= 1 && g->d_model >= 1 && g->n_head >= 1 && g->head_dim >= 2 &&
                 g->d_ff >= 1 && g->vocab >= 1,
             PD_EINVAL, "model dimensions must be positive");
  PD_REQUIRE((int64_t)g->n_head * g->head_dim == g->d_model, PD_EINVAL,
             "n_head * head_dim (%d * %d) != d_model (%d)", g->n_head, g->head_dim, g->d_model);
  PD_REQUIRE(g->head_dim % 2 == 0 && g->head_dim <= 256, PD_EINVAL,
             "head_dim must be even and <= 256 (got %d)", g->head_dim);
  PD_REQUIRE(g->ffn_kind == 0 || g->ffn_kind == 1, PD_EINVAL, "ffn_kind must be 0 or 1");
  PD_REQUIRE(g->norm_kind == 0 || g->norm_kind == 1, PD_EINVAL, "norm_kind must be 0 or 1");
  PD_REQUIRE(g->pos_kind == 0 || g->pos_kind == 1, PD_EINVAL, "pos_kind must be 0 or 1");
  PD_REQUIRE(g->dtype == 0 || g->dtype == 1, PD_EINVAL, "dtype must be 0 (fp32) or 1 (bf16)");
  PD_REQUIRE(g->norm_eps > 0.f, PD_EINVAL, "norm_eps must be positive");
  PD_REQUIRE(g->pos_kind == 0 || g->rope_base > 1.f, PD_EINVAL, "rope_base must be > 1");
  PD_REQUIRE(g->max_batch >= 1 && g->max_ctx >= 1 && g->max_sub >= 1 && g->max_sub_tokens >= 1,
             PD_EINVAL, "capacities (max_batch, max_ctx, max_sub, max_sub_tokens) must be >= 1");
  PD_REQUIRE(g->max_pos >= 1, PD_EINVAL, "max_pos must be >= 1");
  PD_REQUIRE(g->kv_pair_layers >= -1 && g->kv_pair_layers <= g->n_layer, PD_EINVAL,
             "kv_pair_layers = %d outside [-1, n_layer]", g->kv_pair_layers);
  PD_REQUIRE(g->bos_id >= 0 && g->bos_id < g->vocab, PD_EINVAL, "bos_id out of range");
  PD_REQUIRE(g->eos_id < g->vocab, PD_EINVAL, "eos_id out of range");
  PD_REQUIRE((int64_t)g->max_sub * (g->max_sub_tokens + 1) + g->max_ctx < (1 << 24), PD_EINVAL,
             "KV capacity too large");
  PD_REQUIRE(g->max_sub <= 65535, PD_EINVAL, "max_sub = %d exceeds 65535 (subsequence tags are 16 bit)",
             g->max_sub);
  return PD_OK;
}

// kv_pair_layers = -1: one pair layer from width 4096 on (where the cache rounding of the first
// layer alone reaches the logit tolerance), none below
static int resolve_pair_layers(const pd_config *g) {
  if (g->dtype != 1) return 0;
  if (g->kv_pair_layers >= 0) return g->kv_pair_layers;
  return g->d_model >= 4096 ? 1 : 0;
}

static bool mfma_eligible(const pd_config *g) {
  return g->dtype == 1 && g->head_dim % 32 == 0 && g->head_dim <= 128 && g->d_model % 32 == 0 &&
         g->d_ff % 32 == 0;
}

struct Carver {
  char *base; size_t off;
  template <typename T> T *take(size_t n) {
    off = (off + 255) & ~(size_t)255;
    T *p = base ? (T *)(base + off) : nullptr;
    off += n * sizeof(T);
    return p;
  }
};

// Lays the workspace out; with base == NULL only the size is computed.
// `e` != NULL: encoder-decoder form (g is the decoder stack's configuration derived from it).
static size_t carve(const pd_config *g, char *base, pd_ctx *c, const pd_encdec_config *e = nullptr) {
  pd_ctx tmp_ctx;
  pd_ctx *x = c ? c : &tmp_ctx;
  int d = g->d_model, ff = g->d_ff, H = g->n_head, hd = g->head_dim, V = g->vocab;
  int B = g->max_batch, S = g->max_sub, M = g->max_sub_tokens;
  x->impl = mfma_eligible(g) ? 1 : 0;
  x->pair_layers = resolve_pair_layers(g);
  x->gen_cap = S * (M + 1);
  x->gen_stride = (x->gen_cap + 8 + 7) / 8 * 8;
  // encoder-decoder form: the decoder's own caches hold generated tokens only and the caches of the
  // encoder states the input only; one capacity serves both kinds
  x->kv_cap = ((e ? std::max(g->max_ctx, x->gen_cap) : g->max_ctx + x->gen_cap) + 63) / 64 * 64;
  // Rows of the context pass per launch: as many as give the many-row projection kernel a block
  // per compute unit even for small matrices (measured: the cfg4 context pass takes 0.172 s in chunks
  // of 128 rows, 0.059 s in chunks of 1024, 0.052 s in chunks of 2048 and 0.049 s in chunks of 4096),
  // at most the 4096 (request, head, 16 rows) units of one attention launch allow.  The fp32 path
  // keeps one score row per (row, head) and stays at 128.
  {
    int cap = std::min(4096, 16 * (4096 / std::max(H, 1)) / 16 * 16);
    x->prefill_chunk_cap = x->impl == 1 ? std::max(128, std::min(cap, (g->max_ctx + 127) / 128 * 128)) : 128;
    x->prefill_chunk = x->prefill_chunk_cap;
  }
  int a_max = std::min(S, M + 1);
  x->R_cap = std::max(B * a_max, x->prefill_chunk_cap);
  // row buffers are read in tiles of 16 rows, 1/2/4/8 tiles per launch
  int tiles = (x->R_cap + 15) / 16, t2 = 1;
  while (t2 < tiles && t2 < 8) t2 *= 2;
  x->R_pad = std::max(tiles, t2) * 16;
  if (x->R_pad > 128) x->R_pad = (x->R_pad + 127) / 128 * 128;     // whole row groups of 128
  x->vocab_pad = (V + 63) / 64 * 64;
  size_t es = g->dtype == 0 ? 4 : 2;
  x->kv_layer_bytes = (size_t)B * H * x->kv_cap * hd * es;
  Carver cv{base, 0};
  x->layers.resize(g->n_layer);
  for (int l = 0; l < g->n_layer; ++l) {
    x->layers[l].kc = cv.take<char>(x->kv_layer_bytes);
    x->layers[l].vc = cv.take<char>(x->kv_layer_bytes);
    bool pair = l < x->pair_layers;
    x->layers[l].kc_lo = pair ? cv.take<char>(x->kv_layer_bytes) : nullptr;
    x->layers[l].vc_lo = pair ? cv.take<char>(x->kv_layer_bytes) : nullptr;
    x->layers[l].xkc = e ? cv.take<char>(x->kv_layer_bytes) : nullptr;
    x->layers[l].xvc = e ? cv.take<char>(x->kv_layer_bytes) : nullptr;
  }
  x->arch = e ? 1 : 0;
  x->gen_coord = nullptr; x->qinfo_x = nullptr;
  if (e) {
    EncDecState &ed = x->ed;
    ed.n_enc_layer = e->n_enc_layer; ed.rel_buckets = e->rel_buckets; ed.rel_max_distance = e->rel_max_distance;
    ed.enc_len = 2 * e->rel_max_distance + 1; ed.dec_len = e->rel_max_distance + 1;
    ed.enc.resize(e->n_enc_layer);
    // one scratch cache (a single request's keys and values) serves every encoder layer in turn
    void *ekc = cv.take<char>(x->kv_layer_bytes / B), *evc = cv.take<char>(x->kv_layer_bytes / B);
    for (LayerPtrs &lp : ed.enc) { lp.kc = ekc; lp.vc = evc; }
    ed.enc_bias = cv.take<float>((size_t)H * ed.enc_len);
    ed.dec_bias = cv.take<float>((size_t)H * ed.dec_len);
    ed.enc_coord = cv.take<uint16_t>(x->kv_cap);
  }
  x->gen_coord = cv.take<uint16_t>((size_t)B * x->gen_stride);
  x->bias0 = cv.take<float>(H);
  x->loss = cv.take<double>(B);
  x->tf_target = cv.take<int32_t>((size_t)B * S * (M + 2));
  size_t Rp = x->R_pad;
  x->x = cv.take<float>(Rp * d);
  x->xn = cv.take<float>(Rp * d);
  x->q = cv.take<float>(Rp * d);
  x->att = cv.take<float>(Rp * d);
  x->hb = cv.take<float>(Rp * ff);
  x->qkv32 = cv.take<float>(Rp * 3 * d);
  // logits exist for decode rows only (the context pass never runs the head)
  x->logits = cv.take<float>((size_t)((B * a_max + 15) / 16 * 16) * x->vocab_pad);
  x->scores = x->impl == 0 ? cv.take<float>((size_t)x->R_cap * H * x->kv_cap) : nullptr;
  // split partials of the attention kernel: one (max, sum, O) record of 16 queries per (request, head,
  // query group) unit and split; the launch caps its splits so that units * splits <= part_units
  {
    int units_dec = B * ((a_max + 15) / 16) * H, units_pre = (x->prefill_chunk_cap / 16) * H;
    x->part_units = std::max(std::max(units_dec, units_pre), 1024);
  }
  x->att_part = cv.take<float>((size_t)x->part_units * 16 * (hd + 2));
  x->ypart = cv.take<float>((size_t)4 * Rp * d);
  x->lm_parts = (x->vocab_pad / 16);
  x->lm_part_val = cv.take<float>((size_t)x->lm_parts * Rp);
  x->lm_part_idx = cv.take<int32_t>((size_t)x->lm_parts * Rp);
  x->row_argmax = cv.take<int32_t>(Rp);
  x->nll = cv.take<float>(Rp);
  x->rope_rows = g->pos_kind == 1 ? g->max_pos : 0;
  x->rope_cs = g->pos_kind == 1 ? cv.take<float>((size_t)x->rope_rows * hd) : nullptr;
  RowTables &rt = x->rows;
  rt.req = cv.take<int32_t>(Rp); rt.sub = cv.take<int32_t>(Rp); rt.tok = cv.take<int32_t>(Rp);
  rt.pos = cv.take<int32_t>(Rp); rt.slot = cv.take<int32_t>(Rp); rt.lim = cv.take<int32_t>(Rp);
  rt.flags = cv.take<int32_t>(Rp); rt.qinfo = cv.take<int4>(Rp); rt.kvinfo = cv.take<int4>(Rp);
  if (e) x->qinfo_x = cv.take<int4>(Rp);
  SchedState &st = x->sch;
  st.step = cv.take<int32_t>(B); st.k_open = cv.take<int32_t>(B);
  st.n_tok = cv.take<int32_t>((size_t)B * S); st.n_fed = cv.take<int32_t>((size_t)B * S);
  st.fin = cv.take<int32_t>((size_t)B * S); st.done = cv.take<int32_t>(B);
  st.steps = cv.take<int32_t>(B); st.n_gen = cv.take<int32_t>(B); st.kv_len = cv.take<int32_t>(B);
  st.n_rows = cv.take<int32_t>(B);
  st.grid = cv.take<int32_t>((size_t)B * S * (M + 1));
  st.gen_sub = cv.take<uint16_t>((size_t)B * x->gen_stride);
  st.step_tok = cv.take<int32_t>((size_t)B * S); st.force = cv.take<int32_t>((size_t)B * S);
  st.all_done = cv.take<int32_t>(1); st.row_of = cv.take<int32_t>((size_t)B * S);
  x->kv_sat = cv.take<int32_t>(1);
  x->ctx_tok = cv.take<int32_t>((size_t)B * g->max_ctx);
  if (x->impl == 1) {
    // re-packed weights: same element counts as the originals, rows padded to 16
    size_t dd = (size_t)d;
    for (int l = 0; l < g->n_layer; ++l) {
      LayerPtrs &lp = x->layers[l];
      lp.p_wqkv = cv.take<bf16_t>(3 * dd * d);
      lp.p_wo = cv.take<bf16_t>(dd * d);
      lp.p_w1 = cv.take<bf16_t>((g->ffn_kind == 1 ? 2 : 1) * (size_t)ff * d);
      lp.p_w2 = cv.take<bf16_t>(dd * ff);
      lp.c1 = cv.take<float>((g->ffn_kind == 1 ? 2 : 1) * (size_t)ff);
      lp.c2 = cv.take<float>((g->ffn_kind == 1 ? 2 : 1) * (size_t)ff);
      lp.cx1 = e ? cv.take<float>(dd) : nullptr;
      lp.q1 = cv.take<float>(3 * dd); lp.q2 = cv.take<float>(3 * dd);
    }
    x->nstats = cv.take<float2>(std::min<size_t>(Rp, 128) * (d / 16));   // steps of up to 128 rows hand norms over
    x->p_lm_head = cv.take<bf16_t>((size_t)x->vocab_pad * d);
    if (e) {
      for (LayerPtrs &lp : x->ed.enc) {
        lp.p_wqkv = cv.take<bf16_t>(3 * dd * d); lp.p_wo = cv.take<bf16_t>(dd * d);
        lp.p_w1 = cv.take<bf16_t>((size_t)ff * d); lp.p_w2 = cv.take<bf16_t>(dd * ff);
      }
      for (int l = 0; l < g->n_layer; ++l) {
        LayerPtrs &lp = x->layers[l];
        lp.p_cq = cv.take<bf16_t>(dd * d); lp.p_ckv = cv.take<bf16_t>(2 * dd * d); lp.p_co = cv.take<bf16_t>(dd * d);
      }
    }
  }
  return (cv.off + 255) & ~(size_t)255;
}

extern "C" size_t pd_workspace_bytes(const pd_config *cfg) {
  if (check_config(cfg) != PD_OK) return 0;
  return carve(cfg, nullptr, nullptr);
}

// ---------------------------------------------------------------------------
// create / destroy
// ---------------------------------------------------------------------------
__global__ void k_fill_zero(uint4 *p, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
    p[i] = make_uint4(0, 0, 0, 0);
}

// Second half of context creation, shared by both model forms: options, staging buffer, clearing
// the workspace, re-packing the weights.  `c` has its configuration, pointers and carve-up.
static int finish_create(pd_ctx *c, size_t need, void *hip_stream, bool no_alloc, pd_ctx **out) {
  c->prefilled = false; c->host_steps = 0;
  c->embed_pending = false; c->norm_fused = false; c->packed = false; c->opt_splits = 0; c->opt_graph = 0; c->opt_profile = 0; c->opt_split = 1; c->opt_chunk = 0; c->opt_fuse_norm = 1; c->opt_ctx_split = 1; c->opt_ctx_attn = 1;
  c->graph_exec = nullptr; c->graph_ready = false; c->ev_used = 0; c->h_pinned = nullptr;
  c->B = c->L = c->Lx = c->S = c->dt = c->M = c->time_max = c->A = c->R = 0;
  {
    // what a decode step reads at full capacity: every weight once, every request's keys and values once per
    // layer.  Beyond the 256 MB last-level cache nothing survives from one step to the next and the loads
    // take the non-temporal hint (PD_OPT_STREAM_LOADS overrides).
    const pd_config &g = c->cfg;
    // (encoder-decoder form: a decoder layer also reads the two d x d projections around its attention over
    // the encoder states, and that attention's keys and values)
    const double attn_mats = c->arch == 1 ? 6.0 : 4.0, caches = c->arch == 1 ? 2.0 : 1.0;
    const double wbytes = 2.0 * ((double)g.n_layer * (attn_mats * g.d_model * g.d_model +
                                                      (g.ffn_kind == 1 ? 3.0 : 2.0) * g.d_model * g.d_ff) +
                                 (double)g.vocab * g.d_model);
    const double kvbytes = caches * 2.0 * g.max_batch * (double)g.n_layer * 2.0 * c->kv_cap * g.d_model;
    c->stream_loads = (c->impl == 1 && wbytes + kvbytes > 256.0 * (1 << 20)) ? 1 : 0;
  }
  hipStream_t s = (hipStream_t)hip_stream;
  auto fail = [&](int code) { (void)pd_destroy(c); return code; };
  const size_t n_stage = 2 * (size_t)c->cfg.max_batch * c->cfg.max_sub + 16;
  hipError_t e = hipSuccess;
  c->stage_pinned = !no_alloc;
  if (no_alloc) {
    c->h_pinned = new (std::nothrow) int32_t[n_stage];
    if (!c->h_pinned) { pd_set_error("out of host memory"); return fail(PD_ENOMEM); }
  } else {
    e = hipHostMalloc((void **)&c->h_pinned, sizeof(int32_t) * n_stage, 0);
    if (e != hipSuccess) { pd_set_error("hipHostMalloc failed: %s", hipGetErrorString(e)); return fail(PD_EHIP); }
  }
  // Clear everything up to the re-packed weights: caches must hold finite values
  // (masked keys are multiplied by zero), state must start at zero.
  if (no_alloc) {
    hipLaunchKernelGGL(k_fill_zero, dim3(1024), dim3(256), 0, s, (uint4 *)c->ws, need / 16);
    e = hipGetLastError();
  } else {
    e = hipMemsetAsync(c->ws, 0, need, s);
  }
  if (e != hipSuccess) { pd_set_error("clearing the workspace failed: %s", hipGetErrorString(e)); return fail(PD_EHIP); }
  int rc;
  if (c->cfg.pos_kind == 1 && (rc = launch_rope_table(c, s))) return fail(rc);
  if (c->impl == 1 && (rc = mfma_pack_weights(c, s))) return fail(rc);
  if (c->impl == 1 && (rc = mfma_fold_norms(c, s))) return fail(rc);
  if (c->arch == 1) {
    if ((rc = encdec_pack_weights(c, s))) return fail(rc);
    // the activation buffer is free at this point: it lends the few hundred ints the table set-up needs
    if ((rc = encdec_build_tables(c, (int *)c->hb, s))) return fail(rc);
  }
  e = hipStreamSynchronize(s);
  if (e != hipSuccess) { pd_set_error("pd_create: %s", hipGetErrorString(e)); return fail(PD_EHIP); }
  *out = c;
  return PD_OK;
}

// no_alloc: nothing that allocates device or pinned host memory is called (the staging buffer is
// ordinary host memory, the workspace is cleared by a kernel).
static int create_ctx(const pd_config *cfg, const pd_weights *w, void *dev_workspace, size_t bytes,
                      void *hip_stream, bool no_alloc, pd_ctx **out) {
  int rc = check_config(cfg);
  if (rc) return rc;
  PD_REQUIRE(w && out && dev_workspace, PD_EINVAL, "weights, workspace and out must not be NULL");
  PD_REQUIRE(((uintptr_t)dev_workspace & 255) == 0, PD_EINVAL, "workspace must be 256-byte aligned");
  size_t need = carve(cfg, nullptr, nullptr);
  PD_REQUIRE(bytes >= need, PD_ENOMEM, "workspace too small: %zu bytes given, %zu needed", bytes, need);
  PD_REQUIRE(w->tok_emb && w->lm_head && w->final_norm_g && w->wqkv && w->wo && w->w1 && w->w2 &&
                 w->norm1_g && w->norm2_g,
             PD_EINVAL, "a required weight pointer is NULL");
  PD_REQUIRE(cfg->pos_kind == 1 || w->pos_emb, PD_EINVAL, "pos_emb is NULL with learned positions");
  PD_REQUIRE(cfg->ffn_kind == 0 || w->w_up, PD_EINVAL, "w_up is NULL with SwiGLU");
  PD_REQUIRE(cfg->norm_kind == 1 || (w->final_norm_b && w->norm1_b && w->norm2_b), PD_EINVAL,
             "LayerNorm bias pointer is NULL");
  for (int l = 0; l < cfg->n_layer; ++l) {
    PD_REQUIRE(w->wqkv[l] && w->wo[l] && w->w1[l] && w->w2[l] && w->norm1_g[l] && w->norm2_g[l],
               PD_EINVAL, "layer %d: a required weight pointer is NULL", l);
    PD_REQUIRE(cfg->ffn_kind == 0 || w->w_up[l], PD_EINVAL, "layer %d: w_up is NULL", l);
    PD_REQUIRE(cfg->norm_kind == 1 || (w->norm1_b[l] && w->norm2_b[l]), PD_EINVAL,
               "layer %d: LayerNorm bias is NULL", l);
  }
  pd_ctx *c = new (std::nothrow) pd_ctx();
  PD_REQUIRE(c, PD_ENOMEM, "out of host memory");
  c->cfg = *cfg;
  c->ws = (char *)dev_workspace; c->ws_bytes = bytes;
  carve(cfg, c->ws, c);
  c->tok_emb = w->tok_emb; c->pos_emb = cfg->pos_kind == 0 ? w->pos_emb : nullptr;
  c->lm_head = w->lm_head; c->fng = w->final_norm_g;
  c->fnb = cfg->norm_kind == 0 ? w->final_norm_b : nullptr;
  for (int l = 0; l < cfg->n_layer; ++l) {
    LayerPtrs &lp = c->layers[l];
    lp.wqkv = w->wqkv[l]; lp.wo = w->wo[l]; lp.w1 = w->w1[l];
    lp.w_up = cfg->ffn_kind == 1 ? w->w_up[l] : nullptr; lp.w2 = w->w2[l];
    lp.n1g = w->norm1_g[l]; lp.n2g = w->norm2_g[l];
    lp.n1b = cfg->norm_kind == 0 ? w->norm1_b[l] : nullptr;
    lp.n2b = cfg->norm_kind == 0 ? w->norm2_b[l] : nullptr;
  }
  return finish_create(c, need, hip_stream, no_alloc, out);
}

extern "C" int pd_create(const pd_config *cfg, const pd_weights *w, void *dev_workspace,
                         size_t bytes, void *hip_stream, pd_ctx **out) {
  return create_ctx(cfg, w, dev_workspace, bytes, hip_stream, false, out);
}

// ---------------------------------------------------------------------------
// encoder-decoder form
// ---------------------------------------------------------------------------
static int check_encdec(const pd_encdec_config *e) {
  PD_REQUIRE(e != nullptr, PD_EINVAL, "config is NULL");
  PD_REQUIRE(e->n_enc_layer >= 1 && e->n_dec_layer >= 1 && e->d_model >= 1 && e->n_head >= 1 && e->head_dim >= 1 &&
                 e->d_ff >= 1 && e->vocab >= 1,
             PD_EINVAL, "model dimensions must be positive");
  PD_REQUIRE((int64_t)e->n_head * e->head_dim == e->d_model, PD_EINVAL,
             "n_head * head_dim (%d * %d) != d_model (%d)", e->n_head, e->head_dim, e->d_model);
  PD_REQUIRE(e->head_dim % 32 == 0 && e->head_dim <= 128 && e->d_model % 32 == 0 && e->d_ff % 32 == 0, PD_EINVAL,
             "the encoder-decoder form runs on the matrix-core kernels only: head_dim, d_model and d_ff must be "
             "multiples of 32 and head_dim <= 128");
  PD_REQUIRE(e->rel_buckets >= 4 && e->rel_buckets % 4 == 0 && e->rel_buckets <= 256, PD_EINVAL,
             "rel_buckets must be a multiple of 4 in [4, 256] (got %d)", e->rel_buckets);
  PD_REQUIRE(e->rel_max_distance > e->rel_buckets / 2 && e->rel_max_distance <= 128, PD_EINVAL,
             "rel_max_distance must be in (rel_buckets / 2, 128] (got %d)", e->rel_max_distance);
  PD_REQUIRE(e->norm_eps > 0.f, PD_EINVAL, "norm_eps must be positive");
  PD_REQUIRE(e->max_batch >= 1 && e->max_ctx >= 1 && e->max_sub >= 1 && e->max_sub_tokens >= 1, PD_EINVAL,
             "capacities (max_batch, max_ctx, max_sub, max_sub_tokens) must be >= 1");
  PD_REQUIRE(e->max_ctx <= std::min(4096, 16 * (4096 / e->n_head)), PD_EINVAL,
             "max_ctx = %d exceeds the %d input tokens one encoder launch sequence takes", e->max_ctx,
             std::min(4096, 16 * (4096 / e->n_head)));
  PD_REQUIRE(e->bos_id >= 0 && e->bos_id < e->vocab, PD_EINVAL, "bos_id out of range");
  PD_REQUIRE(e->eos_id < e->vocab, PD_EINVAL, "eos_id out of range");
  PD_REQUIRE((int64_t)e->max_sub * (e->max_sub_tokens + 1) < (1 << 24) && e->max_sub <= 65535, PD_EINVAL,
             "KV capacity too large");
  return PD_OK;
}

// the decoder stack as a pd_config of the shared code paths (ffn_kind 2: W2 relu(W1 u); pos_kind 2: no
// absolute positions) -- values pd_create does not accept from callers
static pd_config encdec_decoder_config(const pd_encdec_config *e) {
  pd_config g;
  memset(&g, 0, sizeof(g));
  g.n_layer = e->n_dec_layer; g.d_model = e->d_model; g.n_head = e->n_head; g.head_dim = e->head_dim;
  g.d_ff = e->d_ff; g.vocab = e->vocab; g.ffn_kind = 2; g.norm_kind = 1; g.pos_kind = 2; g.rope_base = 0.f;
  g.norm_eps = e->norm_eps; g.dtype = 1; g.bos_id = e->bos_id; g.eos_id = e->eos_id;
  g.max_batch = e->max_batch; g.max_ctx = e->max_ctx; g.max_sub = e->max_sub; g.max_sub_tokens = e->max_sub_tokens;
  g.max_pos = 65536;          // grid coordinates are kept in 16 bits
  g.kv_pair_layers = 0;
  return g;
}

extern "C" size_t pd_encdec_workspace_bytes(const pd_encdec_config *cfg) {
  if (check_encdec(cfg) != PD_OK) return 0;
  pd_config g = encdec_decoder_config(cfg);
  return carve(&g, nullptr, nullptr, cfg);
}

extern "C" int pd_encdec_create(const pd_encdec_config *cfg, const pd_encdec_weights *w, void *dev_workspace,
                                size_t bytes, void *hip_stream, pd_ctx **out) {
  int rc = check_encdec(cfg);
  if (rc) return rc;
  PD_REQUIRE(w && out && dev_workspace, PD_EINVAL, "weights, workspace and out must not be NULL");
  PD_REQUIRE(((uintptr_t)dev_workspace & 255) == 0, PD_EINVAL, "workspace must be 256-byte aligned");
  pd_config g = encdec_decoder_config(cfg);
  size_t need = carve(&g, nullptr, nullptr, cfg);
  PD_REQUIRE(bytes >= need, PD_ENOMEM, "workspace too small: %zu bytes given, %zu needed", bytes, need);
  PD_REQUIRE(w->tok_emb && w->lm_head && w->enc_rel_bias && w->dec_rel_bias && w->enc_final_norm_g &&
                 w->dec_final_norm_g && w->enc_wqkv && w->enc_wo && w->enc_w1 && w->enc_w2 && w->enc_norm1_g &&
                 w->enc_norm2_g && w->dec_wqkv && w->dec_wo && w->dec_w1 && w->dec_w2 && w->cross_wq &&
                 w->cross_wkv && w->cross_wo && w->dec_norm1_g && w->dec_norm3_g && w->dec_norm2_g,
             PD_EINVAL, "a required weight pointer is NULL");
  for (int l = 0; l < cfg->n_enc_layer; ++l)
    PD_REQUIRE(w->enc_wqkv[l] && w->enc_wo[l] && w->enc_w1[l] && w->enc_w2[l] && w->enc_norm1_g[l] && w->enc_norm2_g[l],
               PD_EINVAL, "encoder layer %d: a required weight pointer is NULL", l);
  for (int l = 0; l < cfg->n_dec_layer; ++l)
    PD_REQUIRE(w->dec_wqkv[l] && w->dec_wo[l] && w->dec_w1[l] && w->dec_w2[l] && w->cross_wq[l] && w->cross_wkv[l] &&
                   w->cross_wo[l] && w->dec_norm1_g[l] && w->dec_norm3_g[l] && w->dec_norm2_g[l],
               PD_EINVAL, "decoder layer %d: a required weight pointer is NULL", l);
  pd_ctx *c = new (std::nothrow) pd_ctx();
  PD_REQUIRE(c, PD_ENOMEM, "out of host memory");
  c->cfg = g;
  c->ws = (char *)dev_workspace; c->ws_bytes = bytes;
  carve(&g, c->ws, c, cfg);
  c->tok_emb = w->tok_emb; c->pos_emb = nullptr; c->lm_head = w->lm_head;
  c->fng = w->dec_final_norm_g; c->fnb = nullptr;
  c->ed.enc_fng = w->enc_final_norm_g; c->ed.enc_rel_bias = w->enc_rel_bias; c->ed.dec_rel_bias = w->dec_rel_bias;
  for (int l = 0; l < cfg->n_enc_layer; ++l) {
    LayerPtrs &lp = c->ed.enc[l];
    lp.wqkv = w->enc_wqkv[l]; lp.wo = w->enc_wo[l]; lp.w1 = w->enc_w1[l]; lp.w2 = w->enc_w2[l];
    lp.n1g = w->enc_norm1_g[l]; lp.n2g = w->enc_norm2_g[l];
  }
  for (int l = 0; l < cfg->n_dec_layer; ++l) {
    LayerPtrs &lp = c->layers[l];
    lp.wqkv = w->dec_wqkv[l]; lp.wo = w->dec_wo[l]; lp.w1 = w->dec_w1[l]; lp.w2 = w->dec_w2[l];
    lp.cq = w->cross_wq[l]; lp.ckv = w->cross_wkv[l]; lp.co = w->cross_wo[l];
    lp.n1g = w->dec_norm1_g[l]; lp.n3g = w->dec_norm3_g[l]; lp.n2g = w->dec_norm2_g[l];
  }
  return finish_create(c, need, hip_stream, false, out);
}

extern "C" int pd_destroy(pd_ctx *c) {
  if (!c) return PD_OK;
  if (c->graph_exec) (void)hipGraphExecDestroy(c->graph_exec);
  for (hipEvent_t ev : c->ev_pool) (void)hipEventDestroy(ev);
  if (c->h_pinned) {
    if (c->stage_pinned) (void)hipHostFree(c->h_pinned);
    else delete[] c->h_pinned;
  }
  delete c;
  return PD_OK;
}

// ---------------------------------------------------------------------------
// options / instrumentation
// ---------------------------------------------------------------------------
// Whether the context pass carries activations as bf16 pairs (high + low part, as the decode step does;
// the default) or as single bf16 values (PD_OPT_CONTEXT_SPLIT_ACT 0), which halves the multiplies of its
// projections.  Measured over whole runs against the oracle: width 1024 (cfg3) 4.2e-4 -> 2.6e-3 of logit
// error and 0.017 -> 0.014 s, width 2048 (cfg4) 4.8e-4 -> 3.4e-3 and 0.047 -> 0.033 s, every token with a
// margin above 0.05 still equal; width 4096 with 32 layers (cfg5) 9.3e-4 -> 8.6e-2, and a small model with
// a vocabulary projection of 15 times the usual scale 2.1e-2: outside the 2e-2 tolerance, which is why
// the library does not choose single values by itself.
static bool context_pairs(const pd_ctx *c) {
  if (c->impl != 1 || c->arch == 1) return c->opt_split != 0;
  return c->opt_split && c->opt_ctx_split;
}

static void drop_graph(pd_ctx *c) {
  if (c->graph_exec) (void)hipGraphExecDestroy(c->graph_exec);
  c->graph_exec = nullptr; c->graph_ready = false;
}

extern "C" int pd_set_option(pd_ctx *c, int key, int value) {
  PD_REQUIRE(c, PD_EINVAL, "ctx is NULL");
  switch (key) {
    case PD_OPT_ATTN_SPLITS:
      PD_REQUIRE(value >= 0 && value <= 256, PD_EINVAL, "attention splits must be in [0, 256]");
      c->opt_splits = value; drop_graph(c); return PD_OK;
    case PD_OPT_USE_GRAPH:
      c->opt_graph = value ? 1 : 0; drop_graph(c); return PD_OK;
    case PD_OPT_SPLIT_ACT:
      c->opt_split = value ? 1 : 0; drop_graph(c); return PD_OK;
    case PD_OPT_PREFILL_CHUNK:
      PD_REQUIRE(value >= 0, PD_EINVAL, "prefill chunk must be >= 0");
      c->opt_chunk = value == 0 ? 0 : std::min((value + 15) / 16 * 16, c->prefill_chunk_cap);
      return PD_OK;
    case PD_OPT_CONTEXT_SPLIT_ACT:
      c->opt_ctx_split = value ? 1 : 0; return PD_OK;
    case PD_OPT_STREAM_LOADS:
      c->stream_loads = value ? 1 : 0; drop_graph(c); return PD_OK;
    case PD_OPT_CONTEXT_ATTN:
      c->opt_ctx_attn = value < 0 ? 0 : value > 2 ? 2 : value; return PD_OK;
    case PD_OPT_FUSE_NORM:
      c->opt_fuse_norm = value < 0 ? 0 : value > 2 ? 2 : value; drop_graph(c); return PD_OK;
    case PD_OPT_PROFILE:
      c->opt_profile = (value == 2 || value == 3) ? value : (value ? 1 : 0); drop_graph(c); c->ev_used = 0; return PD_OK;
    default:
      pd_set_error("unknown option key %d", key);
      return PD_EINVAL;
  }
}

extern "C" int pd_profile_read(pd_ctx *c, double *attn_avg_us, int32_t *attn_launches) {
  PD_REQUIRE(c && attn_avg_us && attn_launches, PD_EINVAL, "NULL argument");
  size_t pairs = c->ev_used / 2;
  double total = 0.0;
  if (pairs) PD_CHECK_HIP(hipEventSynchronize(c->ev_pool[c->ev_used - 1]));
  for (size_t i = 0; i < pairs; ++i) {
    float ms = 0.f;
    PD_CHECK_HIP(hipEventElapsedTime(&ms, c->ev_pool[2 * i], c->ev_pool[2 * i + 1]));
    total += ms;
  }
  *attn_avg_us = pairs ? total * 1000.0 / (double)pairs : 0.0;
  *attn_launches = (int32_t)pairs;
  c->ev_used = 0;
  return PD_OK;
}

extern "C" int pd_get_info(pd_ctx *c, int key, void *hip_stream, int64_t *value) {
  PD_REQUIRE(c && value, PD_EINVAL, "NULL argument");
  switch (key) {
    case PD_INFO_KERNEL_PATH: *value = c->impl; return PD_OK;
    case PD_INFO_KV_PAIR_LAYERS: *value = c->pair_layers; return PD_OK;
    case PD_INFO_CONTEXT_PAIRS: *value = context_pairs(c) ? 1 : 0; return PD_OK;
    case PD_INFO_STREAM_LOADS: *value = c->stream_loads; return PD_OK;
    case PD_INFO_KV_SATURATED: {
      hipStream_t s = (hipStream_t)hip_stream;
      PD_CHECK_HIP(hipStreamSynchronize(s));        // the staging buffer may be in flight
      int32_t *h = c->h_pinned;
      PD_CHECK_HIP(hipMemcpyAsync(h, c->kv_sat, sizeof(int32_t), hipMemcpyDeviceToHost, s));
      PD_CHECK_HIP(hipStreamSynchronize(s));
      *value = *h;
      return PD_OK;
    }
    default:
      pd_set_error("unknown info key %d", key);
      return PD_EINVAL;
  }
}

// ---------------------------------------------------------------------------
// prefill
// ---------------------------------------------------------------------------
static int run_layers(pd_ctx *c, int R, int A, int nreq, int req0, int kv_override,
                      hipStream_t s) {
  int rc;
  // fp32 path: embedding kernel; matrix-core path: the first norm kernel gathers the rows itself
  if (c->impl == 1) c->embed_pending = true;
  else if ((rc = launch_embed(c, R, s))) return rc;
  c->pend_parts = 0;
  c->norm_fused = false;
  for (int l = 0; l < c->cfg.n_layer; ++l) {
    rc = c->arch == 1 ? encdec_decoder_layer(c, l, R, s)
         : c->impl == 1 ? mfma_layer(c, l, R, A, nreq, req0, kv_override, s)
                        : simple_layer(c, l, R, A, nreq, req0, kv_override, s);
    if (rc) return rc;
  }
  return PD_OK;
}

extern "C" int pd_prefill_context(pd_ctx *c, const int32_t *ctx_tokens, int B, int L, int n_sub,
                                  int delta_t, int max_sub_tokens, int time_max, void *hip_stream) {
  PD_REQUIRE(c && ctx_tokens, PD_EINVAL, "ctx or ctx_tokens is NULL");
  const pd_config &g = c->cfg;
  PD_REQUIRE(B >= 1 && B <= g.max_batch, PD_EINVAL, "B = %d out of range [1, %d]", B, g.max_batch);
  PD_REQUIRE(L >= 1 && L <= g.max_ctx, PD_EINVAL, "L = %d out of range [1, %d]", L, g.max_ctx);
  PD_REQUIRE(n_sub >= 1 && n_sub <= g.max_sub, PD_EINVAL, "n_sub = %d out of range [1, %d]", n_sub, g.max_sub);
  PD_REQUIRE(delta_t >= 1, PD_EINVAL, "delta_t must be >= 1 (got %d)", delta_t);
  PD_REQUIRE(max_sub_tokens >= 1 && max_sub_tokens <= g.max_sub_tokens, PD_EINVAL,
             "max_sub_tokens = %d out of range [1, %d]", max_sub_tokens, g.max_sub_tokens);
  PD_REQUIRE(time_max >= 0, PD_EINVAL, "time_max must be >= 0");
  int64_t t_last = std::min<int64_t>(time_max, (int64_t)(n_sub - 1) * delta_t + max_sub_tokens + 1);
  // encoder-decoder form: a position index is a grid coordinate and does not count the input
  int64_t p_max = (int64_t)(c->arch == 1 ? 0 : L) + std::max<int64_t>(t_last, 1) + n_sub - 2;
  PD_REQUIRE(p_max < g.max_pos, PD_EINVAL,
             "largest position index %lld does not fit max_pos = %d", (long long)p_max, g.max_pos);
  for (int64_t i = 0; i < (int64_t)B * L; ++i)
    PD_REQUIRE(ctx_tokens[i] >= 0 && ctx_tokens[i] < g.vocab, PD_EINVAL,
               "context token %lld = %d out of range [0, %d)", (long long)i, ctx_tokens[i], g.vocab);
  hipStream_t s = (hipStream_t)hip_stream;
  c->prefilled = false;
  drop_graph(c);
  c->B = B; c->L = c->arch == 1 ? 0 : L; c->Lx = c->arch == 1 ? L : 0; c->S = n_sub; c->dt = delta_t; c->M = max_sub_tokens; c->time_max = time_max;
  c->A = std::min(n_sub, max_sub_tokens / delta_t + 1);
  c->R = B * c->A;
  PD_REQUIRE(c->A <= 1024, PD_EINVAL, "%d rows per request exceed the 1024 one step supports", c->A);
  PD_CHECK_HIP(hipMemcpyAsync(c->ctx_tok, ctx_tokens, sizeof(int32_t) * (size_t)B * L,
                              hipMemcpyHostToDevice, s));
  PD_CHECK_HIP(hipStreamSynchronize(s));
  int rc;
  if ((rc = launch_reset_state(c, s))) return rc;
  for (int b = 0; b < B && c->arch == 1; ++b)
    if ((rc = encdec_encode(c, b, s))) return rc;
  // the context pass may carry its activations as single bf16 values (see context_pairs)
  const int split_decode = c->opt_split;
  if (!context_pairs(c)) c->opt_split = 0;
  for (int b = 0; b < B && c->arch == 0 && !rc; ++b) {
    const int chunk = c->opt_chunk > 0 ? c->opt_chunk : c->prefill_chunk;
    for (int p0 = 0; p0 < L && !rc; p0 += chunk) {
      int n = std::min(chunk, L - p0);
      if ((rc = launch_prefill_rows(c, b, p0, n, s, c->L, 0, b))) break;
      rc = run_layers(c, n, n, 1, b, p0 + n, s);
    }
  }
  c->opt_split = split_decode;
  if (rc) return rc;
  // leave the row tables empty so that a stray head/commit sees no rows
  if ((rc = launch_reset_state(c, s))) return rc;
  c->prefilled = true;
  c->host_steps = 0;
  return PD_OK;
}

extern "C" int pd_reset_decode(pd_ctx *c, void *hip_stream) {
  PD_REQUIRE(c, PD_EINVAL, "ctx is NULL");
  PD_REQUIRE(c->prefilled, PD_ESTATE, "pd_reset_decode before pd_prefill_context");
  c->host_steps = 0;
  return launch_reset_state(c, (hipStream_t)hip_stream);
}

// ---------------------------------------------------------------------------
// decode step
// ---------------------------------------------------------------------------
// Rows of request 0 that step t can have at most: subsequence i has a row from the step that opens
// it to the step after its last token, (i-1) dt < t <= (i-1) dt + M + 1 (an earlier <eos> only takes
// rows away, and rows are numbered without gaps).
static int rows_bound(const pd_ctx *c, int64_t t) {
  int n = 0;
  for (int i = 0; i < c->S; ++i) {
    int64_t first = (int64_t)i * c->dt + 1;
    if (t >= first && t <= first + c->M) ++n;
  }
  return std::min(n, c->A);
}

static int enqueue_step(pd_ctx *c, float *out_logits, hipStream_t s) {
  int rc;
  if ((rc = launch_tick(c, s))) return rc;
  // Row indices in use this step: b * A + a.  When they all stay below 8 the matrix-core path keeps
  // every activation as a packed pair (half the fragments and multiplies in the projections).  A
  // captured graph is replayed for every step, so it keeps the general layout.
  int R = c->R;
  if (c->impl == 1 && c->opt_split && !c->opt_graph) {
    int r_used = c->B == 1 ? rows_bound(c, (int64_t)c->host_steps + 1) : c->R;
    if (r_used <= 8) { c->packed = true; R = std::min(R, std::max(r_used, 1)); }
  }
  rc = run_layers(c, R, c->A, c->B, 0, -1, s);
  if (!rc) rc = c->impl == 1 ? mfma_head(c, R, out_logits != nullptr, s) : simple_head(c, R, s);
  c->packed = false;
  if (rc) return rc;
  return launch_commit(c, out_logits, s);
}

// One step, optionally replayed from a captured graph (only without logits output
// and without profiling events, which cannot be recorded into a graph here).
static int run_step(pd_ctx *c, float *out_logits, hipStream_t s) {
  if (!c->opt_graph || out_logits || c->opt_profile) return enqueue_step(c, out_logits, s);
  if (!c->graph_ready) {
    hipGraph_t graph = nullptr;
    PD_CHECK_HIP(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
    int rc = enqueue_step(c, nullptr, s);
    hipError_t e = hipStreamEndCapture(s, &graph);
    if (rc) { if (graph) (void)hipGraphDestroy(graph); return rc; }
    PD_CHECK_HIP(e);
    e = hipGraphInstantiate(&c->graph_exec, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    PD_CHECK_HIP(e);
    c->graph_ready = true;
  }
  PD_CHECK_HIP(hipGraphLaunch(c->graph_exec, s));
  return PD_OK;
}

extern "C" int pd_decode_step(pd_ctx *c, const int32_t *force_tokens, int32_t *out_tokens,
                              float *out_logits, int32_t *out_all_done, void *hip_stream) {
  PD_REQUIRE(c, PD_EINVAL, "ctx is NULL");
  PD_REQUIRE(c->prefilled, PD_ESTATE, "pd_decode_step before pd_prefill_context");
  hipStream_t s = (hipStream_t)hip_stream;
  size_t bs = (size_t)c->B * c->S;
  if (force_tokens) {
    for (size_t i = 0; i < bs; ++i)
      PD_REQUIRE(force_tokens[i] < c->cfg.vocab, PD_EINVAL, "force token %zu = %d out of range", i,
                 force_tokens[i]);
    // the staging buffer may still be in flight from the previous call
    PD_CHECK_HIP(hipStreamSynchronize(s));
    memcpy(c->h_pinned, force_tokens, bs * sizeof(int32_t));
    PD_CHECK_HIP(hipMemcpyAsync(c->sch.force, c->h_pinned, bs * sizeof(int32_t),
                                hipMemcpyHostToDevice, s));
  }
  int rc = run_step(c, out_logits, s);
  if (rc) return rc;
  c->host_steps++;
  if (out_tokens || out_all_done) {
    int32_t *h_tok = c->h_pinned + bs, *h_done = c->h_pinned + 2 * bs;
    PD_CHECK_HIP(hipMemcpyAsync(h_tok, c->sch.step_tok, bs * sizeof(int32_t), hipMemcpyDeviceToHost, s));
    PD_CHECK_HIP(hipMemcpyAsync(h_done, c->sch.all_done, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    PD_CHECK_HIP(hipStreamSynchronize(s));
    if (out_tokens) memcpy(out_tokens, h_tok, bs * sizeof(int32_t));
    if (out_all_done) *out_all_done = (*h_done >= c->B) ? 1 : 0;
  }
  return PD_OK;
}

extern "C" int pd_decode_steps(pd_ctx *c, int n_steps, void *hip_stream) {
  PD_REQUIRE(c, PD_EINVAL, "ctx is NULL");
  PD_REQUIRE(c->prefilled, PD_ESTATE, "pd_decode_steps before pd_prefill_context");
  PD_REQUIRE(n_steps >= 0, PD_EINVAL, "n_steps must be >= 0");
  for (int i = 0; i < n_steps; ++i) {
    int rc = run_step(c, nullptr, (hipStream_t)hip_stream);
    if (rc) return rc;
    c->host_steps++;
  }
  return PD_OK;
}

// ---------------------------------------------------------------------------
// teacher-forced forward (Section 3.3)
// ---------------------------------------------------------------------------
extern "C" int pd_teacher_forced(pd_ctx *c, const int32_t *target, int max_len, float *out_logits, int rows_cap,
                                 float *out_row_nll, double *out_loss, int32_t *out_rows, void *hip_stream) {
  PD_REQUIRE(c && target && out_logits && out_loss, PD_EINVAL, "ctx, target, out_logits or out_loss is NULL");
  PD_REQUIRE(c->prefilled, PD_ESTATE, "pd_teacher_forced before pd_prefill_context");
  PD_REQUIRE(c->impl == 1, PD_EINVAL,
             "the teacher-forced forward runs on the matrix-core kernels (dtype 1, head_dim, d_model, d_ff multiples "
             "of 32)");
  const pd_config &g = c->cfg;
  const int B = c->B, S = c->S, L = c->L;
  PD_REQUIRE(max_len >= 1 && max_len <= g.max_sub_tokens + 2, PD_EINVAL, "max_len = %d out of range [1, %d]", max_len,
             g.max_sub_tokens + 2);
  std::vector<int> rows(B, 0);
  for (int b = 0; b < B; ++b) {
    bool ended = false;
    for (int i = 0; i < S; ++i) {
      const int32_t *t = target + ((size_t)b * S + i) * max_len;
      int n = 0;
      while (n < max_len && t[n] >= 0) ++n;
      for (int j = 0; j < max_len; ++j) {
        PD_REQUIRE(t[j] < g.vocab, PD_EINVAL, "request %d subsequence %d token %d = %d out of range", b, i, j, t[j]);
        PD_REQUIRE(j < n || t[j] < 0, PD_EINVAL, "request %d subsequence %d: token after the padding", b, i);
      }
      PD_REQUIRE(!(ended && n > 0), PD_EINVAL, "request %d: subsequence %d follows an empty one", b, i);
      ended = ended || n == 0;
      if (n > 0) {
        int64_t coord = (int64_t)i * c->dt + (n - 1) + i;
        PD_REQUIRE(coord < 65536 && (g.pos_kind == 1 ? coord + L < (int64_t)c->rope_rows : coord + L < g.max_pos),
                   PD_EINVAL, "request %d subsequence %d: position index %lld out of range", b, i, (long long)(coord + L));
      }
      rows[b] += n;
    }
    PD_REQUIRE(rows[b] >= 1, PD_EINVAL, "request %d has an empty target", b);
    PD_REQUIRE(rows[b] <= c->gen_cap && rows[b] <= c->R_cap && rows[b] <= rows_cap, PD_EINVAL,
               "request %d: %d target tokens exceed the capacity (%d cache slots, %d rows per pass, %d rows of out_logits)",
               b, rows[b], c->gen_cap, c->R_cap, rows_cap);
  }
  hipStream_t s = (hipStream_t)hip_stream;
  drop_graph(c);
  PD_CHECK_HIP(hipMemcpyAsync(c->tf_target, target, sizeof(int32_t) * (size_t)B * S * max_len, hipMemcpyHostToDevice, s));
  PD_CHECK_HIP(hipStreamSynchronize(s));
  AttnMode am;
  memset(&am, 0, sizeof(am));
  am.L = L; am.scale = 1.f / sqrtf((float)g.head_dim);
  am.bias = c->bias0; am.bias_len = 1; am.bias_off = 0;
  am.coord = c->gen_coord; am.coord_stride = c->gen_stride; am.coord_req_stride = c->gen_stride;
  am.coord_off = L & ~7; am.pos0 = L;
  int rc;
  std::vector<float> nll_host;
  for (int b = 0; b < B; ++b) {
    const int n = rows[b];
    if ((rc = launch_teacher_rows(c, c->tf_target, b, max_len, s))) return rc;
    c->packed = false; c->embed_pending = true; c->pend_parts = 0; c->norm_fused = false;
    for (int l = 0; l < g.n_layer; ++l)
      if ((rc = c->arch == 1 ? encdec_decoder_layer(c, l, n, s, n, 1, b, n) : mfma_layer(c, l, n, n, 1, b, L + n, s, &am)))
        return rc;
    float *lg = out_logits + (size_t)b * rows_cap * g.vocab;
    if ((rc = mfma_head(c, n, true, s, lg))) return rc;
    if ((rc = launch_row_nll(c, lg, n, c->loss + b, s))) return rc;
    if (out_row_nll) {
      PD_CHECK_HIP(hipMemcpyAsync(out_row_nll + (size_t)b * rows_cap, c->nll, sizeof(float) * n, hipMemcpyDeviceToHost, s));
      PD_CHECK_HIP(hipStreamSynchronize(s));        // c->nll is reused by the next request
    }
  }
  PD_CHECK_HIP(hipMemcpyAsync(out_loss, c->loss, sizeof(double) * B, hipMemcpyDeviceToHost, s));
  // the generated side of the caches and the schedule state were used as scratch: back to t = 0
  c->host_steps = 0;
  if ((rc = launch_reset_state(c, s))) return rc;
  PD_CHECK_HIP(hipStreamSynchronize(s));
  if (out_rows) for (int b = 0; b < B; ++b) out_rows[b] = rows[b];
  return PD_OK;
}

// ---------------------------------------------------------------------------
// generate: Algorithm 1 as a whole
// ---------------------------------------------------------------------------
extern "C" int pd_generate(pd_ctx *c, const int32_t *ctx_tokens, int B, int L, int n_sub,
                           int delta_t, int max_sub_tokens, int time_max, int32_t *out_tokens,
                           int32_t *out_lens, int32_t *out_steps, void *hip_stream) {
  PD_REQUIRE(out_tokens && out_lens && out_steps, PD_EINVAL, "output pointer is NULL");
  int rc = pd_prefill_context(c, ctx_tokens, B, L, n_sub, delta_t, max_sub_tokens, time_max, hip_stream);
  if (rc) return rc;
  hipStream_t s = (hipStream_t)hip_stream;
  int S = n_sub, M = max_sub_tokens;
  // Upper bound on the iterations: the loop cannot outlast time_max, nor the step
  // after which every subsequence has reached its length limit.
  int64_t bound = std::min<int64_t>(time_max, (int64_t)(S - 1) * delta_t + M);
  int32_t *h_done = c->h_pinned + 2 * (size_t)B * S;
  int64_t t = 0;
  bool finished = bound == 0;
  while (!finished) {
    // Without <eos> the length of the run is known; otherwise look at the
    // termination counter every few steps (steps after termination are no-ops).
    int burst = c->cfg.eos_id < 0 ? (int)std::min<int64_t>(bound - t, 64) : (int)std::min<int64_t>(bound - t, 8);
    if ((rc = pd_decode_steps(c, burst, s))) return rc;
    t += burst;
    PD_CHECK_HIP(hipMemcpyAsync(h_done, c->sch.all_done, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    PD_CHECK_HIP(hipStreamSynchronize(s));
    finished = (*h_done >= B) || t >= bound;
  }
  if (bound == 0) {            // time_max == 0: one tick marks the requests terminated
    if ((rc = launch_tick(c, s))) return rc;
  }
  std::vector<int32_t> grid((size_t)B * S * (M + 1)), ntok((size_t)B * S), fin((size_t)B * S), steps(B);
  PD_CHECK_HIP(hipMemcpyAsync(grid.data(), c->sch.grid, grid.size() * 4, hipMemcpyDeviceToHost, s));
  PD_CHECK_HIP(hipMemcpyAsync(ntok.data(), c->sch.n_tok, ntok.size() * 4, hipMemcpyDeviceToHost, s));
  PD_CHECK_HIP(hipMemcpyAsync(fin.data(), c->sch.fin, fin.size() * 4, hipMemcpyDeviceToHost, s));
  PD_CHECK_HIP(hipMemcpyAsync(steps.data(), c->sch.steps, steps.size() * 4, hipMemcpyDeviceToHost, s));
  PD_CHECK_HIP(hipStreamSynchronize(s));
  for (int b = 0; b < B; ++b) {
    out_steps[b] = steps[b];
    for (int i = 0; i < S; ++i) {
      size_t bi = (size_t)b * S + i;
      int n = ntok[bi] > 0 ? ntok[bi] - 1 - (fin[bi] == 1 ? 1 : 0) : 0;   // drop <bos> and <eos>
      out_lens[bi] = n;
      for (int j = 0; j < M; ++j)
        out_tokens[bi * M + j] = j < n ? grid[bi * (M + 1) + 1 + j] : -1;
    }
  }
  return PD_OK;
}

// ---------------------------------------------------------------------------
// pd_generate for callers that cannot allocate: the workspace is a device array of this library
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[PD_STATIC_WORKSPACE_BYTES];

// `scratch` is a host-side stand-in in host code; the array's device address is asked for once per
// device (every GPU holds its own copy) and only that address is handed to kernels and copies.
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[64] = {};

static int scratch_of_current_device(void **ptr) {
  int dev = -1;
  PD_CHECK_HIP(hipGetDevice(&dev));
  PD_REQUIRE(dev >= 0 && dev < 64, PD_EINVAL, "device index %d outside [0, 64)", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    PD_CHECK_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    PD_REQUIRE(p != nullptr, PD_EHIP, "hipGetSymbolAddress returned no address for the static workspace");
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return PD_OK;
}

extern "C" int pd_generate_static(const pd_config *cfg, const pd_weights *w, const int32_t *ctx_tokens, int B,
                                  int L, int n_sub, int delta_t, int max_sub_tokens, int time_max,
                                  int32_t *out_tokens, int32_t *out_lens, int32_t *out_steps,
                                  void *hip_stream) {
  PD_REQUIRE(out_tokens && out_lens && out_steps, PD_EINVAL, "output pointer is NULL");
  int rc = check_config(cfg);
  if (rc) return rc;
  const size_t need = carve(cfg, nullptr, nullptr);
  PD_REQUIRE(need <= (size_t)PD_STATIC_WORKSPACE_BYTES, PD_ENOMEM,
             "this configuration needs %zu bytes of workspace; the static workspace of pd_generate_static "
             "holds %zu (use pd_create with a workspace of the caller's)",
             need, (size_t)PD_STATIC_WORKSPACE_BYTES);
  void *ws = nullptr;
  if ((rc = scratch_of_current_device(&ws))) return rc;
  pd_ctx *c = nullptr;
  // the context lives for this call only; create_ctx clears the part of the array it uses (the
  // array keeps whatever the previous call left) and re-packs the weights into it
  if ((rc = create_ctx(cfg, w, ws, (size_t)PD_STATIC_WORKSPACE_BYTES, hip_stream, true, &c))) return rc;
  rc = pd_generate(c, ctx_tokens, B, L, n_sub, delta_t, max_sub_tokens, time_max, out_tokens, out_lens,
                   out_steps, hip_stream);
  (void)pd_destroy(c);
  return rc;
}

// ---------------------------------------------------------------------------
// plain streaming read: the bandwidth a kernel that does nothing but read can reach
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_stream_read(const uint4 *p, size_t n, unsigned *sink) {
  size_t base = (size_t)blockIdx.x * 2048 + threadIdx.x;
  uint4 v[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    size_t j = base + u * 256;
    v[u] = p[j < n ? j : n - 1];
  }
  unsigned acc = 0;
#pragma unroll
  for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  if (acc == 0x9e3779b9u) *sink = acc;       // keeps the loads alive; practically never taken
}

extern "C" int pd_measure_read_bandwidth(const void *dev_buf, size_t buf_bytes, size_t chunk_bytes, int iters,
                                         void *hip_stream, double *gb_per_s) {
  PD_REQUIRE(dev_buf && gb_per_s && iters >= 1, PD_EINVAL, "NULL buffer / result or iters < 1");
  PD_REQUIRE(chunk_bytes >= 4096 && chunk_bytes % 16 == 0 && chunk_bytes + 256 <= buf_bytes, PD_EINVAL,
             "chunk_bytes must be a multiple of 16, at least 4096 and smaller than the buffer");
  PD_REQUIRE(((uintptr_t)dev_buf & 15) == 0, PD_EINVAL, "buffer must be 16-byte aligned");
  hipStream_t s = (hipStream_t)hip_stream;
  hipEvent_t e0, e1;
  PD_CHECK_HIP(hipEventCreate(&e0));
  PD_CHECK_HIP(hipEventCreate(&e1));
  size_t n16 = chunk_bytes / 16, slots = (buf_bytes - 256) / chunk_bytes;
  unsigned *sink = (unsigned *)((char *)dev_buf + (buf_bytes - 256) / 16 * 16);   // last bytes: never read
  unsigned nb = (unsigned)((n16 + 2047) / 2048);
  auto run = [&](int n) {
    for (int i = 0; i < n; ++i)      // a different chunk every launch, so that no cache serves it
      hipLaunchKernelGGL(k_stream_read, dim3(nb), dim3(256), 0, s,
                         (const uint4 *)((const char *)dev_buf + (size_t)(i % slots) * chunk_bytes), n16, sink);
  };
  run(3);
  PD_CHECK_HIP(hipEventRecord(e0, s));
  run(iters);
  PD_CHECK_HIP(hipEventRecord(e1, s));
  PD_CHECK_HIP(hipEventSynchronize(e1));
  float ms = 0.f;
  PD_CHECK_HIP(hipEventElapsedTime(&ms, e0, e1));
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  PD_CHECK_HIP(hipGetLastError());
  *gb_per_s = (double)chunk_bytes * iters / (ms * 1e-3) * 1e-9;
  return PD_OK;
}
