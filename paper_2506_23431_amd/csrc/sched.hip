// Schedule and glue kernels: the integer bookkeeping of Algorithm 1 kept on the
// device (so that a decode step never waits for the host), embedding gather,
// rotary table.
#include "pd_internal.h"

// ---------------------------------------------------------------------------
// reset: t = 0, no subsequences, nothing generated (Algorithm 1, lines 1-2)
// ---------------------------------------------------------------------------
__global__ void k_reset_state(SchedState st, RowTables rt, int B, int S, int L, int R_cap) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < B) {
    st.step[i] = 0; st.k_open[i] = 0; st.done[i] = 0; st.steps[i] = 0;
    st.n_gen[i] = 0; st.kv_len[i] = L; st.n_rows[i] = 0;
  }
  if (i < B * S) {
    st.n_tok[i] = 0; st.n_fed[i] = 0; st.fin[i] = 0; st.step_tok[i] = -1; st.force[i] = -1;
    st.row_of[i] = -1;
  }
  if (i < R_cap) { rt.flags[i] = 0; rt.qinfo[i] = make_int4(0, -1, 0, 0); rt.kvinfo[i] = make_int4(0, 0, 0, 0); }
  if (i == 0) *st.all_done = 0;
}

int launch_reset_state(pd_ctx *c, hipStream_t s) {
  int n = c->B * c->S;
  if (n < c->R_cap) n = c->R_cap;
  hipLaunchKernelGGL(k_reset_state, dim3((n + 255) / 256), dim3(256), 0, s, c->sch, c->rows, c->B,
                     c->S, c->L, c->R_cap);
  PD_CHECK_HIP(hipGetLastError());
  return PD_OK;
}

// ---------------------------------------------------------------------------
// tick: Algorithm 1 lines 5-7 plus the row list of this time-step.
// One block per request; the work is a few dozen integers, done by one thread.
// A subsequence has a row when it holds a token that was not fed yet: its newest
// token (coordinate tau = t).  A subsequence that finished in the previous step is
// fed once more so that its last token enters the KV cache; that row selects no token.
// ---------------------------------------------------------------------------
__global__ void k_tick(SchedState st, RowTables rt, int S, int dt, int M, int L, int A,
                       int time_max, int bos, int gen_cap, int gen_stride) {
  int b = blockIdx.x;
  if (threadIdx.x != 0) return;
  for (int a = 0; a < A; ++a) { rt.flags[b * A + a] = 0; rt.qinfo[b * A + a] = make_int4(0, -1, 0, b); rt.kvinfo[b * A + a] = make_int4(0, b, 0, 0); }
  for (int i = 0; i < S; ++i) { st.row_of[b * S + i] = -1; st.step_tok[b * S + i] = -1; }
  st.n_rows[b] = 0;
  if (st.done[b]) return;
  int t = st.step[b] + 1;
  if (t > time_max) {            // only reachable with time_max == 0
    st.done[b] = 1;
    atomicAdd(st.all_done, 1);
    return;
  }
  st.step[b] = t;
  int k = st.k_open[b];
  if ((t - 1) % dt == 0 && k < S) {
    st.grid[(size_t)(b * S + k) * (M + 1)] = bos;
    st.n_tok[b * S + k] = 1; st.n_fed[b * S + k] = 0; st.fin[b * S + k] = 0;
    ++k;
    st.k_open[b] = k;
  }
  int a = 0, ng = st.n_gen[b];
  for (int i = 0; i < k; ++i) {
    int nt = st.n_tok[b * S + i];
    if (nt > st.n_fed[b * S + i] && a < A && ng + a < gen_cap) {
      int r = b * A + a;
      rt.req[r] = b; rt.sub[r] = i + 1;
      rt.tok[r] = st.grid[(size_t)(b * S + i) * (M + 1) + nt - 1];
      rt.pos[r] = L + (t - 1) + i;
      rt.slot[r] = L + ng + a;
      rt.lim[r] = L;
      rt.flags[r] = ROW_VALID | (st.fin[b * S + i] ? 0 : ROW_PRODUCE);
      rt.qinfo[r] = make_int4(rt.flags[r], i + 1, L, b);
      rt.kvinfo[r] = make_int4(rt.flags[r], b, L + ng + a, L + (t - 1) + i);
      st.gen_sub[(size_t)b * gen_stride + (L & 7) + ng + a] = (uint16_t)(i + 1);
      st.n_fed[b * S + i] = nt;
      st.row_of[b * S + i] = r;
      ++a;
    }
  }
  st.n_gen[b] = ng + a; st.kv_len[b] = L + ng + a; st.n_rows[b] = a;
}

int launch_tick(pd_ctx *c, hipStream_t s) {
  hipLaunchKernelGGL(k_tick, dim3(c->B), dim3(64), 0, s, c->sch, c->rows, c->S, c->dt, c->M, c->L,
                     c->A, c->time_max, c->cfg.bos_id, c->gen_cap, c->gen_stride);
  PD_CHECK_HIP(hipGetLastError());
  return PD_OK;
}

// ---------------------------------------------------------------------------
// prefill rows: context tokens p0 .. p0+n-1 of request b as rows 0 .. n-1.
// Row for position p sees the keys 0..p (causal prefix), nothing generated.
// ---------------------------------------------------------------------------
__global__ void k_prefill_rows(RowTables rt, const int32_t *ctx_tok, int b, int L, int p0, int n,
                               int R_cap) {
  int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= R_cap) return;
  if (r < n) {
    int p = p0 + r;
    rt.req[r] = b; rt.sub[r] = 0; rt.tok[r] = ctx_tok[(size_t)b * L + p]; rt.pos[r] = p;
    rt.slot[r] = p; rt.lim[r] = p + 1; rt.flags[r] = ROW_VALID;
    rt.qinfo[r] = make_int4(ROW_VALID, 0, p + 1, b);
    rt.kvinfo[r] = make_int4(ROW_VALID, b, p, p);
  } else {
    rt.flags[r] = 0;
    rt.qinfo[r] = make_int4(0, -1, 0, b);
    rt.kvinfo[r] = make_int4(0, b, 0, 0);
  }
}

int launch_prefill_rows(pd_ctx *c, int b, int p0, int n, hipStream_t s) {
  hipLaunchKernelGGL(k_prefill_rows, dim3((c->R_cap + 255) / 256), dim3(256), 0, s, c->rows,
                     c->ctx_tok, b, c->L, p0, n, c->R_cap);
  PD_CHECK_HIP(hipGetLastError());
  return PD_OK;
}

// ---------------------------------------------------------------------------
// embedding: x[r] = E_tok[tok] (+ E_pos[pos]); rows without a token are zeroed
// ---------------------------------------------------------------------------
template <typename WT>
__global__ void k_embed(float *x, const WT *tok_emb, const WT *pos_emb, RowTables rt, int d) {
  int r = blockIdx.x;
  int fl = rt.flags[r], tok = rt.tok[r], pos = rt.pos[r];     // independent loads, one round trip
  bool valid = fl & ROW_VALID;
  size_t tb = valid ? (size_t)tok * d : 0, pb = valid ? (size_t)pos * d : 0;
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    float v = 0.f;
    if (valid) {
      v = ld_f32(tok_emb, tb + c);
      if (pos_emb) v += ld_f32(pos_emb, pb + c);
    }
    x[(size_t)r * d + c] = v;
  }
}

int launch_embed(pd_ctx *c, int R, hipStream_t s) {
  int d = c->cfg.d_model;
  if (c->cfg.dtype == 0)
    hipLaunchKernelGGL(k_embed<float>, dim3(R), dim3(256), 0, s, c->x, (const float *)c->tok_emb,
                       (const float *)c->pos_emb, c->rows, d);
  else
    hipLaunchKernelGGL(k_embed<bf16_t>, dim3(R), dim3(256), 0, s, c->x, (const bf16_t *)c->tok_emb,
                       (const bf16_t *)c->pos_emb, c->rows, d);
  PD_CHECK_HIP(hipGetLastError());
  return PD_OK;
}

// ---------------------------------------------------------------------------
// commit: Algorithm 1 lines 9-13 for one request per block, plus the optional
// copy of this step's logits to the caller's [B][S][V] buffer.
// ---------------------------------------------------------------------------
__global__ void k_commit(SchedState st, RowTables rt, const int32_t *row_argmax, int S, int M,
                         int time_max, int eos, int B, int V) {
  int b = blockIdx.x;
  if (threadIdx.x != 0) return;
  if (st.done[b]) return;
  int t = st.step[b], k = st.k_open[b];
  bool all_fin = k > 0;
  for (int i = 0; i < k; ++i) {
    int r = st.row_of[b * S + i];
    if (r >= 0 && (rt.flags[r] & ROW_PRODUCE)) {
      int f = st.force[b * S + i];
      int tok = f >= 0 ? f : row_argmax[r];
      // non-finite logits leave the argmax without a winner: keep the id inside the vocabulary so
      // that the next embedding gather stays in bounds
      if (tok < 0 || tok >= V) tok = 0;
      int nt = st.n_tok[b * S + i];
      st.grid[(size_t)(b * S + i) * (M + 1) + nt] = tok;
      st.n_tok[b * S + i] = nt + 1;
      st.step_tok[b * S + i] = tok;
      if (eos >= 0 && tok == eos) st.fin[b * S + i] = 1;
      else if (nt >= M) st.fin[b * S + i] = 2;       // nt generated tokens now held
    }
    st.force[b * S + i] = -1;
    all_fin = all_fin && st.fin[b * S + i] != 0;
  }
  for (int i = k; i < S; ++i) st.force[b * S + i] = -1;
  if (all_fin || t >= time_max) {
    st.done[b] = 1; st.steps[b] = t;
    atomicAdd(st.all_done, 1);
  }
}

__global__ void k_scatter_logits(float *dst, const float *src, RowTables rt, int S, int V) {
  int r = blockIdx.x;
  if (!(rt.flags[r] & ROW_VALID)) return;
  size_t o = ((size_t)rt.req[r] * S + (rt.sub[r] - 1)) * V, i = (size_t)r * V;
  for (int v = blockIdx.y * blockDim.x + threadIdx.x; v < V; v += gridDim.y * blockDim.x)
    dst[o + v] = src[i + v];
}

int launch_commit(pd_ctx *c, float *out_logits, hipStream_t s) {
  if (out_logits) {
    hipLaunchKernelGGL(k_scatter_logits, dim3(c->R, 8), dim3(256), 0, s, out_logits, c->logits,
                       c->rows, c->S, c->cfg.vocab);
    PD_CHECK_HIP(hipGetLastError());
  }
  hipLaunchKernelGGL(k_commit, dim3(c->B), dim3(64), 0, s, c->sch, c->rows, c->row_argmax, c->S,
                     c->M, c->time_max, c->cfg.eos_id, c->B, c->cfg.vocab);
  PD_CHECK_HIP(hipGetLastError());
  return PD_OK;
}

// ---------------------------------------------------------------------------
// rotary table: cs[p][j] = (cos, sin)(p * base^(-2j/hd)), evaluated in fp64
// ---------------------------------------------------------------------------
__global__ void k_rope_table(float *cs, int rows, int half, double base) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * half) return;
  int p = i / half, j = i % half;
  double ang = (double)p * pow(base, -(double)j / (double)half);
  cs[2 * (size_t)i] = (float)cos(ang);
  cs[2 * (size_t)i + 1] = (float)sin(ang);
}

int launch_rope_table(pd_ctx *c, hipStream_t s) {
  int half = c->cfg.head_dim / 2, n = c->rope_rows * half;
  hipLaunchKernelGGL(k_rope_table, dim3((n + 255) / 256), dim3(256), 0, s, c->rope_cs,
                     c->rope_rows, half, (double)c->cfg.rope_base);
  PD_CHECK_HIP(hipGetLastError());
  return PD_OK;
}
