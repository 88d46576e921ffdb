// Schedule and glue kernels: the integer bookkeeping of Algorithm 1 kept on the
// device (so that a decode step never waits for the host), embedding gather,
// rotary table.
#include "mfma_common.h"

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
// One wave per request: lane i looks after subsequences i, i + 64, ...; rows are numbered in
// subsequence order with a ballot and a population count.
// A subsequence has a row when it holds a token that was not fed yet: its newest
// token (coordinate tau = t).  A subsequence that finished in the previous step is
// fed once more so that its last token enters the KV cache; that row selects no token.
// ---------------------------------------------------------------------------
// Encoder-decoder form (qinfo_x != NULL): L is 0 (the decoder's own cache holds generated tokens only);
// every row also gets an entry of a second table for the attention over the Lx encoder states, and
// every new key slot its grid coordinate (t - 1) + (i - 1), whose difference between a query and a
// visible key is their Manhattan distance (Section 4.3).
__global__ __launch_bounds__(64) void k_tick(SchedState st, RowTables rt, int S, int dt, int M, int L, int A,
                                             int time_max, int bos, int gen_cap, int gen_stride,
                                             uint16_t *gen_coord, int4 *qinfo_x, int Lx) {
  // one wave per request: lane i looks after subsequences i, i + 64, ...
  __shared__ int s_k, s_t;
  const int b = blockIdx.x, lane = threadIdx.x;
  for (int a = lane; a < A; a += 64) {
    rt.flags[b * A + a] = 0;
    rt.qinfo[b * A + a] = make_int4(0, -1, 0, b);
    rt.kvinfo[b * A + a] = make_int4(0, b, 0, 0);
    if (qinfo_x) qinfo_x[b * A + a] = make_int4(0, -1, 0, b);
  }
  for (int i = lane; i < S; i += 64) { st.row_of[b * S + i] = -1; st.step_tok[b * S + i] = -1; }
  if (lane == 0) {
    st.n_rows[b] = 0;
    int k = -1, t = 0;
    if (!st.done[b]) {
      t = st.step[b] + 1;
      if (t > time_max) {          // only reachable with time_max == 0
        st.done[b] = 1;
        atomicAdd(st.all_done, 1);
      } else {
        st.step[b] = t;
        k = st.k_open[b];
        if ((t - 1) % dt == 0 && k < S) {      // Algorithm 1, lines 5-7: open subsequence k + 1
          st.grid[(size_t)(b * S + k) * (M + 1)] = bos;
          st.n_tok[b * S + k] = 1; st.n_fed[b * S + k] = 0; st.fin[b * S + k] = 0;
          ++k;
          st.k_open[b] = k;
        }
      }
    }
    s_k = k; s_t = t;
  }
  __syncthreads();
  const int k = s_k, t = s_t;
  if (k < 0) return;
  // rows in subsequence order: the first min(A, free slots) subsequences that hold an unfed token
  const int ng = st.n_gen[b];
  int a_base = 0;
  for (int i0 = 0; i0 < k; i0 += 64) {
    int i = i0 + lane;
    int nt = 0, fin = 0;
    bool has = false;
    if (i < k) {
      nt = st.n_tok[b * S + i];
      fin = st.fin[b * S + i];
      has = nt > st.n_fed[b * S + i];
    }
    unsigned long long m = __ballot(has);
    int a = a_base + __popcll(m & ((1ull << lane) - 1));
    if (has && a < A && ng + a < gen_cap) {
      int r = b * A + a, fl = ROW_VALID | (fin ? 0 : ROW_PRODUCE);
      rt.req[r] = b; rt.sub[r] = i + 1;
      rt.tok[r] = st.grid[(size_t)(b * S + i) * (M + 1) + nt - 1];
      rt.pos[r] = L + (t - 1) + i;
      rt.slot[r] = L + ng + a;
      rt.lim[r] = L;
      rt.flags[r] = fl;
      rt.qinfo[r] = make_int4(fl, i + 1, L, b);
      rt.kvinfo[r] = make_int4(fl, b, L + ng + a, L + (t - 1) + i);
      st.gen_sub[(size_t)b * gen_stride + (L & 7) + ng + a] = (uint16_t)(i + 1);
      if (qinfo_x) {
        qinfo_x[r] = make_int4(fl, 0, Lx, b);
        gen_coord[(size_t)b * gen_stride + ng + a] = (uint16_t)((t - 1) + i);
      }
      st.n_fed[b * S + i] = nt;
      st.row_of[b * S + i] = r;
    }
    a_base += __popcll(m);
  }
  if (lane == 0) {
    int a = min(a_base, min(A, max(gen_cap - ng, 0)));
    st.n_gen[b] = ng + a; st.kv_len[b] = L + ng + a; st.n_rows[b] = a;
  }
}

int launch_tick(pd_ctx *c, hipStream_t s) {
  hipLaunchKernelGGL(k_tick, dim3(c->B), dim3(64), 0, s, c->sch, c->rows, c->S, c->dt, c->M, c->L,
                     c->A, c->time_max, c->cfg.bos_id, c->gen_cap, c->gen_stride, c->gen_coord, c->qinfo_x, c->Lx);
  PD_CHECK_HIP(hipGetLastError());
  return PD_OK;
}

// ---------------------------------------------------------------------------
// prefill rows: context tokens p0 .. p0+n-1 of request b as rows 0 .. n-1.
// Row for position p sees the keys 0..p (causal prefix), nothing generated; with `bidir` (rows of a
// bidirectional encoder) all L keys.  Keys and values of the rows go to cache entry `b_cache`.
// ---------------------------------------------------------------------------
__global__ void k_prefill_rows(RowTables rt, const int32_t *ctx_tok, int b, int L, int p0, int n,
                               int R_cap, int bidir, int b_cache) {
  int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= R_cap) return;
  if (r < n) {
    int p = p0 + r;
    rt.req[r] = b; rt.sub[r] = 0; rt.tok[r] = ctx_tok[(size_t)b * L + p]; rt.pos[r] = p;
    const int lim = bidir ? L : p + 1;
    rt.slot[r] = p; rt.lim[r] = lim; rt.flags[r] = ROW_VALID;
    rt.qinfo[r] = make_int4(ROW_VALID, 0, lim, b_cache);
    rt.kvinfo[r] = make_int4(ROW_VALID, b_cache, p, p);
  } else {
    rt.flags[r] = 0;
    rt.qinfo[r] = make_int4(0, -1, 0, b);
    rt.kvinfo[r] = make_int4(0, b, 0, 0);
  }
}

int launch_prefill_rows(pd_ctx *c, int b, int p0, int n, hipStream_t s, int L, int bidir, int b_cache) {
  hipLaunchKernelGGL(k_prefill_rows, dim3((c->R_cap + 255) / 256), dim3(256), 0, s, c->rows,
                     c->ctx_tok, b, L, p0, n, c->R_cap, bidir, b_cache);
  PD_CHECK_HIP(hipGetLastError());
  return PD_OK;
}

// ---------------------------------------------------------------------------
// teacher-forced rows (Section 3.3, Fig. 3b): every token of request b's training target as one row,
// subsequence-major (row of token j of subsequence i: the lengths before i, plus j), at the grid
// coordinate Algorithm 1 would feed it, tau = (i-1) dt + 1 + j.  tgt: [B][S][ML] token ids, -1 behind a
// subsequence's last token.  Row r writes key slot L + r with its subsequence tag and coordinate;
// next_tok[r] is the token that follows it (-1 behind the last one: a key, but no loss term).
// One block; the schedule state of the request is used as scratch and is reset by the caller afterwards.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_teacher_rows(RowTables rt, SchedState st, uint16_t *gen_coord,
                                                      int32_t *next_tok, const int32_t *tgt, int b, int S, int ML,
                                                      int dt, int L, int gen_stride, int R_cap, int4 *qinfo_x,
                                                      int Lx) {
  const int32_t *tb = tgt + (size_t)b * S * ML;
  int32_t *len = st.n_tok + (size_t)b * S, *off = st.n_fed + (size_t)b * S;
  for (int i = threadIdx.x; i < S; i += blockDim.x) {
    int n = 0;
    while (n < ML && tb[(size_t)i * ML + n] >= 0) ++n;
    len[i] = n;
  }
  __syncthreads();
  __shared__ int s_total;
  if (threadIdx.x == 0) {
    int acc = 0;
    for (int i = 0; i < S; ++i) { off[i] = acc; acc += len[i]; }
    s_total = acc;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < S; i += blockDim.x) {
    for (int j = 0; j < len[i]; ++j) {
      const int r = off[i] + j;
      if (r >= R_cap) break;
      const bool more = j + 1 < len[i];
      const int fl = ROW_VALID | (more ? ROW_PRODUCE : 0), c = (i * dt + j) + i, p = L + c;
      rt.req[r] = b; rt.sub[r] = i + 1; rt.tok[r] = tb[(size_t)i * ML + j]; rt.pos[r] = p;
      rt.slot[r] = L + r; rt.lim[r] = L; rt.flags[r] = fl;
      rt.qinfo[r] = make_int4(fl, i + 1, L, b);
      rt.kvinfo[r] = make_int4(fl, b, L + r, p);
      st.gen_sub[(size_t)b * gen_stride + (L & 7) + r] = (uint16_t)(i + 1);
      gen_coord[(size_t)b * gen_stride + (L & 7) + r] = (uint16_t)c;
      next_tok[r] = more ? tb[(size_t)i * ML + j + 1] : -1;
      if (qinfo_x) qinfo_x[r] = make_int4(fl, 0, Lx, b);     // encoder-decoder form: all Lx encoder states
    }
  }
  for (int r = s_total + threadIdx.x; r < R_cap; r += blockDim.x) {
    rt.flags[r] = 0; rt.qinfo[r] = make_int4(0, -1, 0, b); rt.kvinfo[r] = make_int4(0, b, 0, 0);
    next_tok[r] = -1;
    if (qinfo_x) qinfo_x[r] = make_int4(0, -1, 0, b);
  }
}

int launch_teacher_rows(pd_ctx *c, const int32_t *tgt_dev, int b, int ML, hipStream_t s) {
  hipLaunchKernelGGL(k_teacher_rows, dim3(1), dim3(256), 0, s, c->rows, c->sch, c->gen_coord, c->row_argmax, tgt_dev,
                     b, c->S, ML, c->dt, c->L, c->gen_stride, c->R_cap, c->qinfo_x, c->Lx);
  PD_CHECK_HIP(hipGetLastError());
  return PD_OK;
}

// Eq. 6, one row per block: nll[r] = log sum_v exp(logits[r][v]) - logits[r][next_tok[r]], 0 for rows
// without a successor.
__global__ __launch_bounds__(256) void k_row_nll(float *nll, const float *logits, size_t ld, int V,
                                                 const int32_t *next_tok) {
  __shared__ float sh[4];
  const int r = blockIdx.x, t = next_tok[r];
  if (t < 0) { if (threadIdx.x == 0) nll[r] = 0.f; return; }      // the same for the whole block
  const float *row = logits + (size_t)r * ld;
  float m = -INFINITY;
  for (int v = threadIdx.x; v < V; v += 256) m = fmaxf(m, row[v]);
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = m;
  __syncthreads();
  m = fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
  __syncthreads();
  float e = 0.f;
  for (int v = threadIdx.x; v < V; v += 256) e += expf(row[v] - m);
  for (int o = 32; o > 0; o >>= 1) e += __shfl_xor(e, o);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = e;
  __syncthreads();
  if (threadIdx.x == 0) nll[r] = m + logf((sh[0] + sh[1]) + (sh[2] + sh[3])) - row[t];
}

// loss of one request: the rows' terms added in row order, in double precision (deterministic)
__global__ void k_loss_sum(double *loss, const float *nll, int n) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  double acc = 0.0;
  for (int r = 0; r < n; ++r) acc += (double)nll[r];
  *loss = acc;
}

int launch_row_nll(pd_ctx *c, const float *logits, int n, double *loss_dev, hipStream_t s) {
  hipLaunchKernelGGL(k_row_nll, dim3(n), dim3(256), 0, s, c->nll, logits, (size_t)c->cfg.vocab, c->cfg.vocab,
                     c->row_argmax);
  hipLaunchKernelGGL(k_loss_sum, dim3(1), dim3(64), 0, s, loss_dev, c->nll, n);
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
__global__ __launch_bounds__(1024) void k_commit(SchedState st, RowTables rt, int32_t *row_argmax,
                                                 const float *part_val, const int32_t *part_idx, int n_tiles,
                                                 int S, int M, int A, int time_max, int eos, int V) {
  // Everything the block needs is requested at once, before the first use, so that the kernel costs
  // about one memory round trip: the schedule state of the request, and (matrix-core path) the
  // winners of the vocabulary tiles of every row, whether or not the row selects a token.
  __shared__ int s_arg[1024];           // s_arg[a]: argmax of row a of this request (a < A <= 1024)
  const int b = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nwave = blockDim.x >> 6;
  const int done = st.done[b], t = st.step[b], k = st.k_open[b];
  const int i0 = threadIdx.x;           // subsequence of this thread in the first pass
  int r0 = -1, fin0 = 0, f0 = -1, nt0 = 0;
  if (i0 < S) {
    r0 = st.row_of[b * S + i0]; fin0 = st.fin[b * S + i0]; f0 = st.force[b * S + i0];
    nt0 = st.n_tok[b * S + i0];
  }
  // stage 1: second stage of the argmax, one wave per row; lowest index wins ties (Eq. 4)
  for (int a = wave; a < A; a += nwave) {
    int r = b * A + a;
    int bi = 0x7fffffff;
    if (part_val) {
      const float *pv = part_val + (size_t)r * n_tiles;
      const int32_t *pi = part_idx + (size_t)r * n_tiles;
      float best = -INFINITY;
      for (int t0 = lane; t0 < n_tiles; t0 += 64 * 8) {
        float v[8]; int ix[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          int tt = min(t0 + 64 * u, n_tiles - 1);        // clamped: a repeated candidate changes nothing
          v[u] = pv[tt];
          ix[u] = pi[tt];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (v[u] > best || (v[u] == best && ix[u] < bi)) { best = v[u]; bi = ix[u]; }
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        float ov = __shfl_xor(best, o);
        int oi = __shfl_xor(bi, o);
        if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
      }
    } else {
      bi = row_argmax[r];               // fp32 path: the argmax kernel has decided
    }
    if (lane == 0) s_arg[a] = bi;
  }
  __syncthreads();
  if (done) return;                     // the same for every thread of the block
  // stage 2: Algorithm 1 lines 9-13, thread i for subsequence i.  A subsequence selects a token
  // when it has a row and was unfinished when the rows were laid out.
  int open_unfinished = 0;
  for (int i = i0; i < S; i += blockDim.x) {
    int r = r0, fin = fin0, f = f0, nt = nt0;
    if (i != i0) {
      r = st.row_of[b * S + i]; fin = st.fin[b * S + i]; f = st.force[b * S + i]; nt = st.n_tok[b * S + i];
    }
    if (i < k) {
      if (r >= 0 && fin == 0) {
        int tok = f >= 0 ? f : s_arg[r - b * A];
        // non-finite logits leave the argmax without a winner: keep the id inside the vocabulary so
        // that the next embedding gather stays in bounds
        if (tok < 0 || tok >= V) tok = 0;
        st.grid[(size_t)(b * S + i) * (M + 1) + nt] = tok;
        st.n_tok[b * S + i] = nt + 1;
        st.step_tok[b * S + i] = tok;
        if (eos >= 0 && tok == eos) fin = 1;
        else if (nt >= M) fin = 2;                     // nt generated tokens now held
        st.fin[b * S + i] = fin;
      }
      if (fin == 0) open_unfinished = 1;
    }
    st.force[b * S + i] = -1;
  }
  int any_unfinished = __syncthreads_or(open_unfinished);
  if (threadIdx.x == 0 && ((k > 0 && !any_unfinished) || t >= time_max)) {
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
  // matrix-core path: the vocabulary projection left one winner per tile; fp32 path: row_argmax is final
  const bool tiles = c->impl == 1;
  hipLaunchKernelGGL(k_commit, dim3(c->B), dim3(tiles ? 1024 : 256), 0, s, c->sch, c->rows, c->row_argmax,
                     tiles ? c->lm_part_val : nullptr, tiles ? c->lm_part_idx : nullptr, c->vocab_pad / 16,
                     c->S, c->M, c->A, c->time_max, c->cfg.eos_id, c->cfg.vocab);
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
