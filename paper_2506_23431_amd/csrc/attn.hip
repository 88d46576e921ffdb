// Masked multi-query attention of the pipelined decode step on the matrix cores.
//
// Dependency rule (paper Section 3.2): the row of subsequence i sees every context
// key and the generated-side keys of subsequences i' <= i fed so far, this step's
// included.  In the cache every generated-side slot is tagged with its subsequence,
// so the rule is one integer compare per key.  Prefill rows use the same kernel
// with a causal limit instead (key index < lim).
//
// grid (split, head, request * query-group); block = 4 waves.  The 32-key blocks of one
// (request, head) are dealt round-robin to the 4*nsplit waves that serve it, so the
// first block of every wave is known at launch and its K/V fragments are requested
// before anything else is read.  Per block of 32 keys: 2*(hd/32) K fragments and hd/16 V fragments
// (1 KiB each, contiguous), two 16-key score tiles S^T = K Q^T, mask, online
// softmax (running max / sum per query), O^T += V^T P^T.  Up to 16 query rows of a
// request share every key/value byte read.  Waves are merged through LDS; blocks
// write (max, sum, O) partials that a second, tiny kernel merges by log-sum-exp.
#include "mfma_common.h"

#include <algorithm>

struct AttnArgs {
  const f16_t *q, *q_lo;    // [rows][d] fp16 high / low parts (q_lo NULL: high part only)
  const f16_t *kc, *vc;     // packed fp16 caches of this layer
  bf16_t *out, *out_lo;     // [rows][d] high / low parts (out_lo NULL: high part only)
  RowTables rt;
  const int32_t *kv_len, *gen_sub;
  int kv_override;          // >= 0: number of keys to consider (prefill), else kv_len[req]
  float *part;
  int d, H, kv_cap, gen_cap, L, A, nqg, req0, nsplit, nblk_static;
  float scale_log2;         // log2(e) / sqrt(hd)
};

template <int HD>
struct KVBlock {
  Frag k[2][HD / 32];
  Frag v[HD / 16];
};

template <int HD>
__device__ __forceinline__ void load_block(KVBlock<HD> &b, const uint4 *Kp, const uint4 *Vp, int kb) {
  constexpr int NC = HD / 32, NHB = HD / 16;
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int c = 0; c < NC; ++c) b.k[t][c].u = Kp[((size_t)(kb * 2 + t) * NC + c) * 64];
#pragma unroll
  for (int i = 0; i < NHB; ++i) b.v[i].u = Vp[((size_t)kb * NHB + i) * 64];
}

template <int HD, bool SPLIT, bool DB>
__global__ __launch_bounds__(256, DB ? 1 : 3) void k_attn_mfma(AttnArgs a) {
  constexpr int NC = HD / 32, NHB = HD / 16, PSTR = HD + 2;   // partial: m, l, O[HD] per query
  __shared__ float sm_m[4][16], sm_l[4][16];
  __shared__ float sm_o[4][HD][17];
  int split = blockIdx.x, h = blockIdx.y, z = blockIdx.z;
  int reqi = z / a.nqg, qg = z % a.nqg, req = a.req0 + reqi;
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int n = lane & 15, g = lane >> 4;

  const uint4 *Kp = (const uint4 *)(a.kc + ((size_t)req * a.H + h) * a.kv_cap * HD) + lane;
  const uint4 *Vp = (const uint4 *)(a.vc + ((size_t)req * a.H + h) * a.kv_cap * HD) + lane;
  // 32-key blocks are dealt round-robin to the 4*nsplit waves that serve this (request, head):
  // whatever the current key count, no wave gets more than one block above the average
  const int stride = 4 * a.nsplit;
  int kb = split * 4 + wave;
  KVBlock<HD> A, B;
  if (kb < a.nblk_static) load_block<HD>(A, Kp, Vp, kb);   // in flight while the row data is fetched

  // everything the block needs to know about its queries, requested in one go: no load
  // below depends on the result of another
  int qa = qg * 16 + n;                       // query index inside the request
  bool in_req = qa < a.A;
  int r = reqi * a.A + (in_req ? qa : 0);     // row (clamped: loads stay in bounds)
  int4 qi = a.rt.qinfo[r];                    // {flags, sub, lim, req}
  int n_keys = a.kv_override >= 0 ? a.kv_override : a.kv_len[req];
  Frag qf[NC], ql[SPLIT ? NC : 1];
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    size_t off = act_off(r, h * HD + c * 32 + g * 8, a.d);
    qf[c].u = *(const uint4 *)(a.q + off);
    if (SPLIT) ql[c].u = *(const uint4 *)(a.q_lo + off);
  }
  bool qvalid = in_req && (qi.x & ROW_VALID);
  int q_sub = qvalid ? qi.y : -1, q_lim = qvalid ? qi.z : 0;
  if (!qvalid) {
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      qf[c].u = make_uint4(0, 0, 0, 0);
      if (SPLIT) ql[c].u = make_uint4(0, 0, 0, 0);
    }
  }
  // keys any query of this group can see
  int reach = qvalid ? (n_keys > a.L && q_sub >= 1 ? n_keys : min(q_lim, n_keys)) : 0;
  for (int o = 1; o < 16; o <<= 1) reach = max(reach, __shfl_xor(reach, o));
  int end = min(a.nblk_static, (reach + 31) >> 5);
  const int32_t *gs = a.gen_sub + (size_t)req * a.gen_cap;

  float m_run = -INFINITY, l_run = 0.f;
  floatx4 o_acc[NHB];
#pragma unroll
  for (int i = 0; i < NHB; ++i) o_acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};

  auto compute = [&](const KVBlock<HD> &blk, int kbc) {
    floatx4 s[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      s[t] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < NC; ++c) s[t] = mfma16h(blk.k[t][c], qf[c], s[t]);
      if (SPLIT) {
#pragma unroll
        for (int c = 0; c < NC; ++c) s[t] = mfma16h(blk.k[t][c], ql[c], s[t]);
      }
    }
    // lane (n, g), tile t, register j  <->  key kbc*32 + 8g + 4t + j
    int key0 = kbc * 32 + 8 * g;
    float sv[8];
    bool tail = key0 + 8 > a.L || key0 + 8 > q_lim;     // needs the per-key test
    float mloc = -INFINITY;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      int key = key0 + e;
      bool vis = true;
      if (tail) {
        vis = key < q_lim;
        if (!vis && key >= a.L && key < n_keys) vis = gs[key - a.L] <= q_sub;
      }
      float v = vis ? s[e >> 2][e & 3] * a.scale_log2 : -INFINITY;
      sv[e] = v;
      mloc = fmaxf(mloc, v);
    }
    mloc = fmaxf(mloc, __shfl_xor(mloc, 16));
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
    float m_new = fmaxf(m_run, mloc);
    float alpha = m_new == -INFINITY ? 1.f : exp2f(m_run - m_new);
    float p[8], psum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      p[e] = sv[e] == -INFINITY ? 0.f : exp2f(sv[e] - m_new);
      psum += p[e];
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    Frag pf, pl;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pf.hh[e] = (f16_t)p[e];
      if (SPLIT) pl.hh[e] = (f16_t)(p[e] - (float)pf.hh[e]);
    }
#pragma unroll
    for (int i = 0; i < NHB; ++i) {
      o_acc[i] *= alpha;
      o_acc[i] = mfma16h(blk.v[i], pf, o_acc[i]);
      if (SPLIT) o_acc[i] = mfma16h(blk.v[i], pl, o_acc[i]);
    }
  };

  if (DB) {
    // ping-pong over the wave's blocks kb, kb+4, ...: the next block is requested
    // before the current one is consumed
    while (kb < end) {
      int kn = kb + stride;
      if (kn < end) load_block<HD>(B, Kp, Vp, kn);
      compute(A, kb);
      if (kn >= end) break;
      kb = kn;
      kn = kb + stride;
      if (kn < end) load_block<HD>(A, Kp, Vp, kn);
      compute(B, kb);
      kb = kn;
    }
  } else {
    // one block in flight per wave; the resident waves of the compute unit overlap
    while (kb < end) {
      compute(A, kb);
      kb += stride;
      if (kb < end) load_block<HD>(A, Kp, Vp, kb);
    }
  }
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);

  // ---- merge the 4 waves of the block (log-sum-exp) ----
  if (g == 0) { sm_m[wave][n] = m_run; sm_l[wave][n] = l_run; }
#pragma unroll
  for (int i = 0; i < NHB; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) sm_o[wave][i * 16 + 4 * g + j][n] = o_acc[i][j];
  __syncthreads();
  // thread -> (query qn, dims dd, dd + 16, ...)
  int qn = threadIdx.x & 15, dd = threadIdx.x >> 4;
  float mw[4], M = -INFINITY;
#pragma unroll
  for (int w = 0; w < 4; ++w) { mw[w] = sm_m[w][qn]; M = fmaxf(M, mw[w]); }
  float fw[4], lsum = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    fw[w] = mw[w] == -INFINITY ? 0.f : exp2f(mw[w] - M);
    lsum += fw[w] * sm_l[w][qn];
  }
  int out_qa = qg * 16 + qn, out_r = reqi * a.A + out_qa;
  bool out_valid = out_qa < a.A && (__shfl(qi.x, qn) & ROW_VALID);
  if (!out_valid) return;
  if (a.nsplit == 1) {
    float inv = 1.f / lsum;
    for (int dim = dd; dim < HD; dim += 16) {
      float o = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) o += fw[w] * sm_o[w][dim][qn];
      bf16_t hi = f32_to_bf16(o * inv);
      size_t off = act_off(out_r, h * HD + dim, a.d);
      a.out[off] = hi;
      if (a.out_lo) a.out_lo[off] = f32_to_bf16(bf16_residual(o * inv, hi));
    }
    return;
  }
  // partial of this block: rows m, l, O[0..HD) of 16 floats (one per query): stores of
  // neighbouring lanes are contiguous
  size_t unit = (size_t)z * a.H + h;
  float *pp = a.part + (unit * a.nsplit + split) * (size_t)(PSTR * 16) + qn;
  if (dd == 0) { pp[0] = M; pp[16] = lsum; }
  for (int dim = dd; dim < HD; dim += 16) {
    float o = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) o += fw[w] * sm_o[w][dim][qn];
    pp[(2 + dim) * 16] = o;
  }
}

// Merge of the split partials by log-sum-exp.  Block = (unit, 16 dims); thread = (query, dim).
// The (max, sum) pairs of a query are read once, spread over the 4 lanes of a wave that share
// the query, and reduced by shuffles; then every thread accumulates its dim over the splits with
// 16 splits' loads in flight at a time.  Neighbouring lanes read neighbouring floats.
template <int HD>
__global__ __launch_bounds__(256) void k_attn_merge(AttnArgs a) {
  constexpr int PSTR = HD + 2;
  int unit = blockIdx.x, z = unit / a.H, h = unit % a.H;
  int reqi = z / a.nqg, qg = z % a.nqg;
  int qn = threadIdx.x & 15, dg = (threadIdx.x >> 4) & 3, dim = blockIdx.y * 16 + (threadIdx.x >> 4);
  int qa = qg * 16 + qn, r = reqi * a.A + min(qa, a.A - 1);
  int fl = a.rt.flags[r];
  const float *pb = a.part + (size_t)unit * a.nsplit * (PSTR * 16) + qn;
  const size_t sstr = (size_t)PSTR * 16;
  // lane group dg takes splits dg, dg + 4, ...  (nsplit <= 256: at most 64 each, 16 per pass)
  float M = -INFINITY, lg = 0.f;
  for (int s0 = dg; s0 < a.nsplit; s0 += 64) {
    float mv[16], lv[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      int sp = s0 + 4 * u;
      bool in = sp < a.nsplit;
      mv[u] = in ? pb[sp * sstr] : -INFINITY;
      lv[u] = in ? pb[sp * sstr + 16] : 0.f;
    }
    float Mn = M;
#pragma unroll
    for (int u = 0; u < 16; ++u) Mn = fmaxf(Mn, mv[u]);
    if (Mn != -INFINITY) {
      lg *= exp2f(M - Mn);        // M == -inf: lg is 0 and stays 0
#pragma unroll
      for (int u = 0; u < 16; ++u) lg += mv[u] == -INFINITY ? 0.f : exp2f(mv[u] - Mn) * lv[u];
      M = Mn;
    }
  }
#pragma unroll
  for (int off = 16; off <= 32; off <<= 1) {     // combine the 4 lane groups of the query
    float Mo = __shfl_xor(M, off), lo = __shfl_xor(lg, off);
    float Mn = fmaxf(M, Mo);
    lg = (M == -INFINITY ? 0.f : lg * exp2f(M - Mn)) + (Mo == -INFINITY ? 0.f : lo * exp2f(Mo - Mn));
    M = Mn;
  }
  float o = 0.f;
  for (int s0 = 0; s0 < a.nsplit; s0 += 16) {
    float mv[16], ov[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      size_t sp = min(s0 + u, a.nsplit - 1);
      mv[u] = pb[sp * sstr];
      ov[u] = pb[sp * sstr + (2 + dim) * 16];
    }
#pragma unroll
    for (int u = 0; u < 16; ++u)
      o += (s0 + u < a.nsplit && mv[u] != -INFINITY) ? exp2f(mv[u] - M) * ov[u] : 0.f;
  }
  if (qa >= a.A || !(fl & ROW_VALID)) return;
  float y = o / lg;
  bf16_t hi = f32_to_bf16(y);
  size_t off = act_off(r, h * HD + dim, a.d);
  a.out[off] = hi;
  if (a.out_lo) a.out_lo[off] = f32_to_bf16(bf16_residual(y, hi));
}

static int pick_splits(pd_ctx *c, int units, int nblk) {
  int cap = std::max(1, 4096 / units);
  if (c->opt_splits > 0) return std::min(c->opt_splits, cap);
  // about 3 blocks per compute unit, each with at least one key block per wave
  int want = std::max(1, 768 / units);
  int by_keys = std::max(1, nblk / 4);
  return std::max(1, std::min(std::min(want, by_keys), cap));
}

int mfma_attention(pd_ctx *c, const LayerPtrs &lw, int A, int nreq, int req0, int kv_override,
                   hipStream_t s) {
  const pd_config &g = c->cfg;
  AttnArgs a;
  a.q = (const f16_t *)c->q; a.q_lo = (const f16_t *)mfma_lo(c, c->q, g.d_model);
  a.out_lo = mfma_lo(c, c->att, g.d_model); a.kc = (const f16_t *)lw.kc; a.vc = (const f16_t *)lw.vc;
  a.out = (bf16_t *)c->att; a.rt = c->rows; a.kv_len = c->sch.kv_len; a.gen_sub = c->sch.gen_sub;
  a.kv_override = kv_override; a.part = c->att_part;
  a.d = g.d_model; a.H = g.n_head; a.kv_cap = c->kv_cap; a.gen_cap = c->gen_cap; a.L = c->L;
  a.A = A; a.nqg = (A + 15) / 16; a.req0 = req0;
  a.scale_log2 = 1.4426950408889634f / sqrtf((float)g.head_dim);
  int units = nreq * a.nqg * g.n_head;
  PD_REQUIRE(units <= 4096, PD_EINVAL, "too many (request, head, query group) units: %d", units);
  // the most keys this launch can meet: prefill knows it, decode takes the end of the run
  int n_keys = kv_override >= 0 ? kv_override : c->L + c->S * (c->M + 1);
  a.nblk_static = std::min((n_keys + 31) / 32, c->kv_cap / 32);
  a.nsplit = pick_splits(c, units, a.nblk_static);
  dim3 grid(a.nsplit, g.n_head, nreq * a.nqg);
  bool prof = c->opt_profile && kv_override < 0;
  if (prof) {
    while (c->ev_pool.size() < c->ev_used + 2) {
      hipEvent_t ev;
      PD_CHECK_HIP(hipEventCreate(&ev));
      c->ev_pool.push_back(ev);
    }
    PD_CHECK_HIP(hipEventRecord(c->ev_pool[c->ev_used], s));
  }
#define PD_ATTN(HDV)                                                                        \
  do {                                                                                      \
    if (a.q_lo && c->opt_db) hipLaunchKernelGGL((k_attn_mfma<HDV, true, true>), grid, dim3(256), 0, s, a);   \
    else if (a.q_lo) hipLaunchKernelGGL((k_attn_mfma<HDV, true, false>), grid, dim3(256), 0, s, a);          \
    else if (c->opt_db) hipLaunchKernelGGL((k_attn_mfma<HDV, false, true>), grid, dim3(256), 0, s, a);       \
    else hipLaunchKernelGGL((k_attn_mfma<HDV, false, false>), grid, dim3(256), 0, s, a);                     \
    if (a.nsplit > 1)                                                                       \
      hipLaunchKernelGGL(k_attn_merge<HDV>, dim3(units, HDV / 16), dim3(256), 0, s, a);            \
  } while (0)
  switch (g.head_dim) {
    case 32: PD_ATTN(32); break;
    case 64: PD_ATTN(64); break;
    case 96: PD_ATTN(96); break;
    case 128: PD_ATTN(128); break;
    default: pd_set_error("head_dim %d not supported by the MFMA attention", g.head_dim); return PD_EINVAL;
  }
#undef PD_ATTN
  PD_CHECK_HIP(hipGetLastError());
  if (prof) {
    PD_CHECK_HIP(hipEventRecord(c->ev_pool[c->ev_used + 1], s));
    c->ev_used += 2;
  }
  return PD_OK;
}
