// Attention of the context pass (the encoding of the input that precedes decoding; Eq. 1's role):
// causal attention of a chunk of context rows over the keys encoded so far, on the matrix cores.
//
// The decode kernel (attn.hip) gives every block 16 queries, because a decode step has no more per
// request; run over a chunk of thousands of context rows it loads every key and value fragment once
// per 16 queries and is bound by the path that brings loaded data into the compute unit.  Here a
// block holds QT = 2 query tiles (32 consecutive rows of one request and head): each wave takes every
// fourth 32-key block of the causal range, loads its 2 * (hd/32) key and hd/16 value fragments once and
// uses them for both query tiles (48 multiplies per 16 loads instead of 24), with one running
// (max, sum, O) state per tile; the four waves are merged through LDS tile by tile.  Same cache layout,
// same online softmax, same probabilities as single fp16 as the decode kernel; no split over blocks,
// no partials, no subsequence tags (context rows see keys with index < their own position + 1).
// Blocks are numbered so that the rows with the longest causal range start first.
#include "mfma_common.h"

#include <algorithm>

struct CtxAttnArgs {
  const f16_t *q, *q_lo;    // [rows][d] fp16 high / low parts (q_lo NULL: high part only)
  const f16_t *kc, *vc;     // packed fp16 caches of this layer
  bf16_t *out, *out_lo;     // [rows][d] high / low parts (out_lo NULL: high part only)
  const int4 *qinfo;        // [rows] {flags, sub, lim, req}
  int d, H, kv_cap, A, nqg, req0, n_keys;
  float scale_log2;         // log2(e) / sqrt(hd)
};

template <int HD, bool SPLIT, int QT>
__global__ __launch_bounds__(256, 2) void k_attn_ctx(CtxAttnArgs a) {
  constexpr int NC = HD / 32, NHB = HD / 16;
  __shared__ float sm_m[4][16], sm_l[4][16];
  // the query fragments (main loop) and the waves' outputs (merge) share one buffer
  constexpr int NQF = (SPLIT ? 2 : 1) * NC;
  constexpr int SM_N = QT * NQF > 4 * NHB ? QT * NQF : 4 * NHB;
  __shared__ f16x8 sm_raw[SM_N][64];
  f16x8 (*sm_q)[NQF][64] = (f16x8 (*)[NQF][64])sm_raw;
  floatx4 (*sm_o)[NHB][64] = (floatx4 (*)[NHB][64])sm_raw;
  const int h = blockIdx.x, z = blockIdx.y;
  const int reqi = z / a.nqg, qg = a.nqg - 1 - z % a.nqg, req = a.req0 + reqi;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int n = lane & 15, g = lane >> 4;

  // row data and query fragments of the QT tiles, then the wave's first key/value block: every
  // request is issued before anything is waited for
  int r[QT];
  bool in_req[QT];
  int4 qi[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int qa = (qg * QT + t) * 16 + n;
    in_req[t] = qa < a.A;
    r[t] = reqi * a.A + (in_req[t] ? qa : 0);          // clamped: loads stay in bounds
    qi[t] = a.qinfo[r[t]];
  }
  constexpr int NQ = (NC + 3) / 4;                     // query fragments per wave and tile
  f16x8 qh[QT][NQ], ql[SPLIT ? QT : 1][NQ];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const size_t q_off = act_off(r[t], h * HD + g * 8, a.d);
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
      const size_t off = q_off + (size_t)min(wave + 4 * i, NC - 1) * 512;
      qh[t][i] = *(const f16x8 *)(a.q + off);
      if (SPLIT) ql[t][i] = *(const f16x8 *)(a.q_lo + off);
    }
  }
  const f16x8 *Kp = (const f16x8 *)(a.kc + ((size_t)req * a.H + h) * a.kv_cap * HD) + lane;
  const f16x8 *Vp = (const f16x8 *)(a.vc + ((size_t)req * a.H + h) * a.kv_cap * HD) + lane;
  const int nblk = min((a.n_keys + 31) >> 5, a.kv_cap >> 5);
  Frag kf[2][NC], vf[NHB];
  auto load_k = [&](int kbx) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int c = 0; c < NC; ++c) kf[t][c].hv = Kp[((size_t)(kbx * 2 + t) * NC + c) * 64];
  };
  auto load_v = [&](int kbx) {
#pragma unroll
    for (int i = 0; i < NHB; ++i) vf[i].hv = Vp[((size_t)kbx * NHB + i) * 64];
  };
  int kb = wave;
  load_k(min(kb, nblk - 1));
  load_v(min(kb, nblk - 1));
#pragma unroll
  for (int t = 0; t < QT; ++t)
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
      const int c = min(wave + 4 * i, NC - 1);         // waves beyond the fragment count repeat the last one
      sm_q[t][c][lane] = qh[t][i];
      if (SPLIT) sm_q[t][NC + c][lane] = ql[t][i];
    }
  __syncthreads();

  int q_lim[QT];
  int reach = 0, lim_min = 0x7fffffff;
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const bool valid = in_req[t] && (qi[t].x & ROW_VALID);
    q_lim[t] = valid ? min(qi[t].z, a.n_keys) : 0;
    reach = max(reach, q_lim[t]);
    lim_min = min(lim_min, valid ? q_lim[t] : 0x7fffffff);
  }
  for (int o = 1; o < 16; o <<= 1) {
    reach = max(reach, __shfl_xor(reach, o));
    lim_min = min(lim_min, __shfl_xor(lim_min, o));
  }
  const int end = __builtin_amdgcn_readfirstlane(min(nblk, (reach + 31) >> 5));
  const int lim_all = __builtin_amdgcn_readfirstlane(lim_min);   // keys below it are visible to every valid query

  float m_run[QT], l_run[QT];
  floatx4 o_acc[QT][NHB];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    m_run[t] = -INFINITY; l_run[t] = 0.f;
#pragma unroll
    for (int i = 0; i < NHB; ++i) o_acc[t][i] = floatx4{0.f, 0.f, 0.f, 0.f};
  }

  while (kb < end) {
    floatx4 s[QT][2];
    int ql_lane = lane;
    asm volatile("" : "+v"(ql_lane));         // keeps the query fragments in LDS (re-read per block)
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      s[t][0] = floatx4{0.f, 0.f, 0.f, 0.f};
      s[t][1] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        Frag qf;
        qf.hv = sm_q[t][c][ql_lane];
        s[t][0] = mfma16h(kf[0][c], qf, s[t][0]);
        s[t][1] = mfma16h(kf[1][c], qf, s[t][1]);
        if (SPLIT) {
          qf.hv = sm_q[t][NC + c][ql_lane];
          s[t][0] = mfma16h(kf[0][c], qf, s[t][0]);
          s[t][1] = mfma16h(kf[1][c], qf, s[t][1]);
        }
      }
    }
    // the next block's keys (clamped after the last block: the same bytes again, never used), requested
    // without a branch so that the waits below count exactly the requests in flight
    const int kn = kb + 4;
    load_k(min(kn, nblk - 1));
    // lane (n, g), tile tt, register j  <->  key kb*32 + 8g + 4tt + j
    const int key0 = kb * 32 + 8 * g;
    const bool all_visible = kb * 32 + 32 <= lim_all;
    Frag pf[QT];
    float alpha[QT];
    bool rescale = false;
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      float sv[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float x = s[t][e >> 2][e & 3] * a.scale_log2;
        sv[e] = (all_visible || key0 + e < q_lim[t]) ? x : -INFINITY;
      }
      float mloc = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
      mloc = fmaxf(mloc, __shfl_xor(mloc, 16));
      mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
      const float m_new = fmaxf(m_run[t], mloc);
      const float m_ref = m_new == -INFINITY ? 0.f : m_new;      // nothing visible yet: exp2(-inf) = 0, never NaN
      alpha[t] = __builtin_amdgcn_exp2f(m_run[t] - m_ref);
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float p = __builtin_amdgcn_exp2f(sv[e] - m_ref);
        psum += p;
        pf[t].hh[e] = (f16_t)p;
      }
      l_run[t] = l_run[t] * alpha[t] + psum;
      m_run[t] = m_new;
      rescale |= alpha[t] != 1.f;
    }
    if (__any(rescale)) {                     // rare once the running maxima have settled
#pragma unroll
      for (int t = 0; t < QT; ++t)
#pragma unroll
        for (int i = 0; i < NHB; ++i) o_acc[t][i] *= alpha[t];
    }
#pragma unroll
    for (int i = 0; i < NHB; ++i)
#pragma unroll
      for (int t = 0; t < QT; ++t) o_acc[t][i] = mfma16h(vf[i], pf[t], o_acc[t][i]);
    load_v(min(kn, nblk - 1));
    kb = kn;
  }

  // merge the 4 waves, one query tile at a time through the same LDS buffers
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    float l = l_run[t];
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    __syncthreads();                          // the query fragments / the previous tile's outputs are no longer read
    if (g == 0) { sm_m[wave][n] = m_run[t]; sm_l[wave][n] = l; }
#pragma unroll
    for (int i = 0; i < NHB; ++i) sm_o[wave][i][lane] = o_acc[t][i];
    __syncthreads();
    float mw[4], M = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) { mw[w] = sm_m[w][n]; M = fmaxf(M, mw[w]); }
    float fw[4], lsum = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      fw[w] = mw[w] == -INFINITY ? 0.f : exp2f(mw[w] - M);
      lsum += fw[w] * sm_l[w][n];
    }
    const bool valid = in_req[t] && (qi[t].x & ROW_VALID);
    const float inv = 1.f / lsum;
    for (int i = wave; i < NHB; i += 4) {
      floatx4 o = fw[0] * sm_o[0][i][lane];
#pragma unroll
      for (int w = 1; w < 4; ++w) o += fw[w] * sm_o[w][i][lane];
      if (valid) {
        float y[4] = {o[0] * inv, o[1] * inv, o[2] * inv, o[3] * inv};
        store4_split(a.out, a.out_lo, act_off(r[t], h * HD + i * 16 + 4 * g, a.d), y);
      }
    }
  }
}

// Returns PD_OK when it ran the launch, 1 when the shape is not one it serves (the caller then uses
// the decode kernel), or an error code.
int mfma_attention_ctx(pd_ctx *c, const LayerPtrs &lw, int A, int nreq, int req0, int n_keys, hipStream_t s) {
  const pd_config &g = c->cfg;
  constexpr int QT = 2;
  if (!c->opt_ctx_attn || lw.kc_lo || (g.head_dim != 128 && g.head_dim != 64) || n_keys < 1) return 1;
  const int nqg = (A + 16 * QT - 1) / (16 * QT);
  // too few blocks to fill the chip, or a single query tile: the split decode kernel does better (option value 2 overrides)
  if (c->opt_ctx_attn != 2 && (nreq * nqg * g.n_head < 512 || A < 16 * QT)) return 1;
  CtxAttnArgs a;
  a.q = (const f16_t *)c->q; a.q_lo = (const f16_t *)mfma_lo(c, c->q, g.d_model);
  a.kc = (const f16_t *)lw.kc; a.vc = (const f16_t *)lw.vc;
  a.out = (bf16_t *)c->att; a.out_lo = mfma_lo(c, c->att, g.d_model);
  a.qinfo = c->rows.qinfo; a.d = g.d_model; a.H = g.n_head; a.kv_cap = c->kv_cap; a.A = A; a.nqg = nqg;
  a.req0 = req0; a.n_keys = n_keys;
  a.scale_log2 = 1.4426950408889634f / sqrtf((float)g.head_dim);
  dim3 grid(g.n_head, nreq * nqg);
  if (g.head_dim == 128) {
    if (a.q_lo) hipLaunchKernelGGL((k_attn_ctx<128, true, QT>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((k_attn_ctx<128, false, QT>), grid, dim3(256), 0, s, a);
  } else {
    if (a.q_lo) hipLaunchKernelGGL((k_attn_ctx<64, true, QT>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((k_attn_ctx<64, false, QT>), grid, dim3(256), 0, s, a);
  }
  PD_CHECK_HIP(hipGetLastError());
  return PD_OK;
}
