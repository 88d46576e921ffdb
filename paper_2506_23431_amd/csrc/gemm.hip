// Weight re-packing, normalisation and the skinny bf16 GEMM with fused epilogues
// (QKV + rotary + KV append, residual add, GELU, SwiGLU, vocabulary argmax).
#include "mfma_common.h"

#ifndef PD_GEMM_EPI   // ---- common part: weight packing, norm kernel -------------------------------

// ---------------------------------------------------------------------------
// weight re-packing (runs once, in pd_create)
//   mode 0: row(n) = n
//   mode 1: rotary QKV.  Inside the Q and K sections every 16-row tile holds 8 low
//           dims and their rotation partners: tile th of head h, packed row m:
//           dim = th*8 + (m & 7) + (m >= 8 ? hd/2 : 0).  V section: identity.
//   mode 2: SwiGLU.  Tile t holds gate rows t*8..t*8+7 (from src) then up rows
//           t*8..t*8+7 (from src2).
// ---------------------------------------------------------------------------
__global__ void k_pack_weight(bf16_t *dst, const bf16_t *src, const bf16_t *src2, int N_src,
                              int N_pad, int K, int mode, int d, int hd) {
  size_t gran = (size_t)blockIdx.x * blockDim.x + threadIdx.x;   // 16-byte granule index
  int KT = K >> 5;
  size_t total = (size_t)(N_pad >> 4) * KT * 64;
  if (gran >= total) return;
  int lane = gran & 63;
  size_t frag = gran >> 6;
  int kt = frag % KT, nt = frag / KT;
  int m = lane & 15, g = lane >> 4;
  int n = nt * 16 + m;
  const bf16_t *row = nullptr;
  if (mode == 0) {
    if (n < N_src) row = src + (size_t)n * K;
  } else if (mode == 1) {
    if (n < 2 * d) {
      int sec = n / d, nl = n % d, h = nl / hd, th = (nl % hd) >> 4;
      int dim = th * 8 + (m & 7) + (m >= 8 ? hd / 2 : 0);
      row = src + ((size_t)sec * d + h * hd + dim) * K;
    } else {
      row = src + (size_t)n * K;
    }
  } else {
    int f = nt * 8 + (m & 7);
    row = (m < 8 ? src : src2) + (size_t)f * K;
  }
  uint4 v = make_uint4(0, 0, 0, 0);
  if (row) v = *(const uint4 *)(row + kt * 32 + g * 8);
  ((uint4 *)dst)[gran] = v;
}

static int pack(bf16_t *dst, const void *src, const void *src2, int N_src, int N_pad, int K,
                int mode, int d, int hd, hipStream_t s) {
  size_t total = (size_t)(N_pad / 16) * (K / 32) * 64;
  hipLaunchKernelGGL(k_pack_weight, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, dst,
                     (const bf16_t *)src, (const bf16_t *)src2, N_src, N_pad, K, mode, d, hd);
  PD_CHECK_HIP(hipGetLastError());
  return PD_OK;
}

int mfma_pack_matrix(bf16_t *dst, const void *src, int N, int K, hipStream_t s) {
  return pack(dst, src, nullptr, N, (N + 15) / 16 * 16, K, 0, 0, 0, s);
}

int mfma_pack_weights(pd_ctx *c, hipStream_t s) {
  const pd_config &g = c->cfg;
  int d = g.d_model, ff = g.d_ff, hd = g.head_dim, rc;
  for (int l = 0; l < g.n_layer; ++l) {
    LayerPtrs &lp = c->layers[l];
    if ((rc = pack(lp.p_wqkv, lp.wqkv, nullptr, 3 * d, 3 * d, d, g.pos_kind == 1 ? 1 : 0, d, hd, s))) return rc;
    if ((rc = pack(lp.p_wo, lp.wo, nullptr, d, d, d, 0, d, hd, s))) return rc;
    if (g.ffn_kind == 1) {
      if ((rc = pack(lp.p_w1, lp.w1, lp.w_up, ff, 2 * ff, d, 2, d, hd, s))) return rc;
    } else {
      if ((rc = pack(lp.p_w1, lp.w1, nullptr, ff, ff, d, 0, d, hd, s))) return rc;
    }
    if ((rc = pack(lp.p_w2, lp.w2, nullptr, d, d, ff, 0, d, hd, s))) return rc;
  }
  return pack(c->p_lm_head, c->lm_head, nullptr, g.vocab, c->vocab_pad, d, 0, d, hd, s);
}

// ---------------------------------------------------------------------------
// c1[n] = sum_k W[n][k] gain[k], c2[n] = sum_k W[n][k] bias[k] over a packed weight matrix (columns n
// in packed order): what a projection needs to finish a norm in its epilogue when it is fed
// gain * x instead of the normalised row.  One wave per 16-column tile; runs once, in pd_create.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void k_norm_fold(float *c1, float *c2, const bf16_t *Wp, const float *gain,
                                                  const float *bias, int KT) {
  const int nt = blockIdx.x, lane = threadIdx.x, m = lane & 15, g = lane >> 4;
  const uint4 *wp = (const uint4 *)Wp + (size_t)nt * KT * 64 + lane;
  float s1 = 0.f, s2 = 0.f;
  for (int kt = 0; kt < KT; ++kt) {
    Frag w;
    w.u = wp[(size_t)kt * 64];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int k = kt * 32 + g * 8 + e;
      const float wv = bf16_to_f32(w.h[e]);
      s1 = fmaf(wv, gain[k], s1);
      if (bias) s2 = fmaf(wv, bias[k], s2);
    }
  }
  s1 += __shfl_xor(s1, 16); s1 += __shfl_xor(s1, 32);
  s2 += __shfl_xor(s2, 16); s2 += __shfl_xor(s2, 32);
  if (g == 0) {
    c1[nt * 16 + m] = s1;
    if (c2) c2[nt * 16 + m] = s2;
  }
}

int mfma_fold(float *c1, float *c2, const bf16_t *Wp, const float *gain, const float *bias, int n_out, int K,
              hipStream_t s) {
  hipLaunchKernelGGL(k_norm_fold, dim3(n_out / 16), dim3(64), 0, s, c1, bias ? c2 : nullptr, Wp, gain, bias, K / 32);
  PD_CHECK_HIP(hipGetLastError());
  return PD_OK;
}

int mfma_fold_norms(pd_ctx *c, hipStream_t s) {
  const pd_config &g = c->cfg;
  const int n_out = (g.ffn_kind == 1 ? 2 : 1) * g.d_ff;
  int rc;
  for (int l = 0; l < g.n_layer; ++l) {
    LayerPtrs &lp = c->layers[l];
    if ((rc = mfma_fold(lp.c1, lp.c2, lp.p_w1, lp.n2g, g.norm_kind == 0 ? lp.n2b : nullptr, n_out, g.d_model, s))) return rc;
    if (c->arch == 0 && (rc = mfma_fold(lp.q1, lp.q2, lp.p_wqkv, lp.n1g, g.norm_kind == 0 ? lp.n1b : nullptr, 3 * g.d_model, g.d_model, s))) return rc;
  }
  return PD_OK;
}

// ---------------------------------------------------------------------------
// norm -> bf16 activations.  One block per row; rows without a token become zero.
// The row is read once into registers (gain and bias are requested at the same
// time), so the kernel costs one memory round trip plus one block reduction (sum and sum of squares
// together: the variance is E[x^2] - mean^2, as in the projections that finish a norm).
// ---------------------------------------------------------------------------
// EMB: the row is not read from x but gathered from the embedding tables (first norm of a step:
// x = E_tok[token] (+ E_pos[position]), zero for rows without a token) and written to x.
template <int NG, int NP, bool EMB>     // 8-value granules per thread: d <= 2048 * NG; NP pending slices
__global__ __launch_bounds__(256) void k_norm_bf16(bf16_t *xn, bf16_t *xn_lo, const float *x, const float *g,
                                                   const float *b, int d, int kind, float eps,
                                                   const int32_t *flags, int R, float *xw,
                                                   const float *ypart, size_t part_stride,
                                                   const bf16_t *tok_emb, const bf16_t *pos_emb,
                                                   const int32_t *tok, const int32_t *pos) {
  int r = blockIdx.x;
  int fl = r < R ? flags[r] : 0;
  const float *xr = x + (size_t)r * d;
  float v[NG][8], gv[NG][8], bv[NG][8];
  const bf16_t *te = nullptr, *pe = nullptr;
  if (EMB) {
    bool has = fl & ROW_VALID;
    te = tok_emb + (has ? (size_t)tok[r] * d : 0);
    pe = pos_emb ? pos_emb + (has ? (size_t)pos[r] * d : 0) : nullptr;
  }
#pragma unroll
  for (int i = 0; i < NG; ++i) {
    int c = (threadIdx.x + i * 256) * 8;
    bool in = c < d;
    Frag et, ep;
    if (EMB) {
      et.u = in ? *(const uint4 *)(te + c) : make_uint4(0, 0, 0, 0);
      ep.u = (in && pe) ? *(const uint4 *)(pe + c) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      float4 t;
      if (EMB) {
        bool has = fl & ROW_VALID;
        t.x = has ? bf16_to_f32(et.h[4 * h]) + bf16_to_f32(ep.h[4 * h]) : 0.f;
        t.y = has ? bf16_to_f32(et.h[4 * h + 1]) + bf16_to_f32(ep.h[4 * h + 1]) : 0.f;
        t.z = has ? bf16_to_f32(et.h[4 * h + 2]) + bf16_to_f32(ep.h[4 * h + 2]) : 0.f;
        t.w = has ? bf16_to_f32(et.h[4 * h + 3]) + bf16_to_f32(ep.h[4 * h + 3]) : 0.f;
        if (in && r < R) *(float4 *)(xw + (size_t)r * d + c + 4 * h) = t;
      } else {
        t = in ? *(const float4 *)(xr + c + 4 * h) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
      float4 tg = in ? *(const float4 *)(g + c + 4 * h) : make_float4(0.f, 0.f, 0.f, 0.f);
      float4 tb = (in && kind == 0 && b) ? *(const float4 *)(b + c + 4 * h) : make_float4(0.f, 0.f, 0.f, 0.f);
      // pending split-K slices of the last projection: requested together with everything else
      float4 y[NP > 0 ? NP : 1];
#pragma unroll
      for (int pp = 0; pp < NP; ++pp)
        y[pp] = in ? *(const float4 *)(ypart + pp * part_stride + (size_t)r * d + c + 4 * h)
                   : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int pp = 0; pp < NP; ++pp) { t.x += y[pp].x; t.y += y[pp].y; t.z += y[pp].z; t.w += y[pp].w; }
      if (NP > 0 && in && r < R) *(float4 *)(xw + (size_t)r * d + c + 4 * h) = t;
      v[i][4 * h] = t.x; v[i][4 * h + 1] = t.y; v[i][4 * h + 2] = t.z; v[i][4 * h + 3] = t.w;
      gv[i][4 * h] = tg.x; gv[i][4 * h + 1] = tg.y; gv[i][4 * h + 2] = tg.z; gv[i][4 * h + 3] = tg.w;
      bv[i][4 * h] = tb.x; bv[i][4 * h + 1] = tb.y; bv[i][4 * h + 2] = tb.z; bv[i][4 * h + 3] = tb.w;
    }
  }
  bool valid = fl & ROW_VALID;
  float s = 0.f, q = 0.f;
#pragma unroll
  for (int i = 0; i < NG; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) { s += v[i][e]; q += v[i][e] * v[i][e]; }
  // one reduction for both sums (values beyond d are zero)
  for (int o = 32; o > 0; o >>= 1) { s += __shfl_xor(s, o); q += __shfl_xor(q, o); }
  __shared__ float2 sh2[4];
  if ((threadIdx.x & 63) == 0) sh2[threadIdx.x >> 6] = make_float2(s, q);
  __syncthreads();
  s = (sh2[0].x + sh2[1].x) + (sh2[2].x + sh2[3].x);
  q = (sh2[0].y + sh2[1].y) + (sh2[2].y + sh2[3].y);
  float mean = kind == 0 ? s / d : 0.f;
  float rstd = rsqrtf(fmaxf(q / d - mean * mean, 0.f) + eps);
#pragma unroll
  for (int i = 0; i < NG; ++i) {
    int c = (threadIdx.x + i * 256) * 8;
    if (c >= d) continue;
    Frag hi, lo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float y = valid ? (v[i][e] - mean) * rstd * gv[i][e] + bv[i][e] : 0.f;
      hi.h[e] = f32_to_bf16(y);
      lo.h[e] = f32_to_bf16(bf16_residual(y, hi.h[e]));
    }
    size_t off = act_off(r, c, d);
    *(uint4 *)(xn + off) = hi.u;
    if (xn_lo) *(uint4 *)(xn_lo + off) = lo.u;
  }
}

// The same for launches of many rows (the context pass): a wave per row, four rows per block.  Lane l takes the
// 8-value granules l, l + 64, ... of its row, the two sums are wave reductions (no barrier, no LDS), and gain and
// bias are asked for only when the statistics are known (they sit in the caches), so a wave holds little more
// than its row and many waves are resident.
template <int NGW, int NP>     // granules per lane: d <= 512 * NGW; NP pending slices
__global__ __launch_bounds__(256) void k_norm_rows(bf16_t *xn, bf16_t *xn_lo, float *x, const float *g,
                                                   const float *b, int d, int kind, float eps,
                                                   const int32_t *flags, int R, const float *ypart,
                                                   size_t part_stride) {
  const int lane = threadIdx.x & 63, r = blockIdx.x * 4 + (threadIdx.x >> 6);
  const bool valid = r < R && (flags[r] & ROW_VALID);
  float *xr = x + (size_t)r * d;
  float v[NGW][8];
#pragma unroll
  for (int i = 0; i < NGW; ++i) {
    const int c = (lane + 64 * i) * 8;
    const bool in = c < d;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      float4 t = in ? *(const float4 *)(xr + c + 4 * h) : make_float4(0.f, 0.f, 0.f, 0.f);
      float4 y[NP > 0 ? NP : 1];
#pragma unroll
      for (int pp = 0; pp < NP; ++pp)
        y[pp] = in ? *(const float4 *)(ypart + pp * part_stride + (size_t)r * d + c + 4 * h)
                   : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int pp = 0; pp < NP; ++pp) { t.x += y[pp].x; t.y += y[pp].y; t.z += y[pp].z; t.w += y[pp].w; }
      if (NP > 0 && in && r < R) *(float4 *)(xr + c + 4 * h) = t;
      v[i][4 * h] = t.x; v[i][4 * h + 1] = t.y; v[i][4 * h + 2] = t.z; v[i][4 * h + 3] = t.w;
    }
  }
  float s1 = 0.f;
#pragma unroll
  for (int i = 0; i < NGW; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) s1 += v[i][e];
  for (int o = 32; o > 0; o >>= 1) s1 += __shfl_xor(s1, o);
  const float mean = kind == 0 ? s1 / d : 0.f;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < NGW; ++i) {
    const bool in = (lane + 64 * i) * 8 < d;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float t = in ? v[i][e] - mean : 0.f;
      q += t * t;
    }
  }
  for (int o = 32; o > 0; o >>= 1) q += __shfl_xor(q, o);
  const float rstd = rsqrtf(q / d + eps);
#pragma unroll
  for (int i = 0; i < NGW; ++i) {
    const int c = (lane + 64 * i) * 8;
    if (c >= d) continue;
    float gv[8], bv[8];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      float4 tg = *(const float4 *)(g + c + 4 * h);
      float4 tb = (kind == 0 && b) ? *(const float4 *)(b + c + 4 * h) : make_float4(0.f, 0.f, 0.f, 0.f);
      gv[4 * h] = tg.x; gv[4 * h + 1] = tg.y; gv[4 * h + 2] = tg.z; gv[4 * h + 3] = tg.w;
      bv[4 * h] = tb.x; bv[4 * h + 1] = tb.y; bv[4 * h + 2] = tb.z; bv[4 * h + 3] = tb.w;
    }
    Frag hi, lo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float y = valid ? (v[i][e] - mean) * rstd * gv[e] + bv[e] : 0.f;
      hi.h[e] = f32_to_bf16(y);
      lo.h[e] = f32_to_bf16(bf16_residual(y, hi.h[e]));
    }
    size_t off = act_off(r, c, d);
    *(uint4 *)(xn + off) = hi.u;
    if (xn_lo) *(uint4 *)(xn_lo + off) = lo.u;
  }
}

int mfma_norm(pd_ctx *c, const float *gain, const float *bias, int R, hipStream_t s) {
  // packed pairs: rows 8-15 of the fragments belong to the low parts of rows 0-7
  int rows = c->packed ? 8 : (R + 15) / 16 * 16, d = c->cfg.d_model;
  bf16_t *xn = (bf16_t *)c->xn;
  const pd_config &g = c->cfg;
  PD_REQUIRE(d <= 2048 * 4, PD_EINVAL, "d_model %d too large for the norm kernel", d);
  if (rows > 128 && !c->embed_pending && !c->packed) {
#define PD_NORM_R(G, P)                                                                           \
  hipLaunchKernelGGL((k_norm_rows<G, P>), dim3(rows / 4), dim3(256), 0, s, xn, mfma_lo(c, xn, d), c->x, gain, bias, \
                     d, g.norm_kind, g.norm_eps, c->rows.flags, R, c->ypart, (size_t)c->R_pad * d)
#define PD_NORM_RP(G)                                                                            \
  switch (c->pend_parts) {                                                                       \
    case 0: PD_NORM_R(G, 0); break;                                                              \
    case 1: PD_NORM_R(G, 1); break;                                                              \
    case 2: PD_NORM_R(G, 2); break;                                                              \
    case 4: PD_NORM_R(G, 4); break;                                                              \
    default: pd_set_error("unsupported number of pending slices: %d", c->pend_parts); return PD_EINVAL; \
  }
    if (d <= 2048) { PD_NORM_RP(4) } else if (d <= 4096) { PD_NORM_RP(8) } else { PD_NORM_RP(16) }
#undef PD_NORM_RP
#undef PD_NORM_R
    PD_CHECK_HIP(hipGetLastError());
    c->pend_parts = 0;
    return PD_OK;
  }
#define PD_NORM(V, P, E)                                                                         \
  hipLaunchKernelGGL((k_norm_bf16<V, P, E>), dim3(rows), dim3(256), 0, s, xn, mfma_lo(c, xn, d), c->x, gain, bias, \
                     d, g.norm_kind, g.norm_eps, c->rows.flags, R, c->x, c->ypart, (size_t)c->R_pad * d,   \
                     (const bf16_t *)c->tok_emb, (const bf16_t *)c->pos_emb, c->rows.tok, c->rows.pos)
#define PD_NORM_P(V)                                                                             \
  if (c->embed_pending) { PD_NORM(V, 0, true); }                                                 \
  else switch (c->pend_parts) {                                                                  \
    case 0: PD_NORM(V, 0, false); break;                                                         \
    case 1: PD_NORM(V, 1, false); break;                                                         \
    case 2: PD_NORM(V, 2, false); break;                                                         \
    case 4: PD_NORM(V, 4, false); break;                                                         \
    default: pd_set_error("unsupported number of pending slices: %d", c->pend_parts); return PD_EINVAL; \
  }
  if (d <= 2048) { PD_NORM_P(1) } else if (d <= 4096) { PD_NORM_P(2) } else { PD_NORM_P(4) }
#undef PD_NORM_P
#undef PD_NORM
  PD_CHECK_HIP(hipGetLastError());
  c->pend_parts = 0;
  c->embed_pending = false;
  return PD_OK;
}

#endif

#ifdef PD_GEMM_EPI
#define PD_GEMM_CAT2(a, b) a##b
#define PD_GEMM_CAT(a, b) PD_GEMM_CAT2(a, b)
#define PD_GEMM_ENTRY PD_GEMM_CAT(mfma_gemm_epi, PD_GEMM_EPI)

// ---------------------------------------------------------------------------
// skinny GEMM  y[r][n] = sum_k xn[r][k] W[n][k],  r < 16*RT rows (RT = 1, 2, 4, 5, 8); weights and
// activations both fragment-major.
// The matrix core computes the transposed tile: A = weight fragment (16 output columns x 32 k),
// B = activations (32 k x 16 rows), D[4g+j][r] = y[r][n0+4g+j].
// A block has NW_K waves that cut K between them; every wave owns the same NT column tiles and all
// RT row tiles, so the block requests every activation fragment of its K range exactly once and
// uses it for NT weight fragments.  The waves' partial tiles are summed through LDS.  The launch
// lives for a few microseconds up to a few tens: every load must be in flight from the first cycle
// on.  Per chunk of U k-tiles a wave requests everything first (the high- and low-part activation
// fragments of the row tiles, then the weight fragments of its tiles) into registers of their own;
// only then the multiplies run.  A share that is not a multiple of U ends with chunks of 4, 2 and
// 1 k-tiles, so that no load is ever conditional.
// This file is compiled once per epilogue (PD_GEMM_EPI = 0..7: kernels and launch code of that
// epilogue) and once without (weight packing, norm kernel, dispatcher).
// ---------------------------------------------------------------------------
// epilogue of one 16-column tile: lane holds y[r][n0 + j], r = i*16 + m, n0 = nt*16 + 4g, j = 0..3
// Mean and reciprocal standard deviation of a row from the per-tile sums the producing projection
// left (EPI_RESID_NORM), stats[row][tile] = (sum, sum of squares).  The NW waves of a block share the
// work: wave w, lane (m, g) takes the tile pairs g + 4 (w + NW u) of row m, u = 0 .. PS-1, requested at
// kernel start so that they arrive with the first weights; what lies beyond (very wide models) is
// read when the sums are taken.  Fixed order, no atomics: deterministic.
constexpr int PS = 4;
__device__ __forceinline__ void stats_request(const GemmArgs &a, int lane, int w, int nw, float4 (&pre)[PS], int r0) {
  const int m = r0 + (lane & 15), g = lane >> 4, npair = a.stats_tiles >> 1;
  const float4 *sp = (const float4 *)(a.stats_in + (size_t)m * a.stats_tiles);
#pragma unroll
  for (int u = 0; u < PS; ++u) {
    pre[u] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (4 * (w + nw * u) < npair) pre[u] = sp[min(g + 4 * (w + nw * u), npair - 1)];   // the same for the whole wave
  }
}
__device__ __forceinline__ float2 stats_partial(const GemmArgs &a, int lane, int w, int nw, const float4 (&pre)[PS], int r0) {
  const int m = r0 + (lane & 15), g = lane >> 4, npair = a.stats_tiles >> 1;
  const float4 *sp = (const float4 *)(a.stats_in + (size_t)m * a.stats_tiles);
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int u = 0; u < PS; ++u)
    if (g + 4 * (w + nw * u) < npair) { s1 += pre[u].x + pre[u].z; s2 += pre[u].y + pre[u].w; }
  for (int p = g + 4 * (w + nw * PS); p < npair; p += 4 * nw) {
    float4 v = sp[p];
    s1 += v.x + v.z; s2 += v.y + v.w;
  }
  s1 += __shfl_xor(s1, 16); s1 += __shfl_xor(s1, 32);
  s2 += __shfl_xor(s2, 16); s2 += __shfl_xor(s2, 32);
  return make_float2(s1, s2);
}
__device__ __forceinline__ float2 stats_finish(const GemmArgs &a, float2 s) {
  const float inv_d = 1.f / (float)a.norm_d;
  const float mean = a.norm_kind == 0 ? s.x * inv_d : 0.f;
  const float var = fmaxf(s.y * inv_d - mean * mean, 0.f);
  return make_float2(mean, rsqrtf(var + a.norm_eps));
}

// what the finishing wave of a tile asked for at kernel start (EPI_RESID_NORM): the residual rows
// and the next norm's gain at its columns
struct ResidPre { float4 x, g; };
// ... and for a projection that finishes a norm: c1 and c2 at the tile's columns
struct NormPre { float4 c1, c2; };

template <int RT, int EPI>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs &a, int nt, const floatx4 (&acc_in)[RT],
                                              const int4 *kvi, int lane, int r0 = 0,
                                              const float2 *nrm = nullptr, const ResidPre *pre = nullptr,
                                              const NormPre *npre = nullptr) {
  int m = lane & 15, g = lane >> 4;
  int n0 = nt * 16 + 4 * g;
  floatx4 acc[RT];
#pragma unroll
  for (int i = 0; i < RT; ++i) acc[i] = acc_in[i];
  if ((EPI == EPI_GELU || EPI == EPI_SWIGLU || EPI == EPI_QKV_NORM) && nrm) {
    // the activations were gain * x: finish the norm here (columns in the packed order of the weights)
    const float4 c1 = npre ? npre->c1 : *(const float4 *)(a.c1 + n0);
    const float4 c2 = npre ? npre->c2 : (a.c2 ? *(const float4 *)(a.c2 + n0) : make_float4(0.f, 0.f, 0.f, 0.f));
#pragma unroll
    for (int i = 0; i < RT; ++i) {
      acc[i][0] = nrm[i].y * (acc[i][0] - nrm[i].x * c1.x) + c2.x;
      acc[i][1] = nrm[i].y * (acc[i][1] - nrm[i].x * c1.y) + c2.y;
      acc[i][2] = nrm[i].y * (acc[i][2] - nrm[i].x * c1.z) + c2.z;
      acc[i][3] = nrm[i].y * (acc[i][3] - nrm[i].x * c1.w) + c2.w;
    }
  }
  // rows at and beyond a.R are never stored: nobody reads them, and with packed activations their
  // slots hold the low parts of rows 0-7
  if (EPI == EPI_RESID) {
    // split-K slice blockIdx.y of y; the following norm kernel adds the slices to x
    float *yp = a.x + (size_t)blockIdx.y * a.part_stride;
#pragma unroll
    for (int i = 0; i < RT; ++i) {
      int r = r0 + i * 16 + m;
      if (r >= a.R) continue;
      *(float4 *)(yp + (size_t)r * a.ld + n0) = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
    }
  } else if (EPI == EPI_RESID_NORM) {
    const float4 gn = pre ? pre->g : *(const float4 *)(a.gain + n0);
#pragma unroll
    for (int i = 0; i < RT; ++i) {
      int r = r0 + i * 16 + m;
      const bool in = r < a.R;
      float4 xo = make_float4(0.f, 0.f, 0.f, 0.f);
      if (in) xo = (pre && RT == 1) ? pre->x : *(const float4 *)(a.x_res + (size_t)r * a.ld + n0);
      float xn[4] = {xo.x + acc[i][0], xo.y + acc[i][1], xo.z + acc[i][2], xo.w + acc[i][3]};
      float s1 = 0.f, s2 = 0.f;
      if (in) {
        *(float4 *)(a.x_res + (size_t)r * a.ld + n0) = make_float4(xn[0], xn[1], xn[2], xn[3]);
        float z[4] = {gn.x * xn[0], gn.y * xn[1], gn.z * xn[2], gn.w * xn[3]};
        store4_split(a.out_bf, a.out_lo, act_off(r, n0, a.ld), z);
        s1 = (xn[0] + xn[1]) + (xn[2] + xn[3]);
        s2 = (xn[0] * xn[0] + xn[1] * xn[1]) + (xn[2] * xn[2] + xn[3] * xn[3]);
      }
      s1 += __shfl_xor(s1, 16); s1 += __shfl_xor(s1, 32);
      s2 += __shfl_xor(s2, 16); s2 += __shfl_xor(s2, 32);
      if (g == 0) a.stats_out[(size_t)r * a.n_tiles + nt] = make_float2(s1, s2);
    }
  } else if (EPI == EPI_GELU) {
#pragma unroll
    for (int i = 0; i < RT; ++i) {
      int r = r0 + i * 16 + m;
      float y[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float t = acc[i][j];
        y[j] = a.act == 1 ? fmaxf(t, 0.f) : 0.5f * t * (1.f + erff(t * 0.70710678118654752f));
      }
      if (r < a.R) store4_split(a.out_bf, a.out_lo, act_off(r, n0, a.ld), y);
    }
  } else if (EPI == EPI_SWIGLU) {
    // groups 0,1: gate of features nt*8 + 4g + j; groups 2,3: up of nt*8 + 4(g-2) + j
#pragma unroll
    for (int i = 0; i < RT; ++i) {
      int r = r0 + i * 16 + m;
      float y[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float mine = acc[i][j];
        float other = __shfl_xor(mine, 32);
        y[j] = mine / (1.f + __expf(-mine)) * other;     // meaningful on groups 0,1
      }
      if (g < 2 && r < a.R) store4_split(a.out_bf, a.out_lo, act_off(r, nt * 8 + 4 * g, a.ld), y);
    }
  } else if (EPI == EPI_QKV || EPI == EPI_QKV_ROPE || EPI == EPI_QKV_NORM) {
    int sec = n0 / a.d + a.sec0, nl = n0 % a.d, h = nl / a.hd;
    int half = a.hd >> 1;
#pragma unroll
    for (int i = 0; i < RT; ++i) {
      int r = r0 + i * 16 + m;
      bool valid = r < a.R && (kvi[i].x & ROW_VALID);
      float y[4];
      int dim0;                                  // head-dim index of y[0]; y[j] is dim0 + j
      if (EPI == EPI_QKV_ROPE && sec < 2) {
        int th = (nl % a.hd) >> 4;
        int jj = th * 8 + 4 * (g & 1);           // rotation pair index of y[0]
        dim0 = jj + (g >= 2 ? half : 0);
        const float *cs = a.rope_cs + ((size_t)(valid ? kvi[i].w : 0) * half + jj) * 2;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float mine = acc[i][j];
          float other = __shfl_xor(mine, 32);
          float cc = cs[2 * j], ss = cs[2 * j + 1];
          // low half: x1*c - x2*s ; high half: x2*c + x1*s
          y[j] = g < 2 ? mine * cc - other * ss : mine * cc + other * ss;
        }
      } else {
        dim0 = (nl % a.hd);
#pragma unroll
        for (int j = 0; j < 4; ++j) y[j] = acc[i][j];
      }
      if (!valid) continue;
      // keys and values beyond the largest half are stored saturated; count them so that the caller
      // can find out (practically never taken)
      if (sec != 0 && fmaxf(fmaxf(fabsf(y[0]), fabsf(y[1])), fmaxf(fabsf(y[2]), fabsf(y[3]))) > 65504.f)
        atomicAdd(a.kv_sat, (fabsf(y[0]) > 65504.f) + (fabsf(y[1]) > 65504.f) + (fabsf(y[2]) > 65504.f) +
                                (fabsf(y[3]) > 65504.f));
      if (sec == 0) {
        store4_split_h((f16_t *)a.out_bf, (f16_t *)a.out_lo, act_off(r, h * a.hd + dim0, a.d), y);
      } else {
        size_t head_base = ((size_t)kvi[i].y * a.H + h) * a.kv_cap * a.hd;
        int slot = kvi[i].z;
        if (sec == 1) {
          store4_split_h(a.kc, a.kc_lo, head_base + k_cache_off(slot, dim0, a.hd), y);
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            size_t o = head_base + v_cache_off(slot, dim0 + j, a.hd);
            f16_t hi = f32_to_f16_sat(y[j]);
            a.vc[o] = hi;
            if (a.vc_lo) a.vc_lo[o] = (f16_t)(y[j] - (float)hi);
          }
        }
      }
    }
  } else if (EPI == EPI_LM) {
#pragma unroll
    for (int i = 0; i < RT; ++i) {
      int r = r0 + i * 16 + m;
      float best = -INFINITY;
      int bi = 0x7fffffff;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int n = n0 + j;
        float t = acc[i][j];
        if (n < a.V) {
          if (a.logits && r < a.R) a.logits[(size_t)r * a.ld_logits + n] = t;
          if (t > best) { best = t; bi = n; }
        }
      }
      // across the 4 column groups of this row; lowest index wins ties
#pragma unroll
      for (int o = 16; o <= 32; o <<= 1) {
        float ov = __shfl_xor(best, o);
        int oi = __shfl_xor(bi, o);
        if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
      }
      if (g == 0 && r < a.R) {      // row-major [row][tile]: the commit kernel reads a row's winners as one run
        a.part_val[(size_t)r * a.n_tiles + nt] = best;
        a.part_idx[(size_t)r * a.n_tiles + nt] = bi;
      }
    }
  }
}

// SW: the weight fragments are loaded with the non-temporal hint.  A step reads every weight once; when the
// step's bytes exceed the last-level cache nothing of them is left there a step later, and keeping them out
// of the caches' way makes the streams faster (cfg4 1.35 -> 1.31 ms per step, cfg5 6.27 -> 6.09); a model
// that fits the cache is served from it step after step and loses with the hint (cfg2 0.187 -> 0.202).
template <bool SW>
__device__ __forceinline__ bf16x8 ld_w(const uint4 *p) {
  return SW ? __builtin_nontemporal_load((const bf16x8 *)p) : *(const bf16x8 *)p;
}

template <int RT, int NT, int U, bool SPLIT, int NA, bool SW>
__device__ __forceinline__ void gemm_chunk(floatx4 (&acc)[NT][RT][NA], const uint4 *wp, const uint4 *xp,
                                           const uint4 *xl, size_t KT, const int (&tile)[NT], int kt) {
  Frag wa[NT][U], xh[RT][U], xo[SPLIT ? RT : 1][U];
#pragma unroll
  for (int i = 0; i < RT; ++i)
#pragma unroll
    for (int u = 0; u < U; ++u) {
      xh[i][u].u = xp[((size_t)i * KT + kt + u) * 64];
      if (SPLIT) xo[i][u].u = xl[((size_t)i * KT + kt + u) * 64];
    }
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int u = 0; u < U; ++u) wa[t][u].v = ld_w<SW>(&wp[((size_t)tile[t] * KT + kt + u) * 64]);
  __builtin_amdgcn_sched_barrier(0);          // every request above is issued before the first multiply
#pragma unroll
  for (int u = 0; u < U; ++u)
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int i = 0; i < RT; ++i) {
        // small tiles keep two accumulators per tile (NA = 2) so that the high- and low-part products
        // do not wait for each other; large tiles have enough independent accumulators anyway
        acc[t][i][0] = mfma16(wa[t][u], xh[i][u], acc[t][i][0]);
        if (SPLIT) acc[t][i][NA - 1] = mfma16(wa[t][u], xo[i][u], acc[t][i][NA - 1]);
      }
}

// PACK (one row tile, at most 8 rows): the activation fragment carries the high parts in rows 0-7
// and the low parts of the same 8 rows in rows 8-15, so one fragment and one multiply per k-tile
// do the work of two; the two halves of the output tile are added before the epilogue.
// ZROWS: the block serves row tiles blockIdx.z * RT .. + RT - 1 only (launches that spread the row tiles of a
// step over blocks, see launch_gemm_zrows).
// SW: weights loaded with the non-temporal hint (see ld_w; chosen per context, never with ZROWS, whose row
// tiles re-read the weights through L2).
template <int RT, int NT, int NW_K, int U, int EPI, bool SPLIT, bool PACK, bool ZROWS = false, bool SW = false>
__global__ __launch_bounds__(64 * NW_K) void k_gemm_s(GemmArgs a) {
  static_assert(!PACK || (RT == 1 && !SPLIT), "packed activations: one row tile, one fragment");
  const int rz = ZROWS ? (int)blockIdx.z * RT : 0;          // first row tile of this block
  __shared__ floatx4 red[NW_K > 1 ? NW_K * NT * RT * 64 : 1];
  const int wk = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int nt0 = blockIdx.x * NT;
  const int m = lane & 15;
  const int KT = a.K >> 5;
  // waves along K: NW_K in this block times gridDim.y blocks (EPI_RESID only)
  const int gk = blockIdx.y * NW_K + wk;
  const int kt0 = min(gk * a.k_share, KT), kt1 = min(kt0 + a.k_share, KT);
  // row data of the KV-append epilogue, requested now so that it arrives with the weights
  int4 kvi[(EPI == EPI_QKV || EPI == EPI_QKV_ROPE || EPI == EPI_QKV_NORM) ? RT : 1];
  if (EPI == EPI_QKV || EPI == EPI_QKV_ROPE || EPI == EPI_QKV_NORM) {
#pragma unroll
    for (int i = 0; i < RT; ++i) kvi[i] = a.rt.kvinfo[(rz + i) * 16 + m];
  }
  int tile[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) tile[t] = min(nt0 + t, a.n_tiles - 1);   // tiles past the end repeat the last one
  // one row tile: what the epilogue needs from memory is asked for now, so that it arrives with the weights
  constexpr bool FUSED_IN = RT == 1 && (EPI == EPI_GELU || EPI == EPI_SWIGLU || EPI == EPI_QKV_NORM);
  constexpr bool FUSED_OUT = RT == 1 && EPI == EPI_RESID_NORM;
  __shared__ float2 sm_stat[FUSED_IN ? NW_K : 1][16];
  float4 pre_s[PS];
  const bool fused_norm = FUSED_IN && a.stats_in != nullptr;          // the same for the whole launch
  NormPre pre_n;
  if (fused_norm) stats_request(a, lane, wk, NW_K, pre_s, rz * 16);
  if (fused_norm && wk < NT) {      // wave w < NT finishes tile nt0 + w
    const int n0 = min(nt0 + wk, a.n_tiles - 1) * 16 + 4 * (lane >> 4);
    pre_n.c1 = *(const float4 *)(a.c1 + n0);
    pre_n.c2 = a.c2 ? *(const float4 *)(a.c2 + n0) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  ResidPre pre_r;
  if (FUSED_OUT && wk < NT) {       // wave w < NT finishes tile nt0 + w
    const int n0 = min(nt0 + wk, a.n_tiles - 1) * 16 + 4 * (lane >> 4);
    pre_r.g = *(const float4 *)(a.gain + n0);
    // (rows beyond R read row R - 1 and are masked where the value is used, not here: touching the
    // value now would make the wave wait for it before it has asked for its weights)
    pre_r.x = *(const float4 *)(a.x_res + (size_t)min(rz * 16 + m, max(a.R - 1, 0)) * a.ld + n0);
  }
  constexpr int NA = (SPLIT && NT * RT <= 2) ? 2 : 1;
  floatx4 acc2[NT][RT][NA];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int i = 0; i < RT; ++i) acc2[t][i][0] = acc2[t][i][NA - 1] = floatx4{0.f, 0.f, 0.f, 0.f};
  const uint4 *wp = (const uint4 *)a.W + lane;
  const uint4 *xp = (const uint4 *)a.xn + lane + (size_t)rz * KT * 64;
  const uint4 *xl = SPLIT ? (const uint4 *)a.xn_lo + lane + (size_t)rz * KT * 64 : nullptr;
  int kt = kt0;
  while (kt + U <= kt1) { gemm_chunk<RT, NT, U, SPLIT, NA, SW>(acc2, wp, xp, xl, KT, tile, kt); kt += U; }
  if (U > 4 && kt + 4 <= kt1) { gemm_chunk<RT, NT, 4, SPLIT, NA, SW>(acc2, wp, xp, xl, KT, tile, kt); kt += 4; }
  if (U > 2 && kt + 2 <= kt1) { gemm_chunk<RT, NT, 2, SPLIT, NA, SW>(acc2, wp, xp, xl, KT, tile, kt); kt += 2; }
  if (U > 1 && kt < kt1) gemm_chunk<RT, NT, 1, SPLIT, NA, SW>(acc2, wp, xp, xl, KT, tile, kt);
  floatx4 acc[NT][RT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int i = 0; i < RT; ++i) acc[t][i] = NA == 2 ? acc2[t][i][0] + acc2[t][i][1] : acc2[t][i][0];
  if (PACK) {
    // output row m + 8 holds the product with the low parts of row m
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[t][0][j] += __shfl_xor(acc[t][0][j], 8);
  }
  if (NW_K > 1) {
    // every wave leaves its partial tiles in LDS; wave w then sums and finishes column tiles w, w + NW_K, ...
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int i = 0; i < RT; ++i) red[((wk * NT + t) * RT + i) * 64 + lane] = acc[t][i];
    if (fused_norm) {
      float2 sp = stats_partial(a, lane, wk, NW_K, pre_s, rz * 16);
      if (lane < 16) sm_stat[wk][lane] = sp;
    }
    __syncthreads();
    float2 nrm[RT];
    if (fused_norm && wk < NT) {            // finishing waves: add the waves' shares in wave order
      float2 tot = sm_stat[0][m];
#pragma unroll
      for (int w = 1; w < NW_K; ++w) { tot.x += sm_stat[w][m].x; tot.y += sm_stat[w][m].y; }
      nrm[0] = stats_finish(a, tot);
    }
    for (int t = wk; t < NT && nt0 + t < a.n_tiles; t += NW_K) {
      floatx4 sum[RT];
#pragma unroll
      for (int i = 0; i < RT; ++i) sum[i] = red[((0 * NT + t) * RT + i) * 64 + lane];
#pragma unroll
      for (int w = 1; w < NW_K; ++w)
#pragma unroll
        for (int i = 0; i < RT; ++i) sum[i] += red[((w * NT + t) * RT + i) * 64 + lane];
      gemm_epilogue<RT, EPI>(a, nt0 + t, sum, kvi, lane, rz * 16, fused_norm ? nrm : nullptr,
                             (FUSED_OUT && t == wk) ? &pre_r : nullptr, (fused_norm && t == wk) ? &pre_n : nullptr);
    }
  } else {
    float2 nrm[RT];
    if (fused_norm) nrm[0] = stats_finish(a, stats_partial(a, lane, 0, 1, pre_s, rz * 16));
#pragma unroll
    for (int t = 0; t < NT; ++t)
      if (nt0 + t < a.n_tiles)
        gemm_epilogue<RT, EPI>(a, nt0 + t, acc[t], kvi, lane, rz * 16, fused_norm ? nrm : nullptr,
                               (FUSED_OUT && t == 0) ? &pre_r : nullptr, (fused_norm && t == 0) ? &pre_n : nullptr);
  }
}

// ---------------------------------------------------------------------------
// launch
// ---------------------------------------------------------------------------
// 1 row tile.  Two column tiles per wave when that still leaves 128 or more blocks: the
// activation fragments (2 KiB per k-tile with the low parts) are then requested once for 2 KiB of
// weights instead of 1 KiB, and the vector-memory pipeline of a compute unit, which every request
// occupies for the same time whether it is served by HBM or by L2, has a third less to do.  A
// wave's share of K is at most 8 k-tiles (two requests of 4), less when the launch would
// otherwise have fewer than about 1500 waves; up to 16 waves along K per block are summed
// through LDS and, for the residual projections, K is also cut into slices over blocks that the
// next norm kernel sums.
template <int RT, int NT, int EPI, bool SPLIT, bool PACK>
static int launch_gemm_small_nt(GemmArgs a, int ks, hipStream_t s) {
  constexpr int U = 4;
  int KT = a.K / 32, groups = (a.n_tiles + NT - 1) / NT;
  int per_block = (KT + ks - 1) / ks;          // k-tiles of one block
  int nwk = NT;
  while (nwk < 16 && (per_block + nwk - 1) / nwk > 8) nwk *= 2;
  while (nwk < 16 && (long)groups * ks * nwk < 1500 && (per_block + nwk - 1) / nwk > 2) nwk *= 2;
  a.k_share = (per_block + nwk - 1) / nwk;
  dim3 grid(groups, ks);
#define PD_LAUNCH(NWK) \
  do {                                                                                            \
    if (a.stream_w)                                                                               \
      hipLaunchKernelGGL((k_gemm_s<RT, NT, (NWK < NT ? NT : NWK), U, EPI, SPLIT, PACK, false, true>), grid, \
                         dim3(64 * (NWK < NT ? NT : NWK)), 0, s, a);                              \
    else                                                                                          \
      hipLaunchKernelGGL((k_gemm_s<RT, NT, (NWK < NT ? NT : NWK), U, EPI, SPLIT, PACK>), grid,    \
                         dim3(64 * (NWK < NT ? NT : NWK)), 0, s, a);                              \
  } while (0)
  switch (nwk) {
    case 1: PD_LAUNCH(1); break;
    case 2: PD_LAUNCH(2); break;
    case 4: PD_LAUNCH(4); break;
    case 8: PD_LAUNCH(8); break;
    default: PD_LAUNCH(16); break;
  }
#undef PD_LAUNCH
  PD_CHECK_HIP(hipGetLastError());
  if (EPI == EPI_RESID && a.parts_out) *a.parts_out = ks;
  return PD_OK;
}

template <int RT, int EPI, bool SPLIT, bool PACK>
static int launch_gemm_small(const GemmArgs &a, hipStream_t s) {
  int KT = a.K / 32, ks = 1;
  if (EPI == EPI_RESID)    // slices while the launch has fewer than 256 blocks and a slice keeps 8 k-tiles
    while (ks < a.max_parts && ((a.n_tiles + 1) / 2) * ks < 256 && KT / (2 * ks) >= 8) ks *= 2;
  if (RT == 1 && ((a.n_tiles + 1) / 2) * ks >= 128) return launch_gemm_small_nt<RT, 2, EPI, SPLIT, PACK>(a, ks, s);
  return launch_gemm_small_nt<RT, 1, EPI, SPLIT, PACK>(a, ks, s);
}

// 2, 4, 5 or 8 row tiles (many rows per request, many requests at once, prefill chunks).  Here the activation fragments of a
// block (32-128 rows x K, high and low parts) outweigh its weights, every block has to request all
// of them, and a compute unit's vector-memory pipeline is the limit, so what counts is how many
// requests the busiest compute unit issues: rounds of 256 blocks x k-tiles per block x (NT weight
// + 2 RT activation requests per k-tile).  The launch takes the column tiles per wave NT (and, for
// the residual projections, the K slices over blocks) that minimise this count -- typically the
// pair that makes exactly 256 blocks, one per compute unit: measured 29 us against 42 us for the
// QKV projection of cfg5 with 256 instead of 384 blocks.  Blocks are 4 waves along K (one wave per
// SIMD: registers for up to 8 x 4 accumulator tiles) and keep the compute unit to themselves.
template <int RT, int NT, int EPI, bool SPLIT>
static int launch_gemm_wide_nt(GemmArgs a, int ks, hipStream_t s) {
  constexpr int NWK = 4;
  constexpr int U = (NT + 2 * RT) <= 16 ? 4 : 2;
  int KT = a.K / 32, groups = (a.n_tiles + NT - 1) / NT;
  a.k_share = ((KT + ks - 1) / ks + NWK - 1) / NWK;
  if (a.stream_w)
    hipLaunchKernelGGL((k_gemm_s<RT, NT, NWK, U, EPI, SPLIT, false, false, true>), dim3(groups, ks), dim3(64 * NWK), 0, s, a);
  else
    hipLaunchKernelGGL((k_gemm_s<RT, NT, NWK, U, EPI, SPLIT, false>), dim3(groups, ks), dim3(64 * NWK), 0, s, a);
  PD_CHECK_HIP(hipGetLastError());
  if (EPI == EPI_RESID && a.parts_out) *a.parts_out = ks;
  return PD_OK;
}

template <int RT, int EPI, bool SPLIT>
static int launch_gemm_wide(const GemmArgs &a, hipStream_t s) {
  // 4 * NT * RT KiB of LDS, at most 128-160; with 2 row tiles more than 4 column tiles measured slower
  // (7 only with 5 row tiles: the vocabulary projection of a 72-row step then makes 449 blocks, two rounds
  // of one block per compute unit, instead of 524 with 6, where 12 blocks run a third round alone)
  constexpr int NT_MAX = RT <= 2 ? 4 : (RT <= 4 ? 8 : (RT == 5 ? 7 : 4));
  static const int nts[] = {1, 2, 3, 4, 6, 7, 8};
  int KT = a.K / 32, best_nt = 1, best_ks = 1;
  long best = -1;
  for (int ks = 1; ks <= (EPI == EPI_RESID ? a.max_parts : 1); ks *= 2) {
    if (ks > 1 && KT / ks < 8) break;
    for (int nt : nts) {
      if (nt > NT_MAX) break;
      if (nt == 7 && RT != 5) continue;
      long blocks = (long)((a.n_tiles + nt - 1) / nt) * ks;
      long rounds = (blocks + 255) / 256;
      long cost = rounds * ((KT + ks - 1) / ks) * (nt + 2 * RT);
      if (best < 0 || cost < best) { best = cost; best_nt = nt; best_ks = ks; }
    }
  }
  switch (best_nt) {
    case 1: return launch_gemm_wide_nt<RT, 1, EPI, SPLIT>(a, best_ks, s);
    case 2: return launch_gemm_wide_nt<RT, 2, EPI, SPLIT>(a, best_ks, s);
    case 3: return launch_gemm_wide_nt<RT, 3, EPI, SPLIT>(a, best_ks, s);
    case 4: return launch_gemm_wide_nt<RT, 4, EPI, SPLIT>(a, best_ks, s);
    case 6: return launch_gemm_wide_nt<RT, (NT_MAX >= 6 ? 6 : NT_MAX), EPI, SPLIT>(a, best_ks, s);
    case 7: return launch_gemm_wide_nt<RT, (RT == 5 ? 7 : 1), EPI, SPLIT>(a, best_ks, s);
    default: return launch_gemm_wide_nt<RT, (NT_MAX >= 8 ? 8 : NT_MAX), EPI, SPLIT>(a, best_ks, s);
  }
}


// ---------------------------------------------------------------------------
// More than 128 rows (the context pass in chunks of up to 2048 rows): grid (column groups, K slices,
// groups of 128 rows).  A block is NW = 8 waves (two per SIMD: a single wave issues a 16x16x32
// multiply every 29 clocks, two or more every 19) that own NT column tiles each and share the 8 row
// tiles of their row group: per k-tile every wave requests its share of the activation fragments
// (high and low parts) and its own weight fragments, D k-tiles ahead, the activation fragments pass
// through LDS (two buffers of 16 KiB), and every wave multiplies all of them with its weights.  A
// k-tile then costs the compute unit 16 + 8 NT requests for 128 NT multiplies, against 16 + NT for
// 16 NT when the waves cut K instead.
// Measured (useful rate; twice that is executed with the low parts): QKV of cfg5 with 2048 rows
// 320 us = 0.64 PFLOP/s with NT = 3 (512 blocks), gate + up 608 us = 0.61; QKV of cfg4 with 4096 rows
// 177 us = 0.58 PFLOP/s.  An earlier version with 4 waves per block and twice the column tiles per
// wave took nearly twice the time of the 8-wave version of its day.
// ---------------------------------------------------------------------------
template <int NT, int D, int OCC, int EPI, bool SPLIT, int NW = 4, int TAG = 0>
__global__ __launch_bounds__(64 * NW, OCC) void k_gemm_p(GemmArgs a) {
  static_assert(NW == 4 || NW == 8, "4 or 8 waves");
  constexpr int RT = 8, NA = SPLIT ? 2 * RT : RT, NAW = NA / NW;   // fragments per k-tile: all / staged by one wave
  static_assert(D % 2 == 0 || D == 1, "stages alternate between the two LDS buffers");
  __shared__ bf16x8 sm_x[2][NA][64];   // (vector types throughout: struct copies would keep xr in scratch memory)
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  const int m = lane & 15;
  const int KT = a.K >> 5;
  const int per_slice = (KT + (int)gridDim.y - 1) / (int)gridDim.y;
  const int kt0 = min((int)blockIdx.y * per_slice, KT), kt1 = min(kt0 + per_slice, KT);
  const int rt0 = blockIdx.z * RT, r0 = rt0 * 16;
  int4 kvi[(EPI == EPI_QKV || EPI == EPI_QKV_ROPE || EPI == EPI_QKV_NORM) ? RT : 1];
  if (EPI == EPI_QKV || EPI == EPI_QKV_ROPE || EPI == EPI_QKV_NORM) {
#pragma unroll
    for (int i = 0; i < RT; ++i) kvi[i] = a.rt.kvinfo[r0 + i * 16 + m];
  }
  const int nt0 = (blockIdx.x * NW + w) * NT;
  int tile[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) tile[t] = min(nt0 + t, a.n_tiles - 1);   // tiles past the end repeat the last one
  floatx4 acc[NT][RT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int i = 0; i < RT; ++i) acc[t][i] = floatx4{0.f, 0.f, 0.f, 0.f};
  const uint4 *wp = (const uint4 *)a.W + lane;
  // this wave's share of the activation fragments: fragment f = w * NAW + j is row tile f % RT of
  // the high (f < RT) or low parts
  const bf16x8 *xsrc[NAW];
#pragma unroll
  for (int j = 0; j < NAW; ++j) {
    int f = w * NAW + j;
    const bf16_t *base = (SPLIT && f >= RT) ? a.xn_lo : a.xn;
    xsrc[j] = (const bf16x8 *)base + (size_t)(rt0 + f % RT) * KT * 64 + lane;
  }
  // D k-tiles are in flight per wave, each in registers of its own (slot = k-tile index mod D)
  Frag xr[D][NAW];
  Frag wr[D][NT];
  const int len = kt1 - kt0;
  auto k_of = [&](int j) { return kt0 + min(j, len - 1); };   // steps past the end repeat the last k-tile
#pragma unroll
  for (int d = 0; d < D; ++d) {
    int k = len > 0 ? k_of(d) : 0;
#pragma unroll
    for (int j = 0; j < NAW; ++j) xr[d][j].v = xsrc[j][(size_t)k * 64];
#pragma unroll
    for (int t = 0; t < NT; ++t) wr[d][t].u = wp[((size_t)tile[t] * KT + k) * 64];
  }
  for (int j0 = 0; j0 < len; j0 += D) {
#pragma unroll
    for (int d = 0; d < D; ++d) {
      if (j0 + d < len) {           // the same for every wave of the block
        const int buf = D == 1 ? (j0 & 1) : (d & 1);
        Frag wc[NT];
#pragma unroll
        for (int j = 0; j < NAW; ++j) sm_x[buf][w * NAW + j][lane] = xr[d][j].v;
#pragma unroll
        for (int t = 0; t < NT; ++t) wc[t] = wr[d][t];
        {                           // refill the slot with the k-tile D further on
          int k = k_of(j0 + d + D);
#pragma unroll
          for (int j = 0; j < NAW; ++j) xr[d][j].v = xsrc[j][(size_t)k * 64];
#pragma unroll
          for (int t = 0; t < NT; ++t) wr[d][t].u = wp[((size_t)tile[t] * KT + k) * 64];
        }
        // one barrier per k-tile is enough with two buffers: a wave can only write k-tile i + 2 into
        // this buffer after the barrier of k-tile i + 1, which every wave reaches after its reads of i
        __syncthreads();
        // The k-tile's fragments pass from LDS to the matrix cores in groups of GS (fragment f: row tile
        // f % RT, high parts first): two groups are requested up front, and while one group is multiplied
        // the next but one is requested into the registers of the group before it.  A wave then holds 2 GS
        // fragments instead of all NA (which, with the accumulators and the weights in flight, did not fit
        // the 256 registers of a wave at two waves per SIMD), and its LDS reads run under its multiplies.
        // Products into the same accumulator (high and low part of a row tile) are NT * RT multiplies apart.
        constexpr int GS = 4, NG = NA / GS;
        Frag xg[2][GS];
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int u = 0; u < GS; ++u) xg[h][u].v = sm_x[buf][h * GS + u][lane];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
#pragma unroll
          for (int u = 0; u < GS; ++u)
#pragma unroll
            for (int t = 0; t < NT; ++t)
              acc[t][(gi * GS + u) % RT] = mfma16(wc[t], xg[gi & 1][u], acc[t][(gi * GS + u) % RT]);
          __builtin_amdgcn_sched_barrier(0);
          if (gi + 2 < NG) {
#pragma unroll
            for (int u = 0; u < GS; ++u) xg[gi & 1][u].v = sm_x[buf][(gi + 2) * GS + u][lane];
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
    }
  }
#pragma unroll
  for (int t = 0; t < NT; ++t)
    if (nt0 + t < a.n_tiles) gemm_epilogue<RT, EPI>(a, nt0 + t, acc[t], kvi, lane, r0);
}

template <int NT, int EPI, bool SPLIT>
static int launch_gemm_rows_nt(GemmArgs a, int rows, hipStream_t s) {
  constexpr int NW = 8;
  int KT = a.K / 32, gx = (a.n_tiles + NW * NT - 1) / (NW * NT), gz = (rows + 127) / 128, ks = 1;
  if (EPI == EPI_RESID)     // K slices (summed by the next norm kernel) while compute units would stay empty
    while (ks < a.max_parts && (long)gx * gz * ks < 256 && KT / (2 * ks) >= 8) ks *= 2;
  hipLaunchKernelGGL((k_gemm_p<NT, 2, 1, EPI, SPLIT, NW>), dim3(gx, ks, gz), dim3(64 * NW), 0, s, a);
  PD_CHECK_HIP(hipGetLastError());
  if (EPI == EPI_RESID && a.parts_out) *a.parts_out = ks;
  return PD_OK;
}

// Column tiles per wave (2, 3 or 4; blocks of 8 waves, one block per compute unit): what finishes
// first by the measured time of a block per k-tile (1.03 / 1.39 / 1.93 us: close to proportional, the
// matrix cores set the pace; QKV and FFN1 shapes of cfg4 in chunks of 4096 rows) times the rounds of
// 256 blocks the launch needs.
template <int EPI, bool SPLIT>
static int launch_gemm_rows(const GemmArgs &a, int rows, hipStream_t s) {
  auto cost = [&](int nt, double t) {
    long b = (long)((a.n_tiles + 8 * nt - 1) / (8 * nt)) * ((rows + 127) / 128);
    if (EPI == EPI_RESID) {     // the K slices launch_gemm_rows_nt will choose
      int KT = a.K / 32, ks = 1;
      while (ks < a.max_parts && b * ks < 256 && KT / (2 * ks) >= 8) ks *= 2;
      return (double)((b * ks + 255) / 256) * t / ks;
    }
    return (double)((b + 255) / 256) * t;
  };
  double c2 = cost(2, 1.03), c3 = cost(3, 1.39), c4 = cost(4, 1.93);
  if (c4 <= c3 && c4 <= c2) return launch_gemm_rows_nt<4, EPI, SPLIT>(a, rows, s);
  if (c3 <= c2) return launch_gemm_rows_nt<3, EPI, SPLIT>(a, rows, s);
  return launch_gemm_rows_nt<2, EPI, SPLIT>(a, rows, s);
}

// 17-128 rows against a small weight matrix (at most 16 MB: what the L2 caches hold with room to spare).  One
// row tile and four column tiles per block instead of all row tiles and one column tile: a k-tile then costs a
// wave 4 weight + 2 activation requests for 4 output tiles, not 1 + 2 RT for RT, so the busiest compute unit
// issues about half the requests (its vector-memory pipeline is what bounds these launches), all requests
// of a wave go out in one batch, and 5 x 48 blocks fill the chip where 192 did not.  The weights are read
// once per row tile; block ids that differ by a multiple of 8 run on the same XCD (work-groups go to the
// XCDs round-robin), so with a number of column groups that is a multiple of 8 the row tiles of a group
// share one L2 and the repeats stay out of HBM.  Measured at 72 rows, width 1024 (cfg3): QKV 10.9 -> 6.9 us, first
// FFN projection 11.5 -> 9.5, output projection 4.0 (K slices of 8 k-tiles), second FFN projection 8.4 -> 7.7;
// 0.83 -> 0.76 ms per step.
// A projection that completes the residual rows and prepares the next norm (never cut along K over blocks)
// takes one column tile per block, so that the launch still has a block per compute unit: 64 x 5 at width 1024.
template <int EPI, bool SPLIT, int NT = 4>
static int launch_gemm_zrows(GemmArgs a, int rows, hipStream_t s) {
  constexpr int U = 4;
  const int KT = a.K / 32, groups = (a.n_tiles + NT - 1) / NT, rts = (rows + 15) / 16;
  // the residual projections also cut K into slices over blocks (summed by the next norm kernel) until the
  // launch has a block per compute unit
  int ks = 1;
  if (EPI == EPI_RESID)
    while (ks < a.max_parts && groups * rts * ks < 256 && KT / (2 * ks) >= 4) ks *= 2;
  const int per_block = (KT + ks - 1) / ks;
  // 4 or 8 waves along K (16 would leave a wave 128 registers, too few for 4 x 4 weight fragments in flight):
  // one batch of 4 k-tiles per wave up to K = 1024 per slice, two up to 2048.  A block of 8 waves has a compute
  // unit to itself; a launch of more than 256 blocks therefore takes 4 waves per block (two batches per wave),
  // so that all its blocks are resident at once instead of a few left over for a second round (320 blocks at
  // width 1024, 72 rows: first FFN projection 10.3 -> 9.3 us, second 8.1 -> 7.7)
  const int nwk = (per_block > 16 && (per_block > 64 || (long)groups * ks * rts <= 256)) ? 8 : 4;
  a.k_share = (per_block + nwk - 1) / nwk;
  dim3 grid(groups, ks, rts);
  if (nwk == 4) hipLaunchKernelGGL((k_gemm_s<1, NT, 4, U, EPI, SPLIT, false, true>), grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL((k_gemm_s<1, NT, 8, U, EPI, SPLIT, false, true>), grid, dim3(512), 0, s, a);
  PD_CHECK_HIP(hipGetLastError());
  if (EPI == EPI_RESID && a.parts_out) *a.parts_out = ks;
  return PD_OK;
}

template <int EPI, bool SPLIT>
static int launch_gemm_split(const GemmArgs &a, int rows, hipStream_t s) {
  constexpr bool zrows = EPI != EPI_LM;
  if (zrows && mfma_gemm_row_tile_blocks(a.n_tiles, a.K, rows, EPI == EPI_RESID ? a.max_parts : 1))
    return launch_gemm_zrows<EPI, SPLIT, (EPI == EPI_RESID_NORM ? 1 : 4)>(a, rows, s);
  if (EPI == EPI_RESID_NORM || EPI == EPI_QKV_NORM)
    PD_REQUIRE(rows <= 16, PD_EINVAL, "a projection of this shape cannot prepare or finish a norm for %d rows", rows);
  switch (mfma_gemm_row_tiles(rows)) {
    case 16: return launch_gemm_small<1, EPI, SPLIT, false>(a, s);
    case 32: return launch_gemm_wide<2, EPI, SPLIT>(a, s);
    case 64: return launch_gemm_wide<4, EPI, SPLIT>(a, s);
    case 80: return launch_gemm_wide<5, EPI, SPLIT>(a, s);
    default: return launch_gemm_wide<8, EPI, SPLIT>(a, s);
  }
}

template <int EPI>
static int launch_gemm(const GemmArgs &a, int rows, hipStream_t s) {
  if (EPI == EPI_RESID_NORM || EPI == EPI_QKV_NORM)
    PD_REQUIRE(rows <= 128 && a.R <= 128, PD_EINVAL,
               "projections that prepare or finish a norm take at most 128 rows (%d)", rows);
  if (rows > 128) {
    PD_REQUIRE(!a.packed, PD_EINVAL, "packed activations hold at most 8 rows (%d)", rows);
    return a.xn_lo ? launch_gemm_rows<EPI, true>(a, rows, s) : launch_gemm_rows<EPI, false>(a, rows, s);
  }
  if (a.packed) {
    PD_REQUIRE(rows <= 8 && a.R <= 8, PD_EINVAL, "packed activations hold at most 8 rows (%d)", rows);
    return launch_gemm_small<1, EPI, false, true>(a, s);
  }
  return a.xn_lo ? launch_gemm_split<EPI, true>(a, rows, s) : launch_gemm_split<EPI, false>(a, rows, s);
}

// one translation unit per epilogue
int PD_GEMM_ENTRY(const GemmArgs &a, int rows, hipStream_t s) { return launch_gemm<PD_GEMM_EPI>(a, rows, s); }

#else   // ---- common part: dispatcher ----------------------------------------------------------

// 17-128 rows against a weight matrix of at most 16 MB (17-32 rows: 64 MB; the blocks of both row tiles are then
// resident together and the second reader of a weight line finds it in L2) and a K that 8 waves (times the K
// slices over blocks) cover in batches of 4 k-tiles: the launch gives every row tile blocks of its own
// (launch_gemm_zrows)
bool mfma_gemm_row_tile_blocks(int n_tiles, int K, int rows, int k_slices) {
  const size_t bytes = (size_t)n_tiles * 16 * K * 2;
  return rows > 16 && rows <= 128 && (bytes <= ((size_t)16 << 20) || (rows <= 32 && bytes <= ((size_t)64 << 20))) && K / 32 <= 64 * k_slices;
}

int mfma_gemm_row_tiles(int rows) {
  int rt = (rows + 15) / 16;
  return (rt <= 1 ? 1 : rt <= 2 ? 2 : rt <= 4 ? 4 : rt <= 5 ? 5 : 8) * 16;
}

int mfma_gemm_epi0(const GemmArgs &a, int rows, hipStream_t s);
int mfma_gemm_epi1(const GemmArgs &a, int rows, hipStream_t s);
int mfma_gemm_epi2(const GemmArgs &a, int rows, hipStream_t s);
int mfma_gemm_epi3(const GemmArgs &a, int rows, hipStream_t s);
int mfma_gemm_epi4(const GemmArgs &a, int rows, hipStream_t s);
int mfma_gemm_epi5(const GemmArgs &a, int rows, hipStream_t s);
int mfma_gemm_epi6(const GemmArgs &a, int rows, hipStream_t s);
int mfma_gemm_epi7(const GemmArgs &a, int rows, hipStream_t s);

int mfma_gemm(int epi, const GemmArgs &a, int rows, hipStream_t s) {
  switch (epi) {
    case EPI_QKV: return mfma_gemm_epi0(a, rows, s);
    case EPI_QKV_ROPE: return mfma_gemm_epi1(a, rows, s);
    case EPI_RESID: return mfma_gemm_epi2(a, rows, s);
    case EPI_GELU: return mfma_gemm_epi3(a, rows, s);
    case EPI_SWIGLU: return mfma_gemm_epi4(a, rows, s);
    case EPI_LM: return mfma_gemm_epi5(a, rows, s);
    case EPI_RESID_NORM: return mfma_gemm_epi6(a, rows, s);
    case EPI_QKV_NORM: return mfma_gemm_epi7(a, rows, s);
  }
  pd_set_error("unknown epilogue %d", epi);
  return PD_EINVAL;
}

#endif
