// fp32-activation kernels: one straightforward kernel per operation.
// They serve dtype 0 (fp32 weights and KV cache) and, for bf16 weights whose
// shapes the MFMA kernels do not cover, dtype 1 with fp32 activations.
// KV cache layout on this path: K and V each [B][H][kv_cap][hd], row-major.
#include "pd_internal.h"

// ---------------------------------------------------------------------------
// norm: xn[r] = LayerNorm(x[r]) or RMSNorm(x[r]); one block per row
// ---------------------------------------------------------------------------
__device__ __forceinline__ float block_sum(float v, float *sh) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += sh[i];
  return t;
}

__global__ void k_norm_f32(float *xn, const float *x, const float *g, const float *b, int d,
                           int kind, float eps, const int32_t *flags) {
  __shared__ float sh[16];
  int r = blockIdx.x;
  if (!(flags[r] & ROW_VALID)) return;
  const float *xr = x + (size_t)r * d;
  float s = 0.f;
  for (int c = threadIdx.x; c < d; c += blockDim.x) s += xr[c];
  float mean = kind == 0 ? block_sum(s, sh) / d : 0.f;
  float v = 0.f;
  for (int c = threadIdx.x; c < d; c += blockDim.x) { float t = xr[c] - mean; v += t * t; }
  float rstd = rsqrtf(block_sum(v, sh) / d + eps);
  for (int c = threadIdx.x; c < d; c += blockDim.x) {
    float t = (xr[c] - mean) * rstd * g[c];
    if (kind == 0 && b) t += b[c];
    xn[(size_t)r * d + c] = t;
  }
}

// ---------------------------------------------------------------------------
// linear: y[r][n] = sum_k x[r][k] * W[n][k].  One wave per output column and
// tile of 8 rows; lanes stride over k (coalesced weight reads).
//   EPI 0: out = y            EPI 1: out = res + y
//   EPI 2: out = gelu_erf(y)  EPI 3: out = silu(y) * (x . W2[n])
// ---------------------------------------------------------------------------
template <typename WT, int EPI>
__global__ void k_linear(float *out, const float *x, const WT *W, const WT *W2, const float *res,
                         int R, int N, int K, int ldo) {
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  int n = blockIdx.x * (blockDim.x >> 6) + wave;
  int r0 = blockIdx.y * 8;
  if (n >= N) return;
  float acc[8], acc2[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) { acc[i] = 0.f; acc2[i] = 0.f; }
  const WT *w = W + (size_t)n * K;
  const WT *w2 = EPI == 3 ? W2 + (size_t)n * K : nullptr;
  for (int k = lane; k < K; k += 64) {
    float wv = ld_f32(w, k);
    float wv2 = EPI == 3 ? ld_f32(w2, k) : 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int r = r0 + i;
      float xv = r < R ? x[(size_t)r * K + k] : 0.f;
      acc[i] = fmaf(wv, xv, acc[i]);
      if (EPI == 3) acc2[i] = fmaf(wv2, xv, acc2[i]);
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    for (int o = 32; o > 0; o >>= 1) {
      acc[i] += __shfl_xor(acc[i], o);
      if (EPI == 3) acc2[i] += __shfl_xor(acc2[i], o);
    }
  }
  if (lane == 0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int r = r0 + i;
      if (r >= R) break;
      float y = acc[i];
      if (EPI == 1) y += res[(size_t)r * ldo + n];
      if (EPI == 2) y = 0.5f * y * (1.f + erff(y * 0.70710678118654752f));
      if (EPI == 3) y = y / (1.f + expf(-y)) * acc2[i];
      out[(size_t)r * ldo + n] = y;
    }
  }
}

template <typename WT, int EPI>
static int run_linear(float *out, const float *x, const void *W, const void *W2, const float *res,
                      int R, int N, int K, hipStream_t s) {
  dim3 grid((N + 3) / 4, (R + 7) / 8);
  hipLaunchKernelGGL((k_linear<WT, EPI>), grid, dim3(256), 0, s, out, x, (const WT *)W,
                     (const WT *)W2, res, R, N, K, N);
  PD_CHECK_HIP(hipGetLastError());
  return PD_OK;
}

template <int EPI>
static int linear(pd_ctx *c, float *out, const float *x, const void *W, const void *W2,
                  const float *res, int R, int N, int K, hipStream_t s) {
  return c->cfg.dtype == 0 ? run_linear<float, EPI>(out, x, W, W2, res, R, N, K, s)
                           : run_linear<bf16_t, EPI>(out, x, W, W2, res, R, N, K, s);
}

// ---------------------------------------------------------------------------
// rotary + KV append: q (in place) and k rotated by the row's position; k, v
// written to the row's slot of the request's cache.
// ---------------------------------------------------------------------------
template <typename KT>
__global__ void k_qkv_post(float *qkv, KT *kc, KT *vc, KT *kc_lo, KT *vc_lo, RowTables rt,
                           const float *rope_cs, int d, int H, int hd, int kv_cap, int32_t *kv_sat) {
  int r = blockIdx.x;
  if (!(rt.flags[r] & ROW_VALID)) return;
  float *row = qkv + (size_t)r * 3 * d;
  int half = hd / 2;
  size_t base = (size_t)rt.req[r] * H * kv_cap * hd + (size_t)rt.slot[r] * hd;
  const float *cs = rope_cs ? rope_cs + (size_t)rt.pos[r] * half * 2 : nullptr;
  for (int i = threadIdx.x; i < H * half; i += blockDim.x) {
    int h = i / half, j = i % half;
    float q1 = row[h * hd + j], q2 = row[h * hd + j + half];
    float k1 = row[d + h * hd + j], k2 = row[d + h * hd + j + half];
    if (cs) {
      float cc = cs[2 * j], ss = cs[2 * j + 1];
      float a = q1 * cc - q2 * ss, b = q2 * cc + q1 * ss;
      q1 = a; q2 = b;
      a = k1 * cc - k2 * ss; b = k2 * cc + k1 * ss;
      k1 = a; k2 = b;
      row[h * hd + j] = q1; row[h * hd + j + half] = q2;
    }
    size_t o = base + (size_t)h * kv_cap * hd;
    float v1 = row[2 * d + h * hd + j], v2 = row[2 * d + h * hd + j + half];
    if (sizeof(KT) == 2) {   // half cache: count what is stored saturated
      int n_sat = (fabsf(k1) > 65504.f) + (fabsf(k2) > 65504.f) + (fabsf(v1) > 65504.f) + (fabsf(v2) > 65504.f);
      if (n_sat) atomicAdd(kv_sat, n_sat);
    }
    st_f32(kc, o + j, k1); st_f32(kc, o + j + half, k2);
    st_f32(vc, o + j, v1); st_f32(vc, o + j + half, v2);
    if (kc_lo) {      // low halves: what the rounding of the stores above left out
      st_f32(kc_lo, o + j, k1 - ld_f32(kc, o + j)); st_f32(kc_lo, o + j + half, k2 - ld_f32(kc, o + j + half));
      st_f32(vc_lo, o + j, v1 - ld_f32(vc, o + j)); st_f32(vc_lo, o + j + half, v2 - ld_f32(vc, o + j + half));
    }
  }
}

// ---------------------------------------------------------------------------
// attention: one block per (row, head).  Key j of the row's request is visible
// when j < lim[r] (context part) or when it is a generated-side slot (j >= L,
// j < kv_len) whose subsequence index is <= the row's (Section 3.2).
// Three passes over a score scratch in global memory.
// ---------------------------------------------------------------------------
template <typename KT>
__global__ void k_attn(float *out, const float *qkv, const KT *kc, const KT *vc, const KT *kc_lo,
                       const KT *vc_lo, float *scores,
                       RowTables rt, const int32_t *kv_len, const uint16_t *gen_sub, int kv_override,
                       int d, int H, int hd, int kv_cap, int gen_stride, int L, float scale) {
  extern __shared__ float sm[];     // q[hd] | red[16] | o[blockDim.x]
  float *qs = sm, *red = sm + hd, *osum = sm + hd + 16;
  int r = blockIdx.x, h = blockIdx.y;
  if (!(rt.flags[r] & ROW_VALID)) return;
  int req = rt.req[r], lim = rt.lim[r], sub = rt.sub[r];
  int n = kv_override >= 0 ? kv_override : kv_len[req];
  const KT *K = kc + ((size_t)req * H + h) * kv_cap * hd;
  const KT *V = vc + ((size_t)req * H + h) * kv_cap * hd;
  const KT *Kl = kc_lo ? kc_lo + ((size_t)req * H + h) * kv_cap * hd : nullptr;
  const KT *Vl = vc_lo ? vc_lo + ((size_t)req * H + h) * kv_cap * hd : nullptr;
  const uint16_t *gs = gen_sub + (size_t)req * gen_stride;
  const int L8 = L & ~7;            // entry of key slot j >= L is j - L8
  float *sc = scores + ((size_t)r * H + h) * kv_cap;
  for (int c = threadIdx.x; c < hd; c += blockDim.x) qs[c] = qkv[(size_t)r * 3 * d + h * hd + c];
  __syncthreads();
  float mx = -INFINITY;
  for (int j = threadIdx.x; j < n; j += blockDim.x) {
    bool vis = j < lim || (j >= L && (int)gs[j - L8] <= sub);
    float s = -INFINITY;
    if (vis) {
      s = 0.f;
      for (int c = 0; c < hd; ++c) {
        float kv = ld_f32(K, (size_t)j * hd + c);
        if (Kl) kv += ld_f32(Kl, (size_t)j * hd + c);
        s = fmaf(qs[c], kv, s);
      }
      s *= scale;
    }
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
  __syncthreads();
  for (int i = 0; i < (int)(blockDim.x >> 6); ++i) mx = fmaxf(mx, red[i]);
  float sum = 0.f;
  for (int j = threadIdx.x; j < n; j += blockDim.x) {
    float p = sc[j] == -INFINITY ? 0.f : expf(sc[j] - mx);
    sc[j] = p;
    sum += p;
  }
  sum = block_sum(sum, red);        // contains the barriers that publish sc[]
  // thread (g, c): channel c, keys g, g + G, ...
  int G = blockDim.x / hd, g = threadIdx.x / hd, c = threadIdx.x % hd;
  float acc = 0.f;
  if (g < G)
    for (int j = g; j < n; j += G) {
      float vv = ld_f32(V, (size_t)j * hd + c);
      if (Vl) vv += ld_f32(Vl, (size_t)j * hd + c);
      acc = fmaf(sc[j], vv, acc);
    }
  osum[threadIdx.x] = acc;
  __syncthreads();
  if (threadIdx.x < hd) {
    float t = 0.f;
    for (int i = 0; i < G; ++i) t += osum[i * hd + threadIdx.x];
    out[(size_t)r * d + h * hd + threadIdx.x] = t / sum;
  }
}

// ---------------------------------------------------------------------------
// argmax over a logits row, lowest index on ties; one block per row
// ---------------------------------------------------------------------------
__global__ void k_argmax(int32_t *row_argmax, const float *logits, const int32_t *flags, int V) {
  __shared__ float sv[256];
  __shared__ int si[256];
  int r = blockIdx.x;
  if (!(flags[r] & ROW_VALID)) return;
  const float *p = logits + (size_t)r * V;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int v = threadIdx.x; v < V; v += blockDim.x) {
    float x = p[v];
    if (x > best) { best = x; bi = v; }      // strided ascending scan keeps the lowest index
  }
  sv[threadIdx.x] = best; si[threadIdx.x] = bi;
  __syncthreads();
  for (int o = blockDim.x / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) {
      float ov = sv[threadIdx.x + o]; int oi = si[threadIdx.x + o];
      if (ov > sv[threadIdx.x] || (ov == sv[threadIdx.x] && oi < si[threadIdx.x])) {
        sv[threadIdx.x] = ov; si[threadIdx.x] = oi;
      }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) row_argmax[r] = si[0];
}

// ---------------------------------------------------------------------------
// one transformer layer / the head, as sequences of launches
// ---------------------------------------------------------------------------
int simple_layer(pd_ctx *c, int l, int R, int A, int nreq, int req0, int kv_override,
                 hipStream_t s) {
  (void)A; (void)nreq; (void)req0;
  const pd_config &g = c->cfg;
  const LayerPtrs &lw = c->layers[l];
  int d = g.d_model, ff = g.d_ff, H = g.n_head, hd = g.head_dim;
  float *xn = (float *)c->xn, *att = (float *)c->att, *hb = (float *)c->hb;
  int rc;
  hipLaunchKernelGGL(k_norm_f32, dim3(R), dim3(256), 0, s, xn, c->x, lw.n1g, lw.n1b, d, g.norm_kind,
                     g.norm_eps, c->rows.flags);
  PD_CHECK_HIP(hipGetLastError());
  if ((rc = linear<0>(c, c->qkv32, xn, lw.wqkv, nullptr, nullptr, R, 3 * d, d, s))) return rc;
  const float *cs = g.pos_kind == 1 ? c->rope_cs : nullptr;
  float scale = 1.0f / sqrtf((float)hd);
  size_t shm = (hd + 16 + 256) * sizeof(float);
  // context pass, last layer: only its keys and values are ever used
  const bool kv_only = kv_override >= 0 && l == g.n_layer - 1;
  if (g.dtype == 0) {
    hipLaunchKernelGGL(k_qkv_post<float>, dim3(R), dim3(256), 0, s, c->qkv32, (float *)lw.kc,
                       (float *)lw.vc, (float *)nullptr, (float *)nullptr, c->rows, cs, d, H, hd,
                       c->kv_cap, c->kv_sat);
    if (!kv_only) hipLaunchKernelGGL(k_attn<float>, dim3(R, H), dim3(256), shm, s, att, c->qkv32,
                       (const float *)lw.kc, (const float *)lw.vc, (const float *)nullptr,
                       (const float *)nullptr, c->scores, c->rows,
                       c->sch.kv_len, c->sch.gen_sub, kv_override, d, H, hd, c->kv_cap, c->gen_stride,
                       c->L, scale);
  } else {
    hipLaunchKernelGGL(k_qkv_post<f16_t>, dim3(R), dim3(256), 0, s, c->qkv32, (f16_t *)lw.kc,
                       (f16_t *)lw.vc, (f16_t *)lw.kc_lo, (f16_t *)lw.vc_lo, c->rows, cs, d, H, hd,
                       c->kv_cap, c->kv_sat);
    if (!kv_only) hipLaunchKernelGGL(k_attn<f16_t>, dim3(R, H), dim3(256), shm, s, att, c->qkv32,
                       (const f16_t *)lw.kc, (const f16_t *)lw.vc, (const f16_t *)lw.kc_lo,
                       (const f16_t *)lw.vc_lo, c->scores, c->rows,
                       c->sch.kv_len, c->sch.gen_sub, kv_override, d, H, hd, c->kv_cap, c->gen_stride,
                       c->L, scale);
  }
  PD_CHECK_HIP(hipGetLastError());
  if (kv_only) return PD_OK;
  if ((rc = linear<1>(c, c->x, att, lw.wo, nullptr, c->x, R, d, d, s))) return rc;
  hipLaunchKernelGGL(k_norm_f32, dim3(R), dim3(256), 0, s, xn, c->x, lw.n2g, lw.n2b, d, g.norm_kind,
                     g.norm_eps, c->rows.flags);
  PD_CHECK_HIP(hipGetLastError());
  if (g.ffn_kind == 0) {
    if ((rc = linear<2>(c, hb, xn, lw.w1, nullptr, nullptr, R, ff, d, s))) return rc;
  } else {
    if ((rc = linear<3>(c, hb, xn, lw.w1, lw.w_up, nullptr, R, ff, d, s))) return rc;
  }
  return linear<1>(c, c->x, hb, lw.w2, nullptr, c->x, R, d, ff, s);
}

int simple_head(pd_ctx *c, int R, hipStream_t s) {
  const pd_config &g = c->cfg;
  int rc;
  hipLaunchKernelGGL(k_norm_f32, dim3(R), dim3(256), 0, s, (float *)c->xn, c->x, c->fng, c->fnb,
                     g.d_model, g.norm_kind, g.norm_eps, c->rows.flags);
  PD_CHECK_HIP(hipGetLastError());
  if ((rc = linear<0>(c, c->logits, (float *)c->xn, c->lm_head, nullptr, nullptr, R, g.vocab,
                      g.d_model, s)))
    return rc;
  hipLaunchKernelGGL(k_argmax, dim3(R), dim3(256), 0, s, c->row_argmax, c->logits, c->rows.flags,
                     g.vocab);
  PD_CHECK_HIP(hipGetLastError());
  return PD_OK;
}
