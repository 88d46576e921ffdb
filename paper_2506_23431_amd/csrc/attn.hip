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

#include <hip/hip_ext.h>

#include <algorithm>

struct AttnArgs {
  const f16_t *q, *q_lo;    // [rows][d] fp16 high / low parts (q_lo NULL: high part only)
  const f16_t *kc, *vc;     // packed fp16 caches of this layer
  const f16_t *kc_lo, *vc_lo;   // low halves of the same layout (PAIR kernels only)
  bf16_t *out, *out_lo;     // [rows][d] high / low parts (out_lo NULL: high part only)
  RowTables rt;
  const int32_t *kv_len;
  const uint16_t *gen_sub;  // subsequence tag of key slot j >= L at [req][j - (L & ~7)]
  int kv_override;          // >= 0: number of keys to consider (prefill), else kv_len[req]
  float *part;
  int d, H, kv_cap, gen_stride, L, A, nqg, req0, nsplit, nblk_static;
  float scale_log2;         // log2(e) / sqrt(hd)
  // BIAS kernels: every key slot j carries a grid coordinate, coord[req * coord_req_stride + j - coord_off]
  // = (tau - 1) + (i - 1) for a generated-side token (the encoder: its position), and a query has
  // c_q = pos[r] - pos0.
  //  * relative-position bias of the encoder-decoder form (Section 4.3): the score gets
  //    bias[h][clamp(c_q - coord[j] + bias_off, 0, bias_len - 1)] (already times log2(e));
  //  * a generated-side key is visible only if it is not later than the query, tau_k <= tau_q, beside
  //    the subsequence rule.  In a decode step that holds for every key in the cache; in the one-pass
  //    teacher-forced forward (Fig. 3b) all of the target's keys are there at once and this is the
  //    time half of the matrix.  tau - 2 = coordinate - subsequence tag on both sides.
  const float *bias; const uint16_t *coord;
  int bias_len, bias_off, coord_stride, coord_req_stride, coord_off, pos0;
};
constexpr int BIAS_MAX = 264;   // entries of one head's bias table that the kernel keeps in LDS

// PAIR: the layer keeps keys and values as high + low halves.  Scores add q_hi K_lo (q_lo K_lo is
// below the rounding of everything else), outputs add P V_lo; the kernel holds twice the fragments
// and is built for one block per compute unit.
// STREAM: keys and values are loaded with the non-temporal hint.  In a decode step every key/value byte is read
// once per launch and nothing reads it again before the caches have turned over, so keeping it out of the
// caches' way pays (cfg4: 15.9 -> 15.0 us per launch, cfg5: 60.5 -> 52.8); in the context pass the 16-query
// groups of a chunk re-read the same keys from L2, and there the hint costs a third of the pass.
template <bool STREAM>
__device__ __forceinline__ f16x8 ld_kv(const uint4 *p) {
  return STREAM ? __builtin_nontemporal_load((const f16x8 *)p) : *(const f16x8 *)p;
}

template <int HD, bool SPLIT, bool PAIR, bool BIAS = false, bool STREAM = false>
__global__ __launch_bounds__(256, PAIR ? 1 : 3) void k_attn_mfma(AttnArgs a) {
  constexpr int NC = HD / 32, NHB = HD / 16, PSTR = HD + 2;   // partial: m, l, O[HD] per query
  __shared__ float sm_m[4][16], sm_l[4][16];
  __shared__ float sm_bias[BIAS ? BIAS_MAX : 1];
  __shared__ floatx4 sm_o[4][HD / 16][64];
  __shared__ uint4 sm_q[(SPLIT ? 2 : 1) * NC][64];
  int split = blockIdx.x, h = blockIdx.y, z = blockIdx.z;
  int reqi = z / a.nqg, qg = z % a.nqg, req = a.req0 + reqi;
  int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  int n = lane & 15, g = lane >> 4;

  // Everything the block needs to know about its queries is requested first (a few lines that sit
  // in the L2 cache), then the first key/value block; no load below depends on the result of
  // another, and the wait for the row data does not wait for the key/value block behind it.
  int qa = qg * 16 + n;                       // query index inside the request
  bool in_req = qa < a.A;
  int r = reqi * a.A + (in_req ? qa : 0);     // row (clamped: loads stay in bounds)
  int4 qi = a.rt.qinfo[r];                    // {flags, sub, lim, req}
  int n_keys = a.kv_override >= 0 ? a.kv_override : a.kv_len[req];
  int q_pos = 0;
  float bias_pre[2] = {0.f, 0.f};
  if (BIAS) {
    q_pos = a.rt.pos[r] - a.pos0;
    bias_pre[0] = a.bias[(size_t)h * a.bias_len + min((int)threadIdx.x, a.bias_len - 1)];
    bias_pre[1] = a.bias[(size_t)h * a.bias_len + min((int)threadIdx.x + 256, a.bias_len - 1)];
  }
  // Query fragments (high and low parts) go to LDS, in operand order: the four waves share them,
  // and keeping them out of the registers leaves room for three waves per SIMD.  Rows without a
  // token keep whatever finite numbers their q slots hold: all their keys are masked below, and
  // their output is never written.
  const size_t q_off = act_off(r, h * HD + g * 8, a.d);
  constexpr int NQ = (NC + 3) / 4;            // fragments per wave
  uint4 qh[NQ], qlo[SPLIT ? NQ : 1];
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    int c = min(wave + 4 * i, NC - 1);
    size_t off = q_off + (size_t)c * 512;     // the next 32 dims are the next fragment
    qh[i] = *(const uint4 *)(a.q + off);
    if (SPLIT) qlo[i] = *(const uint4 *)(a.q_lo + off);
  }

  const uint4 *Kp = (const uint4 *)(a.kc + ((size_t)req * a.H + h) * a.kv_cap * HD) + lane;
  const uint4 *Vp = (const uint4 *)(a.vc + ((size_t)req * a.H + h) * a.kv_cap * HD) + lane;
  const uint4 *Kl = PAIR ? (const uint4 *)(a.kc_lo + ((size_t)req * a.H + h) * a.kv_cap * HD) + lane : nullptr;
  const uint4 *Vl = PAIR ? (const uint4 *)(a.vc_lo + ((size_t)req * a.H + h) * a.kv_cap * HD) + lane : nullptr;
  // subsequence tags of the generated-side slots, 8 keys (16 bytes) per lane group
  const uint16_t *gs = a.gen_sub + (size_t)req * a.gen_stride;
  const int L8 = a.L & ~7;
  // 32-key blocks are dealt round-robin to the 4*nsplit waves that serve this (request, head):
  // whatever the current key count, no wave gets more than one block above the average
  const int stride = 4 * a.nsplit;
  int kb = split * 4 + wave;
  Frag kf[2][NC], vf[NHB];
  Frag kl[PAIR ? 2 : 1][PAIR ? NC : 1], vl[PAIR ? NHB : 1];
  union { uint4 u; uint16_t s[8]; } tg, kco;
  const uint16_t *kcp = BIAS ? a.coord + (size_t)req * a.coord_req_stride : nullptr;
  auto load_k = [&](int kbx) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        kf[t][c].hv = ld_kv<STREAM>(&Kp[((size_t)(kbx * 2 + t) * NC + c) * 64]);
        if (PAIR) kl[t][c].hv = ld_kv<STREAM>(&Kl[((size_t)(kbx * 2 + t) * NC + c) * 64]);
      }
  };
  auto load_v = [&](int kbx) {
    // tags of the lane's 8 keys (clamped: context blocks read entry 0 and never use it)
    tg.u = *(const uint4 *)(gs + min(max(kbx * 32 + 8 * g - L8, 0), a.gen_stride - 8));
    if (BIAS) kco.u = *(const uint4 *)(kcp + min(max(kbx * 32 + 8 * g - a.coord_off, 0), a.coord_stride - 8));
#pragma unroll
    for (int i = 0; i < NHB; ++i) {
      vf[i].hv = ld_kv<STREAM>(&Vp[((size_t)kbx * NHB + i) * 64]);
      if (PAIR) vl[i].hv = ld_kv<STREAM>(&Vl[((size_t)kbx * NHB + i) * 64]);
    }
  };
  // requested unconditionally (a wave beyond the last block fetches that block and ignores it), so
  // that the wait for the query rows above never has to wait for these
  load_k(min(kb, a.nblk_static - 1));
  load_v(min(kb, a.nblk_static - 1));
  // (waves beyond the fragment count store a copy of the last fragment: same bytes, same place)
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    int c = min(wave + 4 * i, NC - 1);
    sm_q[c][lane] = qh[i];
    if (SPLIT) sm_q[NC + c][lane] = qlo[i];
  }
  if (BIAS) {
    sm_bias[threadIdx.x] = bias_pre[0];
    if (threadIdx.x + 256 < BIAS_MAX) sm_bias[threadIdx.x + 256] = bias_pre[1];
  }
  __syncthreads();

  bool qvalid = in_req && (qi.x & ROW_VALID);
  int q_sub = qvalid ? qi.y : -1, q_lim = qvalid ? qi.z : 0;
  // keys any query of this group can see
  int reach = qvalid ? (n_keys > a.L && q_sub >= 1 ? n_keys : min(q_lim, n_keys)) : 0;
  for (int o = 1; o < 16; o <<= 1) reach = max(reach, __shfl_xor(reach, o));
  const int end = __builtin_amdgcn_readfirstlane(min(a.nblk_static, (reach + 31) >> 5));
  // keys below lim_all are visible to every query of the group that has a token (the others are
  // never written, whatever they compute): blocks below it skip the per-key test
  int lim_q = qvalid ? min(q_lim, a.L) : 0x7fffffff;
  for (int o = 1; o < 16; o <<= 1) lim_q = min(lim_q, __shfl_xor(lim_q, o));
  const int lim_all = __builtin_amdgcn_readfirstlane(lim_q);

  float m_run = -INFINITY, l_run = 0.f;
  floatx4 o_acc[NHB];
#pragma unroll
  for (int i = 0; i < NHB; ++i) o_acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};

  // One block per wave is resident in registers.  The key fragments of the wave's next block are
  // requested as soon as the score products have consumed the current ones, the value fragments
  // (and tags) as soon as the output products have: the loads of block i+1 overlap the softmax
  // and the output products of block i without a second set of registers.
  while (kb < end) {
    floatx4 s[2] = {floatx4{0.f, 0.f, 0.f, 0.f}, floatx4{0.f, 0.f, 0.f, 0.f}};
    // the query fragments are re-read from LDS for every block (the empty asm keeps the compiler
    // from hoisting the reads out of the loop, which would put them back into 32 registers)
    int ql_lane = lane;
    asm volatile("" : "+v"(ql_lane));
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      Frag qf;
      qf.u = sm_q[c][ql_lane];
      s[0] = mfma16h(kf[0][c], qf, s[0]);
      s[1] = mfma16h(kf[1][c], qf, s[1]);
      if (PAIR) {
        s[0] = mfma16h(kl[0][c], qf, s[0]);
        s[1] = mfma16h(kl[1][c], qf, s[1]);
      }
      if (SPLIT) {
        qf.u = sm_q[NC + c][ql_lane];
        s[0] = mfma16h(kf[0][c], qf, s[0]);
        s[1] = mfma16h(kf[1][c], qf, s[1]);
      }
    }
    const int kn = kb + stride;
    const bool more = kn < end;
    if (more) load_k(kn);
    // lane (n, g), tile t, register j  <->  key kb*32 + 8g + 4t + j
    const int key0 = kb * 32 + 8 * g;
    float sv[8];
    float bv[8];
    if (BIAS) {
      const int q_off = q_pos + a.bias_off, last = a.bias_len - 1;
#pragma unroll
      for (int e = 0; e < 8; ++e) bv[e] = sm_bias[min(max(q_off - (int)kco.s[e], 0), last)];
    }
    if (kb * 32 + 32 <= lim_all) {
      // every query of the group sees the whole block (the same for all lanes of the wave)
#pragma unroll
      for (int e = 0; e < 8; ++e) sv[e] = BIAS ? s[e >> 2][e & 3] * a.scale_log2 + bv[e] : s[e >> 2][e & 3] * a.scale_log2;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        int key = key0 + e;
        bool vis = (key < q_lim) | ((key >= a.L) & (key < n_keys) & ((int)tg.s[e] <= q_sub) &
                                    (!BIAS || (int)kco.s[e] - (int)tg.s[e] <= q_pos - q_sub));
        sv[e] = vis ? (BIAS ? s[e >> 2][e & 3] * a.scale_log2 + bv[e] : s[e >> 2][e & 3] * a.scale_log2) : -INFINITY;
      }
    }
    float mloc = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
    mloc = fmaxf(mloc, __shfl_xor(mloc, 16));
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
    const float m_new = fmaxf(m_run, mloc);
    // while nothing is visible yet the reference is 0 instead of -inf: every exponential below is
    // then exp2(-inf) = 0 and never exp2(NaN)
    const float m_ref = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_ref);
    float p[8], psum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      p[e] = __builtin_amdgcn_exp2f(sv[e] - m_ref);
      psum += p[e];
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    // probabilities enter the matrix core as fp16 (the same 11 significant bits as the values they multiply)
    Frag pf, pl;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pf.hh[e] = (f16_t)p[e];
      if (PAIR) pl.hh[e] = (f16_t)(p[e] - (float)pf.hh[e]);
    }
    if (__any(alpha != 1.f)) {                // the running maximum of some query moved: rescale
#pragma unroll
      for (int i = 0; i < NHB; ++i) o_acc[i] *= alpha;
    }
#pragma unroll
    for (int i = 0; i < NHB; ++i) {
      o_acc[i] = mfma16h(vf[i], pf, o_acc[i]);
      if (PAIR) {
        o_acc[i] = mfma16h(vl[i], pf, o_acc[i]);
        o_acc[i] = mfma16h(vf[i], pl, o_acc[i]);
      }
    }
    if (more) load_v(kn);
    kb = kn;
  }
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);

  // ---- merge the 4 waves of the block (log-sum-exp) ----
  // every wave stores its accumulators as 16-byte quads (lane order: conflict-free); after the
  // barrier wave w owns the 16-dim blocks w, w + 4, ... and sums the four copies of each
  if (g == 0) { sm_m[wave][n] = m_run; sm_l[wave][n] = l_run; }
#pragma unroll
  for (int i = 0; i < NHB; ++i) sm_o[wave][i][lane] = o_acc[i];
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
  if (!qvalid) return;                        // lane (n, g) writes for query n only
  // partial of this block: m[16], l[16], then O as [dim / 4][query][4 dims]: a wave's store of one
  // 16-dim block is 1 KiB of consecutive bytes
  size_t unit = (size_t)z * a.H + h;
  float *pp = a.part + (unit * a.nsplit + split) * (size_t)(PSTR * 16);
  if (a.nsplit > 1 && wave == 0 && g == 0) { pp[n] = M; pp[16 + n] = lsum; }
  const float inv = 1.f / lsum;
  for (int i = wave; i < NHB; i += 4) {
    floatx4 o = fw[0] * sm_o[0][i][lane];
#pragma unroll
    for (int w = 1; w < 4; ++w) o += fw[w] * sm_o[w][i][lane];
    if (a.nsplit == 1) {
      float y[4] = {o[0] * inv, o[1] * inv, o[2] * inv, o[3] * inv};
      store4_split(a.out, a.out_lo, act_off(r, h * HD + i * 16 + 4 * g, a.d), y);
    } else {
      *(floatx4 *)(pp + 32 + ((i * 4 + g) * 16 + n) * 4) = o;
    }
  }
}

// Merge of the split partials by log-sum-exp.  Block = (unit, 16-dim block), 4 waves; wave w merges
// the splits w, w + 4, ... online (running max, sum and 4 output dims per lane), 8 splits' loads in
// flight at a time; the four running states are then combined through LDS.
template <int HD>
__global__ __launch_bounds__(256) void k_attn_merge(AttnArgs a) {
  constexpr int PSTR = HD + 2, U = 8;
  __shared__ float sm_M[4][64], sm_L[4][64];
  __shared__ floatx4 sm_O[4][64];
  int unit = blockIdx.x, i = blockIdx.y, z = unit / a.H, h = unit % a.H;
  int reqi = z / a.nqg, qg = z % a.nqg;
  int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 15, g = lane >> 4;
  int qa = qg * 16 + n, r = reqi * a.A + min(qa, a.A - 1);
  int fl = a.rt.flags[r];
  const size_t sstr = (size_t)PSTR * 16;
  const float *pb = a.part + (size_t)unit * a.nsplit * sstr;
  const int o_off = 32 + ((i * 4 + g) * 16 + n) * 4;
  float M = -INFINITY, l = 0.f;
  floatx4 o = floatx4{0.f, 0.f, 0.f, 0.f};
  for (int s0 = wave; s0 < a.nsplit; s0 += 4 * U) {
    float mv[U], lv[U];
    floatx4 ov[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float *ps = pb + (size_t)min(s0 + 4 * u, a.nsplit - 1) * sstr;   // clamped: masked below
      mv[u] = ps[n];
      lv[u] = ps[16 + n];
      ov[u] = *(const floatx4 *)(ps + o_off);
    }
    float Mn = M;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (s0 + 4 * u >= a.nsplit) mv[u] = -INFINITY;
      Mn = fmaxf(Mn, mv[u]);
    }
    if (Mn != -INFINITY) {
      float sc = exp2f(M - Mn);               // M == -inf: 0, and l, o are 0 anyway
      l *= sc; o *= sc;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float w = mv[u] == -INFINITY ? 0.f : exp2f(mv[u] - Mn);
        l += w * lv[u];
        o += w * ov[u];
      }
      M = Mn;
    }
  }
  sm_M[wave][lane] = M; sm_L[wave][lane] = l; sm_O[wave][lane] = o;
  __syncthreads();
  if (wave != 0) return;
  float Mt = fmaxf(fmaxf(sm_M[0][lane], sm_M[1][lane]), fmaxf(sm_M[2][lane], sm_M[3][lane]));
  float lt = 0.f;
  floatx4 ot = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    float f = sm_M[w][lane] == -INFINITY ? 0.f : exp2f(sm_M[w][lane] - Mt);
    lt += f * sm_L[w][lane];
    ot += f * sm_O[w][lane];
  }
  if (qa >= a.A || !(fl & ROW_VALID)) return;
  float inv = 1.f / lt;
  float y[4] = {ot[0] * inv, ot[1] * inv, ot[2] * inv, ot[3] * inv};
  store4_split(a.out, a.out_lo, act_off(r, h * HD + i * 16 + 4 * g, a.d), y);
}

static int pick_splits(pd_ctx *c, int units, int nblk) {
  int cap = std::max(1, c->part_units / units);
  if (c->opt_splits > 0) return std::min(c->opt_splits, cap);
  // One block per compute unit, every wave streaming several key blocks back to back (measured at
  // 16 heads x 8k keys: 16.2 us with 256 blocks, 17.2 with 512 or 768, 18.7 with 320; at 4 x 32 heads
  // x 4k keys 256 blocks are 4 us per launch faster than 768).  Always at least one key block per wave.
  // Up to 32 key blocks (8 per wave) a single block per (request, head) is faster than splits plus the
  // merge kernel (measured at 12 heads, 512 + 280 keys: 0.54 against 0.59 ms for a step of 12 layers
  // with two attentions each; at 1024 + 300 keys one split is slower than the automatic 12).
  if (nblk <= 32) return 1;
  int want = std::max(1, 256 / units);
  int by_keys = std::max(1, nblk / 4);
  return std::max(1, std::min(std::min(want, by_keys), cap));
}

template <int HD, bool SPLIT, bool PAIR, bool BIAS, bool STREAM>
static void launch_attn(dim3 grid, hipStream_t s, hipEvent_t e0, hipEvent_t e1, const AttnArgs &a) {
  if (e0 || e1) hipExtLaunchKernelGGL((k_attn_mfma<HD, SPLIT, PAIR, BIAS, STREAM>), grid, dim3(256), 0, s, e0, e1, 0, a);
  else hipLaunchKernelGGL((k_attn_mfma<HD, SPLIT, PAIR, BIAS, STREAM>), grid, dim3(256), 0, s, a);
}

int mfma_attention(pd_ctx *c, const LayerPtrs &lw, int A, int nreq, int req0, int kv_override,
                   hipStream_t s, const AttnMode *mode) {
  const pd_config &g = c->cfg;
  if (kv_override >= 0 && !mode && c->opt_profile == 0) {     // context pass: many rows per request
    int rc = mfma_attention_ctx(c, lw, A, nreq, req0, kv_override, s);
    if (rc != 1) return rc;
  }
  AttnArgs a;
  memset(&a, 0, sizeof(a));
  a.q = (const f16_t *)c->q; a.q_lo = (const f16_t *)mfma_lo(c, c->q, g.d_model);
  a.out_lo = mfma_lo(c, c->att, g.d_model); a.kc = (const f16_t *)lw.kc; a.vc = (const f16_t *)lw.vc;
  a.kc_lo = (const f16_t *)lw.kc_lo; a.vc_lo = (const f16_t *)lw.vc_lo;
  a.out = (bf16_t *)c->att; a.rt = c->rows; a.kv_len = c->sch.kv_len; a.gen_sub = c->sch.gen_sub;
  a.kv_override = kv_override; a.part = c->att_part;
  a.d = g.d_model; a.H = g.n_head; a.kv_cap = c->kv_cap; a.gen_stride = c->gen_stride; a.L = c->L;
  a.A = A; a.nqg = (A + 15) / 16; a.req0 = req0;
  a.scale_log2 = 1.4426950408889634f / sqrtf((float)g.head_dim);
  if (mode) {
    PD_REQUIRE(!a.kc_lo, PD_EINVAL, "the encoder-decoder form keeps no pair layers");
    if (mode->kc) { a.kc = (const f16_t *)mode->kc; a.vc = (const f16_t *)mode->vc; }
    if (mode->qinfo) a.rt.qinfo = const_cast<int4 *>(mode->qinfo);
    a.L = mode->L;
    a.scale_log2 = 1.4426950408889634f * mode->scale;
    if (mode->bias) {
      PD_REQUIRE(mode->bias_len >= 1 && mode->bias_len <= BIAS_MAX && mode->coord && mode->coord_stride >= 8,
                 PD_EINVAL, "relative-position bias table of %d entries (at most %d)", mode->bias_len, BIAS_MAX);
      a.bias = mode->bias; a.coord = mode->coord; a.bias_len = mode->bias_len; a.bias_off = mode->bias_off;
      a.coord_stride = mode->coord_stride; a.coord_req_stride = mode->coord_req_stride;
      a.coord_off = mode->coord_off; a.pos0 = mode->pos0;
    }
  }
  int units = nreq * a.nqg * g.n_head;
  PD_REQUIRE(units <= c->part_units, PD_EINVAL, "too many (request, head, query group) units: %d", units);
  // the most keys this launch can meet: prefill knows it, decode takes the end of the run
  int n_keys = kv_override >= 0 ? kv_override : c->L + c->S * (c->M + 1);
  a.nblk_static = std::min((n_keys + 31) / 32, c->kv_cap / 32);
  a.nsplit = pick_splits(c, units, a.nblk_static);
  dim3 grid(a.nsplit, g.n_head, nreq * a.nqg);
  // measurement: mode 1 attaches a start and a stop event to the dispatch of the main kernel itself
  // (their difference is the kernel's execution time), mode 2 records events before the main kernel
  // and after the merge kernel
  // mode 3 records nothing: it launches the main kernel one extra time first, on the cache of the layer half
  // the stack away (other bytes of the same size: no cache serves them) and with the same outputs, which the
  // real launch then overwrites.  Timing a run of steps with and without it gives the kernel's cost where it
  // runs, between its neighbours, without any event next to it.
  const bool twice = c->opt_profile == 3 && kv_override < 0 && !a.bias && !a.kc_lo;
  AttnArgs a_extra = a;
  if (twice) {
    const size_t n = c->layers.size(), l = (size_t)(&lw - c->layers.data());
    const LayerPtrs &other = c->layers[(l + n / 2) % n];
    a_extra.kc = (const f16_t *)other.kc; a_extra.vc = (const f16_t *)other.vc;
  }
  bool prof = (c->opt_profile == 1 || c->opt_profile == 2) && kv_override < 0 && !a.bias;   // (the instantiations with coordinates take no events)
  hipEvent_t ev0 = nullptr, ev1 = nullptr;
  if (prof) {
    while (c->ev_pool.size() < c->ev_used + 2) {
      hipEvent_t ev;
      PD_CHECK_HIP(hipEventCreate(&ev));
      c->ev_pool.push_back(ev);
    }
    ev0 = c->ev_pool[c->ev_used];
    ev1 = c->ev_pool[c->ev_used + 1];
    if (c->opt_profile == 2) PD_CHECK_HIP(hipEventRecord(ev0, s));
  }
  const bool attach = prof && c->opt_profile == 1;
  hipEvent_t pe0 = attach ? ev0 : nullptr, pe1 = attach ? ev1 : nullptr;
  // decode steps of the decoder-only form stream their keys and values (see STREAM); the context pass, the
  // teacher-forced forward and the encoder-decoder launches (small or re-read key sets) do not
  const bool stream = kv_override < 0 && !mode && c->stream_loads;
#define PD_ATTN_ONE(HDV, ARGS)                                                                         \
  do {                                                                                                 \
    const bool sp = a.q_lo != nullptr, pr = a.kc_lo != nullptr, bi = a.bias != nullptr;                \
    if (bi && sp) launch_attn<HDV, true, false, true, false>(grid, s, pe0, pe1, ARGS);                 \
    else if (bi) launch_attn<HDV, false, false, true, false>(grid, s, pe0, pe1, ARGS);                 \
    else if (pr && sp && stream) launch_attn<HDV, true, true, false, true>(grid, s, pe0, pe1, ARGS);   \
    else if (pr && sp) launch_attn<HDV, true, true, false, false>(grid, s, pe0, pe1, ARGS);            \
    else if (pr && stream) launch_attn<HDV, false, true, false, true>(grid, s, pe0, pe1, ARGS);        \
    else if (pr) launch_attn<HDV, false, true, false, false>(grid, s, pe0, pe1, ARGS);                 \
    else if (sp && stream) launch_attn<HDV, true, false, false, true>(grid, s, pe0, pe1, ARGS);        \
    else if (sp) launch_attn<HDV, true, false, false, false>(grid, s, pe0, pe1, ARGS);                 \
    else if (stream) launch_attn<HDV, false, false, false, true>(grid, s, pe0, pe1, ARGS);             \
    else launch_attn<HDV, false, false, false, false>(grid, s, pe0, pe1, ARGS);                        \
  } while (0)
#define PD_ATTN(HDV)                                                                                   \
  do {                                                                                                 \
    if (twice) PD_ATTN_ONE(HDV, a_extra);                                                              \
    PD_ATTN_ONE(HDV, a);                                                                               \
    if (a.nsplit > 1)                                                                                  \
      hipLaunchKernelGGL(k_attn_merge<HDV>, dim3(units, HDV / 16), dim3(256), 0, s, a);                \
  } while (0)
  switch (g.head_dim) {
    case 32: PD_ATTN(32); break;
    case 64: PD_ATTN(64); break;
    case 96: PD_ATTN(96); break;
    case 128: PD_ATTN(128); break;
    default: pd_set_error("head_dim %d not supported by the MFMA attention", g.head_dim); return PD_EINVAL;
  }
#undef PD_ATTN
#undef PD_ATTN_ONE
  PD_CHECK_HIP(hipGetLastError());
  if (prof) {
    if (c->opt_profile != 1) PD_CHECK_HIP(hipEventRecord(c->ev_pool[c->ev_used + 1], s));
    c->ev_used += 2;
  }
  return PD_OK;
}
