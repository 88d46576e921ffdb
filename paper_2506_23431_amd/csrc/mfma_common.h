// bf16 matrix-core path for gfx950.
//
// Design rule of this file: every large operand that is streamed from HBM once per
// step (weights, key cache, value cache) is stored in HBM in the exact order in
// which the 16x16x32 MFMA instruction (bf16 for weights x activations, fp16 for the
// attention products) wants it in registers.  A "fragment" is
// the A operand of one such instruction: 16 rows x 32 contraction values = 1 KiB,
// lane l (0..63) holding 8 consecutive contraction values (16 bytes) of row l%16,
// contraction group l/16.  A fragment is stored as 64 consecutive 16-byte granules
// in lane order, so one wave-wide 16-byte load reads 1 KiB contiguous and lands in
// the operand registers with no shuffle and no LDS round trip.
//
//   packed weight  W[N][K]:  fragments [N/16][K/32]; fragment (nt, kt) row m, group g,
//                            element e  <->  W[row(nt*16+m)][kt*32 + g*8 + e]
//   K cache (per request, head): blocks of 32 keys; block kb holds 2 tiles x (hd/32)
//                            fragments; tile t row m=4g'+j <-> key kb*32 + 8g' + 4t + j,
//                            contraction = head-dim chunk c: dim c*32 + g*8 + e
//   V cache (per request, head): block kb holds hd/16 fragments; fragment hb row r <->
//                            dim hb*16 + r, contraction slot (g, e) <-> key kb*32 + 8g + e
//
// The key order inside a K tile is chosen so that the score tile S^T = K Q^T comes out
// of the matrix core already in the register order the P^T operand of O^T = V^T P^T
// needs: scores never leave registers between the two contractions.
#pragma once
#include "pd_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

union Frag {
  uint4 u;
  bf16x8 v;
  bf16_t h[8];
  f16x8 hv;       // fp16 view: KV cache, queries and probabilities of the attention kernel
  f16_t hh[8];
};

__device__ __forceinline__ floatx4 mfma16(const Frag &a, const Frag &b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.v, b.v, c, 0, 0, 0);
}

__device__ __forceinline__ floatx4 mfma16h(const Frag &a, const Frag &b, floatx4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a.hv, b.hv, c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  return (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
}

// Activations are carried as a pair of bf16 values, x ~ hi + lo with hi = bf16(x) and
// lo = bf16(x - hi): two matrix-core passes over the same weight fragment then see the
// activation to about 16 mantissa bits, which costs no extra HBM traffic.
__device__ __forceinline__ float bf16_residual(float x, bf16_t hi) { return x - bf16_to_f32(hi); }

// Activation matrices [rows][K] that feed a matrix multiply are stored fragment-major too:
// the B operand of the instruction for row tile rt (16 rows) and k-tile kt (32 values) is
// 64 consecutive 16-byte granules, lane g*16 + m holding row rt*16 + m, k = kt*32 + g*8 .. +7.
// A wave therefore reads a B operand as 1 KiB contiguous, like a weight fragment.
__device__ __forceinline__ size_t act_off(int r, int k, int K) {
  return ((((size_t)(r >> 4) * (K >> 5) + (k >> 5)) * 64) + ((k & 31) >> 3) * 16 + (r & 15)) * 8 + (k & 7);
}

// store 4 consecutive values (k multiple of 4) as hi (and, if lo != NULL, lo) bf16 quadruples
__device__ __forceinline__ void store4_split(bf16_t *hi, bf16_t *lo, size_t off, const float y[4]) {
  bf16_t h0 = f32_to_bf16(y[0]), h1 = f32_to_bf16(y[1]), h2 = f32_to_bf16(y[2]), h3 = f32_to_bf16(y[3]);
  *(uint2 *)(hi + off) = make_uint2((uint32_t)h0 | ((uint32_t)h1 << 16), (uint32_t)h2 | ((uint32_t)h3 << 16));
  if (lo)
    *(uint2 *)(lo + off) = make_uint2(pack2(bf16_residual(y[0], h0), bf16_residual(y[1], h1)),
                                      pack2(bf16_residual(y[2], h2), bf16_residual(y[3], h3)));
}

// the same for fp16 pairs (queries: they meet the fp16 key cache in the matrix core)
__device__ __forceinline__ void store4_split_h(f16_t *hi, f16_t *lo, size_t off, const float y[4]) {
  union { f16_t h[4]; uint2 u; } a, b;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    a.h[j] = f32_to_f16_sat(y[j]);
    b.h[j] = (f16_t)(y[j] - (float)a.h[j]);
  }
  *(uint2 *)(hi + off) = a.u;
  if (lo) *(uint2 *)(lo + off) = b.u;
}

// element offsets inside the packed caches (per request and head)
__device__ __forceinline__ size_t k_cache_off(int key, int dim, int hd) {
  int kb = key >> 5, w = key & 31, gk = w >> 3, j8 = w & 7, t = j8 >> 2, m = gk * 4 + (j8 & 3);
  int c = dim >> 5, g = (dim & 31) >> 3, e = dim & 7;
  return ((size_t)(kb * 2 + t) * (hd >> 5) + c) * 512 + (g * 16 + m) * 8 + e;
}
__device__ __forceinline__ size_t v_cache_off(int key, int dim, int hd) {
  int kb = key >> 5, w = key & 31, g = w >> 3, e = w & 7;
  int hb = dim >> 4, r = dim & 15;
  return ((size_t)kb * (hd >> 4) + hb) * 512 + (g * 16 + r) * 8 + e;
}


// ---- entry points between the sources of the bf16 path -------------------------------------
enum { EPI_QKV = 0, EPI_QKV_ROPE = 1, EPI_RESID = 2, EPI_GELU = 3, EPI_SWIGLU = 4, EPI_LM = 5, EPI_RESID_NORM = 6,
       EPI_QKV_NORM = 7 /* EPI_QKV fed gain * x: finishes the norm in its epilogue (stats_in, c1, c2) */ };

struct GemmArgs {
  const bf16_t *W;       // packed
  const bf16_t *xn;      // [16*RT][K] bf16, fragment-major: activations (high part)
  const bf16_t *xn_lo;   // same shape: bf16(x - high part), or NULL to use the high part only
  int K, n_tiles, R;
  int k_share;           // k-tiles per wave along K (set by the launch)
  int packed;            // 1: xn holds high parts in rows 0-7 and low parts in rows 8-15 (R <= 8); xn_lo unused
  // epilogue
  float *x;              // EPI_RESID: split-K slices of y, [slices][part_stride], row-major [rows][ld]
  size_t part_stride; int max_parts; int *parts_out;   // EPI_RESID: slice stride, limit, slices written
  bf16_t *out_bf;        // EPI_GELU / EPI_SWIGLU: [rows][ld]; EPI_QKV*: q [rows][d]
  bf16_t *out_lo;        // low parts of out_bf (written when not NULL)
  int ld;
  f16_t *kc, *vc;        // EPI_QKV*: caches of this layer (fp16)
  f16_t *kc_lo, *vc_lo;  // their low halves, or NULL
  int32_t *kv_sat;       // EPI_QKV*: counter of keys / values stored saturated
  RowTables rt;
  const float *rope_cs;
  int d, H, hd, kv_cap;
  float *logits; int V, ld_logits;     // EPI_LM: optional logits [rows][ld_logits]
  float *part_val; int32_t *part_idx;  // EPI_LM: [16*RT][n_tiles] best value / index per tile
  // EPI_RESID_NORM (at most 16 rows, K not cut over blocks): x_res += y in place, out_bf / out_lo receive
  // gain * x_res as activation fragments, stats_out[row][tile] the sum and the sum of squares of x_res
  // over the tile's 16 columns
  float *x_res; const float *gain; float2 *stats_out;
  // EPI_GELU / EPI_SWIGLU with stats_in != NULL: the activations are gain * x (not normalised); the
  // epilogue applies the norm, y = rstd * (acc - mean * c1[n]) + c2[n], with mean and rstd of every row
  // from stats_in[row][stats_tiles] and c1 = W gain, c2 = W bias (c2 NULL: no bias)
  const float2 *stats_in; int stats_tiles; const float *c1, *c2; int norm_kind, norm_d; float norm_eps;
  int act;               // EPI_GELU: 0 gelu(erf), 1 relu
  int sec0;              // EPI_QKV*: section of the weight's first d columns (0: Q, K, V follow; 1: K, V only)
  int stream_w;          // 1: load the weights with the non-temporal hint (a step's bytes exceed the last-level cache)
};

int mfma_gemm(int epi, const GemmArgs &a, int rows, hipStream_t s);
int mfma_gemm_row_tiles(int rows);            // rows a launch reads/writes: 16 * RT
// whether a projection of n_tiles x K at this many rows is launched with one row tile per block
bool mfma_gemm_row_tile_blocks(int n_tiles, int K, int rows, int k_slices);
int mfma_norm(pd_ctx *c, const float *gain, const float *bias, int R, hipStream_t s);
// low-part twin of an activation buffer (NULL when the split is switched off)
bf16_t *mfma_lo(pd_ctx *c, void *buf, size_t cols);
// pieces of a layer's launch sequence (mfma.hip)
void mfma_gemm_base(pd_ctx *c, GemmArgs &a, int R);
// c1 != NULL: the rows in c->xn are gain * x with per-tile sums in c->nstats (c->norm_fused): the epilogue finishes the norm
int mfma_qkv(pd_ctx *c, GemmArgs &a, const bf16_t *W, int n_tiles, int sec0, void *kc, void *vc, void *kc_lo,
             void *vc_lo, int R, hipStream_t s, const float *c1 = nullptr, const float *c2 = nullptr);
// next_gain != NULL (and at most 16 rows): the projection also prepares the norm with that gain for the
// projection that follows (sets c->norm_fused)
int mfma_out(pd_ctx *c, GemmArgs &a, const bf16_t *p_wo, int R, hipStream_t s, const float *next_gain = nullptr);
// next_gain != NULL: the second FFN projection may prepare the next layer's first norm (sets c->norm_fused)
int mfma_out_ffn(pd_ctx *c, GemmArgs &a, const bf16_t *p_wo, const LayerPtrs &lw, int R, hipStream_t s,
                 const float *next_gain = nullptr);
bool mfma_can_fuse_norm(pd_ctx *c, int R);
int mfma_fold(float *c1, float *c2, const bf16_t *Wp, const float *gain, const float *bias, int n_out, int K,
              hipStream_t s);
int mfma_pack_matrix(bf16_t *dst, const void *src, int N, int K, hipStream_t s);   // row-major [N][K] -> fragments
// What an attention launch of the encoder-decoder form changes (NULL: the decoder-only defaults).
struct AttnMode {
  const void *kc, *vc;     // caches to read (NULL: the layer's own)
  const int4 *qinfo;       // {flags, sub, lim, req} per row (NULL: the step's row table)
  int L;                   // keys below L are visible up to a row's limit, keys from L on by their tags
  float scale;             // factor on q.k
  // Grid coordinates (bias NULL: none, the plain kernel).  coord[key] at coord[req * coord_req_stride +
  // key - coord_off], coord_stride entries readable; a query's coordinate is pos[row] - pos0.  The score
  // gets bias[h][clamp(c_q - coord[key] + bias_off, 0, bias_len - 1)] (already times log2(e); a table of
  // one zero: no bias), and generated-side keys later than the query are masked.
  const float *bias; const uint16_t *coord;
  int bias_len, bias_off, coord_stride, coord_req_stride, coord_off, pos0;
};
int mfma_attention(pd_ctx *c, const LayerPtrs &lw, int A, int nreq, int req0, int kv_override,
                   hipStream_t s, const AttnMode *mode = nullptr);
// context pass, many rows: PD_OK when it ran the launch, 1 when the shape is not one it serves (attn_ctx.hip)
int mfma_attention_ctx(pd_ctx *c, const LayerPtrs &lw, int A, int nreq, int req0, int n_keys, hipStream_t s);
