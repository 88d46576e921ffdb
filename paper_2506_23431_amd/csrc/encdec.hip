// Encoder-decoder form of the pipelined decoder, the form the paper itself runs (Eq. 1: the input is
// encoded once by a stacked bidirectional encoder; Eq. 3: every decoder layer attends to the
// generated side under the dependency rule of Section 3.2 and then to the encoder states; Section
// 4.3: the relative position of two generated-side tokens is the Manhattan distance of their grid
// coordinates, which feeds the bucketed relative-position bias of the backbone).
//
// Everything here is a launch sequence over the kernels of the decoder-only path:
//   * the projections, norms, vocabulary head, schedule tick and commit are the same kernels
//     (RMS norm, W2 relu(W1 u), no biases, no absolute positions);
//   * the attention kernel runs in its BIAS instantiation for the two self-attentions: the score of a
//     query at coordinate c_q and a key at coordinate c_k gets table[h][c_q - c_k + offset].  For the
//     decoder the coordinate of a token is (t - 1) + (i - 1): on every visible pair both |t_q - t_k| and
//     |i_q - i_k| are differences without sign, so the Manhattan distance is c_q - c_k.  For the
//     encoder it is the position, and the table covers both signs.  The tables hold the bucketed
//     bias already looked up per clamped distance (beyond max_distance the bucket no longer changes);
//   * the attention over the encoder states is the unbiased instantiation over a second cache that
//     the encoder pass fills once per request: all Lx keys visible, no generated side.
#include "mfma_common.h"

#include <cmath>
#include <vector>

int encdec_pack_weights(pd_ctx *c, hipStream_t s) {
  const pd_config &g = c->cfg;
  const int d = g.d_model, ff = g.d_ff;
  int rc;
  for (LayerPtrs &lp : c->ed.enc) {
    if ((rc = mfma_pack_matrix(lp.p_wqkv, lp.wqkv, 3 * d, d, s))) return rc;
    if ((rc = mfma_pack_matrix(lp.p_wo, lp.wo, d, d, s))) return rc;
    if ((rc = mfma_pack_matrix(lp.p_w1, lp.w1, ff, d, s))) return rc;
    if ((rc = mfma_pack_matrix(lp.p_w2, lp.w2, d, ff, s))) return rc;
  }
  for (LayerPtrs &lp : c->layers) {
    if ((rc = mfma_pack_matrix(lp.p_cq, lp.cq, d, d, s))) return rc;
    if ((rc = mfma_pack_matrix(lp.p_ckv, lp.ckv, 2 * d, d, s))) return rc;
    if ((rc = mfma_pack_matrix(lp.p_co, lp.co, d, d, s))) return rc;
    // the query projection over the encoder states can finish the norm in front of it
    if ((rc = mfma_fold(lp.cx1, nullptr, lp.p_cq, lp.n3g, nullptr, d, d, s))) return rc;
  }
  return PD_OK;
}

// tab[h][i] = log2(e) * rel_bias[bucket][h] for the distance that index i stands for.
//   decoder (bidir 0): i = keys behind the query, 0 .. max_distance
//   encoder (bidir 1): i = query - key + max_distance; keys ahead of the query (i < max_distance) use
//                      the upper half of the buckets, keys behind or at it the lower half
// bucket_of[i] is computed on the host (double-precision logarithm); the kernel only gathers.
__global__ void k_bias_table(float *tab, const float *rel_bias, const int *bucket_of, int len, int H) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= len * H) return;
  int h = i / len, j = i % len;
  tab[i] = 1.4426950408889634f * rel_bias[(size_t)bucket_of[j] * H + h];
}

// Bucket of a key n >= 0 positions behind the query in a table of `buckets` entries: n itself below
// buckets / 2, then logarithmically spaced up to max_distance, the last bucket beyond (the published
// definition of the backbone's relative-position buckets).
static int bucket_behind_host(int n, int buckets, int max_distance) {
  const int max_exact = buckets / 2;
  if (n < max_exact) return n;
  const double v = std::log((double)n / max_exact) / std::log((double)max_distance / max_exact) * (buckets - max_exact);
  return std::min(max_exact + (int)std::floor(v), buckets - 1);
}

// Builds both bias tables and the encoder's key coordinates.  `scratch` is device memory for
// enc_len + dec_len ints (the bucket of every table index), filled from the host.
int encdec_build_tables(pd_ctx *c, int *scratch, hipStream_t s) {
  EncDecState &e = c->ed;
  const int H = c->cfg.n_head, md = e.rel_max_distance, nb = e.rel_buckets;
  std::vector<int> bucket(e.enc_len + e.dec_len);
  for (int i = 0; i < e.enc_len; ++i) {
    const int behind = i - md;                       // query - key
    bucket[i] = behind >= 0 ? bucket_behind_host(behind, nb / 2, md) : nb / 2 + bucket_behind_host(-behind, nb / 2, md);
  }
  for (int i = 0; i < e.dec_len; ++i) bucket[e.enc_len + i] = bucket_behind_host(i, nb, md);
  PD_CHECK_HIP(hipMemcpyAsync(scratch, bucket.data(), bucket.size() * sizeof(int), hipMemcpyHostToDevice, s));
  PD_CHECK_HIP(hipStreamSynchronize(s));             // `bucket` goes out of scope
  hipLaunchKernelGGL(k_bias_table, dim3((e.enc_len * H + 255) / 256), dim3(256), 0, s, e.enc_bias, e.enc_rel_bias,
                     scratch, e.enc_len, H);
  hipLaunchKernelGGL(k_bias_table, dim3((e.dec_len * H + 255) / 256), dim3(256), 0, s, e.dec_bias, e.dec_rel_bias,
                     scratch + e.enc_len, e.dec_len, H);
  PD_CHECK_HIP(hipGetLastError());
  std::vector<uint16_t> coord(c->kv_cap);
  for (int j = 0; j < c->kv_cap; ++j) coord[j] = (uint16_t)j;
  PD_CHECK_HIP(hipMemcpyAsync(e.enc_coord, coord.data(), coord.size() * sizeof(uint16_t), hipMemcpyHostToDevice, s));
  PD_CHECK_HIP(hipMemsetAsync(scratch, 0, bucket.size() * sizeof(int), s));   // borrowed memory goes back cleared
  PD_CHECK_HIP(hipStreamSynchronize(s));
  return PD_OK;
}

// Eq. 1 for request b: H^E = Encoder(X) over its Lx input tokens as one launch sequence (all rows at
// once: the encoder is bidirectional, so a layer's attention needs every key of that layer), then the
// keys and values of H^E under every decoder layer's projection, written to that layer's second cache.
int encdec_encode(pd_ctx *c, int b, hipStream_t s) {
  const pd_config &g = c->cfg;
  EncDecState &e = c->ed;
  const int d = g.d_model, n = c->Lx;
  int rc;
  // rows 0 .. n-1 = positions; their keys and values go to entry 0 of the encoder's scratch cache
  if ((rc = launch_prefill_rows(c, b, 0, n, s, n, 1, 0))) return rc;
  c->packed = false;
  c->embed_pending = true;
  c->pend_parts = 0;
  c->norm_fused = false;
  AttnMode am;
  memset(&am, 0, sizeof(am));
  am.L = n; am.scale = 1.f;
  am.bias = e.enc_bias; am.bias_len = e.enc_len; am.bias_off = e.rel_max_distance;
  am.coord = e.enc_coord; am.coord_stride = c->kv_cap; am.coord_req_stride = 0;
  for (const LayerPtrs &lw : e.enc) {
    if ((rc = mfma_norm(c, lw.n1g, nullptr, n, s))) return rc;
    GemmArgs a;
    mfma_gemm_base(c, a, n);
    if ((rc = mfma_qkv(c, a, lw.p_wqkv, 3 * d / 16, 0, lw.kc, lw.vc, nullptr, nullptr, n, s))) return rc;
    if ((rc = mfma_attention(c, lw, n, 1, 0, n, s, &am))) return rc;
    if ((rc = mfma_out_ffn(c, a, lw.p_wo, lw, n, s))) return rc;
  }
  if ((rc = mfma_norm(c, e.enc_fng, nullptr, n, s))) return rc;      // c->xn = H^E
  // the same rows again, now addressed to request b's entry of the decoder layers' second caches
  if ((rc = launch_prefill_rows(c, b, 0, n, s, n, 1, b))) return rc;
  for (const LayerPtrs &lw : c->layers) {
    GemmArgs a;
    mfma_gemm_base(c, a, n);
    if ((rc = mfma_qkv(c, a, lw.p_ckv, 2 * d / 16, 1, lw.xkc, lw.xvc, nullptr, nullptr, n, s))) return rc;
  }
  return PD_OK;
}

// One decoder layer of a decode step (Eq. 3): self-attention over the generated side under the
// dependency rule with the Manhattan-distance bias, attention over the encoder states, feed-forward.
// A rows per request, nreq requests from req0 on.  kv_self < 0: a decode step (each request's keys so far);
// otherwise the number of generated-side keys to consider (the one-pass teacher-forced forward, where the
// time half of the matrix is the attention kernel's own check).
int encdec_decoder_layer(pd_ctx *c, int l, int R, hipStream_t s, int A, int nreq, int req0, int kv_self) {
  if (A <= 0) { A = c->A; nreq = c->B; req0 = 0; kv_self = -1; }
  const pd_config &g = c->cfg;
  EncDecState &e = c->ed;
  const LayerPtrs &lw = c->layers[l];
  const int d = g.d_model;
  int rc;
  if ((rc = mfma_norm(c, lw.n1g, nullptr, R, s))) return rc;
  GemmArgs a;
  mfma_gemm_base(c, a, R);
  if ((rc = mfma_qkv(c, a, lw.p_wqkv, 3 * d / 16, 0, lw.kc, lw.vc, nullptr, nullptr, R, s))) return rc;
  AttnMode self;
  memset(&self, 0, sizeof(self));
  self.L = 0; self.scale = 1.f;
  self.bias = e.dec_bias; self.bias_len = e.dec_len; self.bias_off = 0;
  self.coord = c->gen_coord; self.coord_stride = c->gen_stride; self.coord_req_stride = c->gen_stride;
  if ((rc = mfma_attention(c, lw, A, nreq, req0, kv_self, s, &self))) return rc;
  // In steps of at most 16 rows the output projection also prepares the norm that follows it and the
  // query projection behind that norm finishes it (gemm.hip): no norm kernel in between.
  if ((rc = mfma_out(c, a, lw.p_wo, R, s, lw.n3g))) return rc;
  // attention over the encoder states: queries from the normalised rows, keys and values from the
  // second cache, every one of the Lx keys visible to every row that carries a token
  const bool finish = c->norm_fused;
  if (!finish && (rc = mfma_norm(c, lw.n3g, nullptr, R, s))) return rc;
  if ((rc = mfma_qkv(c, a, lw.p_cq, d / 16, 0, nullptr, nullptr, nullptr, nullptr, R, s, finish ? lw.cx1 : nullptr)))
    return rc;
  AttnMode cross;
  memset(&cross, 0, sizeof(cross));
  cross.kc = lw.xkc; cross.vc = lw.xvc; cross.qinfo = c->qinfo_x; cross.L = c->Lx; cross.scale = 1.f;
  if ((rc = mfma_attention(c, lw, A, nreq, req0, c->Lx, s, &cross))) return rc;
  return mfma_out_ffn(c, a, lw.p_co, lw, R, s);
}
