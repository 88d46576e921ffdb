"""Encoder-decoder form of the pipelined decoder, as the paper itself runs it (Eq. 1: the input is
encoded once by a stacked encoder into H^E; Eq. 3: the decoder attends to the generated side under
the dependency rule of Section 3.2 and to H^E; Section 4.3: the relative position between two
generated-side tokens, which feeds the backbone's relative-position attention bias, is the
Manhattan distance |t1 - t2| + |i1 - i2| of their grid coordinates).  Test infrastructure only;
fp64 numpy.

The backbone is the published text-to-text transformer family the paper names in Section 4.3,
restated here from its published description:
  * pre-norm residual blocks; the norm rescales by the root mean square (no mean subtraction, no
    bias); feed-forward W2 relu(W1 u); no biases in linear layers
  * attention scores are q.k + bias[head][bucket(relative position)] without a 1/sqrt(head_dim)
    factor; one bias table per stack, shared by all of its layers; cross-attention has no bias
  * bucket(n) for a key n >= 0 positions behind the query (decoder: keys ahead of the query never
    occur): n itself below max_exact = buckets/2, then logarithmically spaced up to max_distance,
    the last bucket taking everything beyond.  The encoder is bidirectional: half of the buckets
    serve keys behind or at the query, the other half keys ahead of it.
Readings where the paper is silent
  * the distance that enters bucket() for a query (i_q, tau_q) and a visible key (i_k, tau_k) is
    (tau_q - tau_k) + (i_q - i_k); both terms are non-negative on visible pairs
  * the vocabulary projection is a separate matrix applied to the normalised decoder output.

Parity status: pinned in tests/test_oracle_encdec.py by the bucket function's definition and
closed-form thresholds, by an independent dense encoder-decoder written with PyTorch library ops
(one subsequence == ordinary decoding with ordinary relative positions; any schedule == one dense
forward under the enumerated mask and Manhattan distances), and by the per-query loop equalling
the matrix-masked form.
"""

import math

import numpy as np

from . import primitives as P

F = np.float64


def bucket_behind(n, buckets, max_distance):
    """Bucket of a key n >= 0 positions behind the query, for a table of `buckets` entries."""
    n = np.asarray(n)
    assert np.all(n >= 0)
    max_exact = buckets // 2
    far = np.maximum(n, 1).astype(F)
    log_part = max_exact + np.floor(np.log(far / max_exact) / math.log(max_distance / max_exact)
                                    * (buckets - max_exact)).astype(np.int64)
    return np.where(n < max_exact, n, np.minimum(log_part, buckets - 1)).astype(np.int64)


def bucket_bidirectional(rel, buckets, max_distance):
    """rel = key position - query position (any sign): keys ahead use the upper half of the table."""
    rel = np.asarray(rel)
    half = buckets // 2
    return np.where(rel > 0, half, 0) + bucket_behind(np.abs(rel), half, max_distance)


def manhattan(i_q, t_q, i_k, t_k):
    """Relative distance of two generated-side tokens (Section 4.3)."""
    return abs(t_q - t_k) + abs(i_q - i_k)


def rms_norm(x, gain, eps):
    return x / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps) * gain


class EncDecModel:
    def __init__(self, cfg, weights):
        self.c = cfg
        self.w = {k: (v.astype(F) if isinstance(v, np.ndarray) else v) for k, v in weights.items()}
        self.enc = [{k: v.astype(F) for k, v in lw.items()} for lw in weights["enc_layers"]]
        self.dec = [{k: v.astype(F) for k, v in lw.items()} for lw in weights["dec_layers"]]

    def heads(self, y):
        return y.reshape(y.shape[0], self.c.n_head, self.c.head_dim)

    def ffn(self, lw, x, key):
        u = rms_norm(x, lw[key], self.c.norm_eps)
        return x + np.maximum(u @ lw["w1"].T, 0.0) @ lw["w2"].T

    def encode(self, ctx_tokens):
        """Eq. 1: H^E = Encoder(X), [l, d]."""
        c = self.c
        tok = np.asarray(ctx_tokens)
        n = tok.shape[0]
        x = self.w["tok_emb"][tok]
        rel = np.arange(n)[None, :] - np.arange(n)[:, None]              # key - query
        bias = self.w["enc_rel_bias"][bucket_bidirectional(rel, c.rel_buckets, c.rel_max_distance)]  # [q,k,H]
        for lw in self.enc:
            u = rms_norm(x, lw["norm1_g"], c.norm_eps)
            q, k, v = self.heads(u @ lw["wq"].T), self.heads(u @ lw["wk"].T), self.heads(u @ lw["wv"].T)
            att = np.empty_like(q)
            for h in range(c.n_head):
                att[:, h, :] = P.softmax(q[:, h] @ k[:, h].T + bias[:, :, h], axis=-1) @ v[:, h]
            x = x + att.reshape(n, -1) @ lw["wo"].T
            x = self.ffn(lw, x, "norm2_g")
        return rms_norm(x, self.w["enc_final_g"], c.norm_eps)

    def cross_kv(self, HE):
        return [(self.heads(HE @ lw["ck"].T), self.heads(HE @ lw["cv"].T)) for lw in self.dec]

    def logits(self, x):
        return rms_norm(x, self.w["dec_final_g"], self.c.norm_eps) @ self.w["lm_head"].T


class EncDecPerQueryDecoder:
    """decoder(G, t) for controller.pipelined_decode: incremental, one query at a time, explicit
    visible set and explicit Manhattan distances per query."""

    def __init__(self, model, ctx_tokens, force=None):
        self.m = model
        self.HE = model.encode(ctx_tokens)
        self.cross = model.cross_kv(self.HE)
        self.gen_sub, self.gen_tau = [], []
        self.gen_K = [[] for _ in model.dec]
        self.gen_V = [[] for _ in model.dec]
        self.encoded = []
        self.trace = []
        self.force = force

    def __call__(self, G, t):
        m, c = self.m, self.m.c
        k_open = len(G)
        while len(self.encoded) < k_open:
            self.encoded.append(0)
        rows = [i for i in range(1, k_open + 1) if len(G[i - 1]) > self.encoded[i - 1]]
        out = [-1] * k_open
        rec = {"t": t, "rows": list(rows)}
        if rows:
            x = m.w["tok_emb"][np.array([G[i - 1][-1] for i in rows])]
            for i in rows:
                self.gen_sub.append(i)
                self.gen_tau.append(t)
            vis = [[n for n in range(len(self.gen_sub)) if self.gen_sub[n] <= i and self.gen_tau[n] <= t]
                   for i in rows]
            dist = [[manhattan(i, t, self.gen_sub[n], self.gen_tau[n]) for n in v] for i, v in zip(rows, vis)]
            for l, lw in enumerate(m.dec):
                u = rms_norm(x, lw["norm1_g"], c.norm_eps)
                q, kk, vv = m.heads(u @ lw["wq"].T), m.heads(u @ lw["wk"].T), m.heads(u @ lw["wv"].T)
                for r in range(len(rows)):
                    self.gen_K[l].append(kk[r])
                    self.gen_V[l].append(vv[r])
                att = np.empty_like(q)
                for r in range(len(rows)):
                    K = np.stack([self.gen_K[l][n] for n in vis[r]], axis=1)          # [H, n, hd]
                    V = np.stack([self.gen_V[l][n] for n in vis[r]], axis=1)
                    b = m.w["dec_rel_bias"][bucket_behind(np.array(dist[r]), c.rel_buckets, c.rel_max_distance)]
                    s = (K @ q[r][:, :, None])[:, :, 0] + b.T                           # [H, n]
                    att[r] = (P.softmax(s, axis=1)[:, None, :] @ V)[:, 0, :]
                x = x + att.reshape(len(rows), -1) @ lw["wo"].T
                u = rms_norm(x, lw["norm3_g"], c.norm_eps)
                q = m.heads(u @ lw["cq"].T)
                Kc, Vc = self.cross[l]
                att = np.empty_like(q)
                for h in range(c.n_head):
                    att[:, h, :] = P.softmax(q[:, h] @ Kc[:, h].T, axis=-1) @ Vc[:, h]
                x = x + att.reshape(len(rows), -1) @ lw["co"].T
                x = m.ffn(lw, x, "norm2_g")
            logits = m.logits(x)
            for r, i in enumerate(rows):
                out[i - 1] = P.argmax_lowest(logits[r])
                self.encoded[i - 1] += 1
            rec["logits"] = logits
            rec["dist"] = dist
        if self.force is not None and t - 1 < len(self.force):
            for i in range(1, k_open + 1):
                if int(self.force[t - 1][i - 1]) >= 0:
                    out[i - 1] = int(self.force[t - 1][i - 1])
        self.trace.append(rec)
        return out


def dense_decoder_forward(model, HE, tokens, mask, distance):
    """Matrix-masked form: all generated-side tokens at once under a boolean matrix and a matrix
    of relative distances (both [N, N], query by key).  Returns logits [N, V]."""
    m, c = model, model.c
    x = m.w["tok_emb"][np.asarray(tokens)]
    N = x.shape[0]
    bias = m.w["dec_rel_bias"][bucket_behind(np.where(mask, distance, 0), c.rel_buckets, c.rel_max_distance)]
    cross = m.cross_kv(HE)
    for l, lw in enumerate(m.dec):
        u = rms_norm(x, lw["norm1_g"], c.norm_eps)
        q, k, v = m.heads(u @ lw["wq"].T), m.heads(u @ lw["wk"].T), m.heads(u @ lw["wv"].T)
        att = np.empty_like(q)
        for h in range(c.n_head):
            s = np.where(mask, q[:, h] @ k[:, h].T + bias[:, :, h], -np.inf)
            att[:, h, :] = P.softmax(s, axis=-1) @ v[:, h]
        x = x + att.reshape(N, -1) @ lw["wo"].T
        u = rms_norm(x, lw["norm3_g"], c.norm_eps)
        q = m.heads(u @ lw["cq"].T)
        Kc, Vc = cross[l]
        att = np.empty_like(q)
        for h in range(c.n_head):
            att[:, h, :] = P.softmax(q[:, h] @ Kc[:, h].T, axis=-1) @ Vc[:, h]
        x = x + att.reshape(N, -1) @ lw["co"].T
        x = m.ffn(lw, x, "norm2_g")
    return m.logits(x)


class EncDecMatrixDecoder:
    """decoder(G, t): full recompute of every generated-side token under the matrix of Fig. 3b,
    coordinates from the closed form tau = (i-1) dt + 1 + j."""

    def __init__(self, model, ctx_tokens, delta_t):
        self.m, self.dt = model, delta_t
        self.HE = model.encode(ctx_tokens)
        self.trace = []

    def __call__(self, G, t):
        coords = [(i, (i - 1) * self.dt + 1 + j, tok) for i, g in enumerate(G, start=1) for j, tok in enumerate(g)]
        ii = np.array([c[0] for c in coords])
        tt = np.array([c[1] for c in coords])
        mask = (ii[None, :] <= ii[:, None]) & (tt[None, :] <= tt[:, None])
        distance = np.abs(tt[:, None] - tt[None, :]) + np.abs(ii[:, None] - ii[None, :])
        logits = dense_decoder_forward(self.m, self.HE, [c[2] for c in coords], mask, distance)
        last, row = {}, 0
        for i, g in enumerate(G, start=1):
            row += len(g)
            last[i] = row - 1
        self.trace.append({"t": t, "logits": {i: logits[last[i]] for i in last}})
        return [P.argmax_lowest(logits[last[i]]) for i in range(1, len(G) + 1)]
