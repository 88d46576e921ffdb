"""Decoder-only transformer in fp64: weights, per-token maps, and the causal pass
over the context.  Test infrastructure only.

The paper's decoder is "a stacked transformer decoder with the same parameters
and architecture as a sequential decoder" (Section 3.2); the block used here is
the pre-norm, bias-free block the workloads name.  The context plays the role of
the encoder states H^E of Eq. 1: it is encoded once, every generated token
attends to all of it.
"""

import numpy as np

from . import primitives as P

F = np.float64


_POOL = None


def _to_f64(a):
    """Decode a weight array: uint16 = bf16 bit patterns, otherwise numeric.  The widening is
    exact; large matrices are widened in row blocks on a few threads (a 7B-parameter model that
    cannot keep fp64 copies of all its layers widens every layer again each time it is used)."""
    if a is None:
        return None
    if a.dtype != np.uint16:
        return a.astype(F)
    if a.ndim < 2 or a.size < (1 << 22):
        return (a.astype(np.uint32) << 16).view(np.float32).astype(F)
    global _POOL
    if _POOL is None:
        from concurrent.futures import ThreadPoolExecutor
        import os
        _POOL = ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1))
    out = np.empty(a.shape, dtype=F)
    n = a.shape[0]
    step = max(1, (n + 31) // 32)

    def widen(lo):
        hi = min(n, lo + step)
        out[lo:hi] = (a[lo:hi].astype(np.uint32) << 16).view(np.float32)

    list(_POOL.map(widen, range(0, n, step)))
    return out


class OracleModel:
    """shape: any object with n_layer, d_model, n_head, head_dim, d_ff, vocab,
    ffn_kind (0 GELU / 1 SwiGLU), norm_kind (0 LayerNorm / 1 RMSNorm),
    pos_kind (0 learned table / 1 rotary), rope_base, norm_eps.
    weights: dict as produced by the workload generator (row-major [out][in]).
    cache_layers=False converts one layer at a time to bound memory."""

    def __init__(self, shape, weights, cache_layers=True):
        self.s = shape
        self.w = weights
        self.tok_emb = weights["tok_emb"]
        self.pos_emb = weights.get("pos_emb")
        self.lm_head = None
        self.final_g = _to_f64(weights["final_norm_g"])
        self.final_b = _to_f64(weights.get("final_norm_b"))
        self._cache = {} if cache_layers else None

    # -- weights ---------------------------------------------------------
    def layer(self, l):
        if self._cache is not None and l in self._cache:
            return self._cache[l]
        lw = {k: _to_f64(v) for k, v in self.w["layers"][l].items()}
        if self._cache is not None:
            self._cache[l] = lw
        return lw

    def _lm(self):
        if self.lm_head is None:
            self.lm_head = _to_f64(self.w["lm_head"])
        return self.lm_head

    # -- per-token maps (x: [..., d]) -------------------------------------
    def norm(self, x, g, b):
        if self.s.norm_kind == 0:
            return P.layer_norm(x, g, b, self.s.norm_eps)
        return P.rms_norm(x, g, self.s.norm_eps)

    def embed(self, tokens, positions):
        """x0 = E_tok[token] (+ E_pos[p] for learned positions)."""
        tokens = np.asarray(tokens)
        x = _to_f64(self.tok_emb[tokens])
        if self.s.pos_kind == 0:
            x = x + _to_f64(self.pos_emb[np.asarray(positions)])
        return x

    def qkv(self, lw, x, positions):
        """x: [n, d] -> q, k, v each [n, H, hd]; rotary applied to q and k."""
        s = self.s
        u = self.norm(x, lw["norm1_g"], lw["norm1_b"])
        y = u @ lw["wqkv"].T
        n = x.shape[0]
        q, k, v = (y[:, i * s.d_model:(i + 1) * s.d_model].reshape(n, s.n_head, s.head_dim)
                   for i in range(3))
        if s.pos_kind == 1:
            pos = np.asarray(positions, dtype=F)[:, None]
            q = P.rope(q, pos, s.rope_base)
            k = P.rope(k, pos, s.rope_base)
        return q, k, v

    def after_attention(self, lw, x, attn):
        """attn: [n, H, hd] -> next residual stream [n, d]."""
        s = self.s
        h = x + attn.reshape(x.shape[0], s.d_model) @ lw["wo"].T
        u = self.norm(h, lw["norm2_g"], lw["norm2_b"])
        if s.ffn_kind == 0:
            f = P.gelu(u @ lw["w1"].T) @ lw["w2"].T
        else:
            f = (P.silu(u @ lw["w1"].T) * (u @ lw["w_up"].T)) @ lw["w2"].T
        return h + f

    def logits(self, x):
        return self.norm(x, self.final_g, self.final_b) @ self._lm().T

    # -- context pass (Eq. 1 analogue) --------------------------------------
    def prefill(self, ctx_tokens, progress=None):
        """Causal forward over the context tokens at positions 0..L-1.

        Returns (K, V): lists over layers of arrays [H, L, hd] — the keys and
        values (post-rotary) of every context token.  progress: optional callable
        invoked with the layer index after each layer (long runs report through it)."""
        s = self.s
        ctx_tokens = np.asarray(ctx_tokens)
        L = ctx_tokens.shape[0]
        if L == 0:      # no context: nothing to encode
            empty = np.zeros((s.n_head, 0, s.head_dim), dtype=F)
            return [empty] * s.n_layer, [empty] * s.n_layer
        pos = np.arange(L)
        x = self.embed(ctx_tokens, pos)
        Ks, Vs = [], []
        causal = np.tril(np.ones((L, L), dtype=bool))
        for l in range(s.n_layer):
            lw = self.layer(l)
            q, k, v = self.qkv(lw, x, pos)
            k_h = np.ascontiguousarray(k.transpose(1, 0, 2))
            v_h = np.ascontiguousarray(v.transpose(1, 0, 2))
            attn = np.empty((L, s.n_head, s.head_dim), dtype=F)
            for h in range(s.n_head):
                sc = (q[:, h, :] @ k_h[h].T) / np.sqrt(s.head_dim)
                sc = np.where(causal, sc, -np.inf)
                attn[:, h, :] = P.softmax(sc, axis=-1) @ v_h[h]
            x = self.after_attention(lw, x, attn)
            Ks.append(k_h)
            Vs.append(v_h)
            if progress is not None:
                progress(l)
        return Ks, Vs
