"""Formulation F2 of the pipelined decoder: at every iteration the whole flattened
sequence (context + every generated-side token) is recomputed from scratch under
one boolean attention matrix -- the teacher-forcing pattern of Fig. 3b applied at
inference.  Test infrastructure only; quadratic, for tiny inputs.

Coordinates come from the closed form of Section 3.2 instead of from bookkeeping:
token j (0 = <bos>) of subsequence i is fed at tau = (i-1)*dt + 1 + j.
mask[q, k] for generated-side rows is (i_k <= i_q) and (tau_k <= tau_q); context
columns are visible to every generated-side row; context rows are causal among
themselves and see nothing generated.
"""

import numpy as np

from . import primitives as P

F = np.float64


def coordinates(G, delta_t):
    """[(i, tau, token)] for every token of every subsequence of G."""
    out = []
    for i, g in enumerate(G, start=1):
        for j, tok in enumerate(g):
            out.append((i, (i - 1) * delta_t + 1 + j, tok))
    return out


def attention_matrix(L, coords):
    """Boolean [L+n, L+n] matrix; coords: [(i, tau, ...)] of the n generated-side tokens."""
    n = len(coords)
    mask = np.zeros((L + n, L + n), dtype=bool)
    mask[:L, :L] = np.tril(np.ones((L, L), dtype=bool))
    mask[L:, :L] = True
    for a, (iq, tq, *_) in enumerate(coords):
        for b, (ik, tk, *_) in enumerate(coords):
            mask[L + a, L + b] = (ik <= iq) and (tk <= tq)
    return mask


def dense_forward(model, tokens, positions, mask):
    """Full forward of all rows under a boolean attention matrix; returns logits [N, V]."""
    s = model.s
    x = model.embed(tokens, positions)
    N = x.shape[0]
    for l in range(s.n_layer):
        lw = model.layer(l)
        q, k, v = model.qkv(lw, x, positions)
        attn = np.empty((N, s.n_head, s.head_dim), dtype=F)
        for h in range(s.n_head):
            sc = q[:, h, :] @ k[:, h, :].T / np.sqrt(s.head_dim)
            sc = np.where(mask, sc, -np.inf)
            attn[:, h, :] = P.softmax(sc, axis=-1) @ v[:, h, :]
        x = model.after_attention(lw, x, attn)
    return model.logits(x)


class MatrixDecoder:
    """Callable decoder(G, t) for controller.pipelined_decode: full recompute."""

    def __init__(self, model, ctx_tokens, delta_t, force=None):
        self.m, self.ctx, self.dt = model, np.asarray(ctx_tokens), delta_t
        self.force = force
        self.trace = []

    def __call__(self, G, t):
        L = self.ctx.shape[0]
        coords = coordinates(G, self.dt)
        tokens = np.concatenate([self.ctx, np.array([c[2] for c in coords], dtype=np.int64)])
        positions = np.concatenate([np.arange(L),
                                    np.array([L + (tau - 1) + (i - 1) for i, tau, _ in coords],
                                             dtype=np.int64)])
        logits = dense_forward(self.m, tokens, positions, attention_matrix(L, coords))
        last, row = {}, L
        for i, g in enumerate(G, start=1):
            row += len(g)
            last[i] = row - 1
        out = [P.argmax_lowest(logits[last[i]]) for i in range(1, len(G) + 1)]
        self.trace.append({"t": t, "logits": {i: logits[last[i]] for i in last},
                           "last_tau": {i: coords_tau_last(G, i, self.dt) for i in last}})
        if self.force is not None and t - 1 < len(self.force):
            for i in range(1, len(G) + 1):
                f = int(self.force[t - 1][i - 1])
                if f >= 0:
                    out[i - 1] = f
        return out


def coords_tau_last(G, i, delta_t):
    return (i - 1) * delta_t + len(G[i - 1])
