"""Formulation F1 of the pipelined decoder: an incremental per-query loop with an
explicit visible set per query.  Test infrastructure only.

Coordinates.  Every generated-side token has a grid coordinate (i, tau): i is its
subsequence (1-based) and tau the time-step at which it is FED to the decoder.
<bos> of subsequence i is fed at the step that opens it, tau = (i-1)*dt + 1; the
token produced in iteration t is fed in iteration t+1 (the superscript t+1 of
Eq. 3), so it has tau = t+1.

Dependency rule (Section 3.2): the token of subsequence i produced in iteration t
depends on the first i subsequences as generated so far and on the whole input.
Hence the query of row (i, t) sees every context token plus every generated-side
token (i', tau') with i' <= i and tau' <= t -- including the tokens that the
lower-numbered subsequences feed in this very iteration, and itself.

Readings where the paper is silent
  * Decoder-only: the context is a causal prefix encoded once (model.prefill);
    context and generated keys share one softmax.
  * Position index of (i, tau) is p = L + (tau-1) + (i-1).  On every visible pair
    the paper's Manhattan distance |dtau| + |di| (Section 4.3) equals p_q - p_k.
  * The last token of a finished subsequence is still fed once, in the following
    iteration, so that later subsequences can see it ("draining" row: its keys and
    values are stored, no token is produced from it).
"""

import numpy as np

from . import primitives as P
from .controller import pipelined_decode

F = np.float64


def position(L, i, tau):
    return L + (tau - 1) + (i - 1)


class PerQueryDecoder:
    """Callable decoder(G, t) for controller.pipelined_decode, backed by the model.

    keep: if true, self.trace gets one record per iteration with the rows fed, their
    positions, visible sets and logits.
    row_order: optional function mapping the list of row subsequence indices to a
    processing order (used to check that the order within a step is irrelevant).
    force: optional int array [steps][S]; where >= 0 it replaces the argmax result
    of that iteration (teacher forcing).  The logits are unaffected.
    context_kv: optional precomputed (K, V) lists to use instead of the causal pass.
    """

    def __init__(self, model, ctx_tokens, keep=True, row_order=None, force=None,
                 context_kv=None):
        self.m = model
        s = model.s
        self.L = int(np.asarray(ctx_tokens).shape[0])
        self.Kc, self.Vc = context_kv if context_kv is not None else model.prefill(ctx_tokens)
        self.gen_sub, self.gen_tau = [], []                 # coordinates of cached tokens
        self.gen_K = [[] for _ in range(s.n_layer)]          # per layer: list of [H, hd]
        self.gen_V = [[] for _ in range(s.n_layer)]
        self.encoded = []                                    # tokens already fed, per subsequence
        self.keep, self.trace = keep, []
        self.row_order = row_order
        self.force = force

    def visible(self, i, t):
        """Indices into the generated-side cache that query (i, t) may attend to."""
        return [n for n in range(len(self.gen_sub))
                if self.gen_sub[n] <= i and self.gen_tau[n] <= t]

    def _attend(self, l, q, idx):
        """q: [H, hd]; joint softmax over all context keys and the cached keys idx."""
        hd = q.shape[-1]
        s_ctx = (self.Kc[l] @ q[:, :, None])[:, :, 0]                       # [H, L]
        if idx:
            Kg = np.stack([self.gen_K[l][n] for n in idx], axis=1)           # [H, n, hd]
            Vg = np.stack([self.gen_V[l][n] for n in idx], axis=1)
            s_gen = (Kg @ q[:, :, None])[:, :, 0]
        else:
            Vg = np.zeros((q.shape[0], 0, hd), dtype=F)
            s_gen = np.zeros((q.shape[0], 0), dtype=F)
        w = P.softmax(np.concatenate([s_ctx, s_gen], axis=1) / np.sqrt(hd), axis=1)
        L = s_ctx.shape[1]
        return (w[:, None, :L] @ self.Vc[l])[:, 0, :] + (w[:, None, L:] @ Vg)[:, 0, :]

    def __call__(self, G, t):
        s = self.m.s
        k = len(G)
        while len(self.encoded) < k:
            self.encoded.append(0)
        rows = [i for i in range(1, k + 1) if len(G[i - 1]) > self.encoded[i - 1]]
        if self.row_order is not None:
            rows = list(self.row_order(rows))
        for i in rows:
            assert len(G[i - 1]) == self.encoded[i - 1] + 1, "exactly one unfed token per row"
        toks = [G[i - 1][-1] for i in rows]
        pos = [position(self.L, i, t) for i in rows]
        out = [None] * k
        rec = {"t": t, "rows": list(rows), "tokens_in": toks, "positions": pos}
        if rows:
            x = self.m.embed(toks, pos)
            base = len(self.gen_sub)
            for i in rows:
                self.gen_sub.append(i)
                self.gen_tau.append(t)
            vis = [self.visible(i, t) for i in rows]
            for l in range(s.n_layer):
                lw = self.m.layer(l)
                q, kk, vv = self.m.qkv(lw, x, pos)
                for r in range(len(rows)):                    # all keys/values first ...
                    self.gen_K[l].append(kk[r])
                    self.gen_V[l].append(vv[r])
                attn = np.empty_like(q)
                for r in range(len(rows)):                    # ... then one query at a time
                    attn[r] = self._attend(l, q[r], vis[r])
                x = self.m.after_attention(lw, x, attn)
            logits = self.m.logits(x)
            for r, i in enumerate(rows):
                out[i - 1] = P.argmax_lowest(logits[r])
                self.encoded[i - 1] += 1
            if self.keep:
                rec["logits"] = logits
                rec["vis"] = [[(self.gen_sub[n], self.gen_tau[n]) for n in v] for v in vis]
                rec["argmax"] = [out[i - 1] for i in rows]
            assert base + len(rows) == len(self.gen_sub)
        if self.force is not None and t - 1 < len(self.force):
            for i in range(1, k + 1):
                f = int(self.force[t - 1][i - 1])
                if f >= 0:
                    out[i - 1] = f
        if self.keep:
            self.trace.append(rec)
        return [o if o is not None else -1 for o in out]


def generate(model, ctx_tokens, n_sub, delta_t, sub_tokens, time_max, bos_id, eos_id=-1,
             force=None, keep=True, row_order=None, context_kv=None):
    """Pipelined generation for one request.  Returns a dict with
    result (subsequences without <bos>/<eos>), steps, emitted (per iteration
    {subsequence: token}) and trace (per iteration rows/positions/vis/logits)."""
    dec = PerQueryDecoder(model, ctx_tokens, keep=keep, row_order=row_order, force=force,
                          context_kv=context_kv)
    result, steps, emitted = pipelined_decode(dec, delta_t, time_max, n_sub, bos_id, eos_id,
                                              sub_tokens)
    return {"result": result, "steps": steps, "emitted": emitted, "trace": dec.trace,
            "decoder": dec}
