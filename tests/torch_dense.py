"""An independent dense transformer written with PyTorch library ops (fp64, CPU).

Used only to pin the oracle: it is the "textbook routine" (ordinary causal LM,
or a dense forward under an arbitrary boolean attention matrix and explicit
position ids).  It shares no code with oracle/ and none with the HIP path.
"""

import numpy as np
import torch
import torch.nn.functional as TF


def _t(a):
    if a is None:
        return None
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).double()
    return torch.from_numpy(np.ascontiguousarray(a)).double()


def _rope_complex(x, pos, base):
    """x [N, H, hd]: treat (x[j], x[j+hd/2]) as a complex number and multiply by e^{i p w_j}."""
    hd = x.shape[-1]
    half = hd // 2
    z = torch.complex(x[..., :half], x[..., half:])
    w = torch.pow(torch.tensor(float(base), dtype=torch.float64),
                  -torch.arange(half, dtype=torch.float64) * 2.0 / hd)
    ang = pos.double()[:, None, None] * w
    z = z * torch.polar(torch.ones_like(ang), ang)
    return torch.cat([z.real, z.imag], dim=-1)


def dense_logits(shape, weights, tokens, positions, mask=None):
    """tokens [N], positions [N], mask bool [N, N] (True = may attend) or None for causal.
    Returns fp64 logits [N, V] as numpy."""
    s = shape
    tokens = torch.as_tensor(np.asarray(tokens), dtype=torch.long)
    pos = torch.as_tensor(np.asarray(positions), dtype=torch.long)
    N = tokens.shape[0]
    x = TF.embedding(tokens, _t(weights["tok_emb"]))
    if s.pos_kind == 0:
        x = x + TF.embedding(pos, _t(weights["pos_emb"]))

    def norm(v, g, b):
        if s.norm_kind == 0:
            return TF.layer_norm(v, (s.d_model,), _t(g), _t(b), s.norm_eps)
        return TF.rms_norm(v, (s.d_model,), _t(g), s.norm_eps)

    am = None if mask is None else torch.as_tensor(np.asarray(mask), dtype=torch.bool)
    for lw in weights["layers"]:
        u = norm(x, lw["norm1_g"], lw["norm1_b"])
        qkv = TF.linear(u, _t(lw["wqkv"])).view(N, 3, s.n_head, s.head_dim)
        q, k, v = qkv[:, 0], qkv[:, 1], qkv[:, 2]
        if s.pos_kind == 1:
            q, k = _rope_complex(q, pos, s.rope_base), _rope_complex(k, pos, s.rope_base)
        o = TF.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1),
                                            attn_mask=am, is_causal=(am is None))
        x = x + TF.linear(o.transpose(0, 1).reshape(N, s.d_model), _t(lw["wo"]))
        u = norm(x, lw["norm2_g"], lw["norm2_b"])
        if s.ffn_kind == 0:
            f = TF.linear(TF.gelu(TF.linear(u, _t(lw["w1"]))), _t(lw["w2"]))
        else:
            f = TF.linear(TF.silu(TF.linear(u, _t(lw["w1"]))) * TF.linear(u, _t(lw["w_up"])),
                          _t(lw["w2"]))
        x = x + f
    x = norm(x, weights["final_norm_g"], weights.get("final_norm_b"))
    return TF.linear(x, _t(weights["lm_head"])).numpy()
