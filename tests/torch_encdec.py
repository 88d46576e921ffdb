"""An independent dense encoder-decoder written with PyTorch library ops (fp64, CPU): the textbook
routine the encoder-decoder oracle is pinned against.  Shares no code with oracle/.

The relative-position bucket is computed differently from the oracle on purpose: from a table of
bucket boundaries in closed form (bucket b >= max_exact starts at the smallest n with
n >= max_exact * (max_distance / max_exact) ** ((b - max_exact) / (buckets - max_exact))),
looked up with a sorted search."""

import numpy as np
import torch
import torch.nn.functional as TF


def _t(a):
    return torch.from_numpy(np.ascontiguousarray(a)).double()


def bucket_table(buckets, max_distance, n_max):
    """bucket of every distance 0..n_max (keys behind the query), by boundaries."""
    max_exact = buckets // 2
    ratio = max_distance / max_exact
    starts = [max_exact * ratio ** ((b - max_exact) / (buckets - max_exact)) for b in range(max_exact, buckets)]
    n = np.arange(n_max + 1)
    large = max_exact + np.searchsorted(np.array(starts), n, side="right") - 1
    return np.where(n < max_exact, n, np.minimum(large, buckets - 1))


def _attend(q, k, v, add):
    """q [Nq,H,hd], k,v [Nk,H,hd], add: float [H,Nq,Nk] additive term (-inf = masked) or None."""
    o = TF.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1),
                                        attn_mask=add, scale=1.0)
    return o.transpose(0, 1).reshape(q.shape[0], -1)


def encode(cfg, w, ctx_tokens):
    n = len(ctx_tokens)
    x = TF.embedding(torch.as_tensor(np.asarray(ctx_tokens), dtype=torch.long), _t(w["tok_emb"]))
    half = cfg.rel_buckets // 2
    tab = bucket_table(half, cfg.rel_max_distance, n)
    rel = np.arange(n)[None, :] - np.arange(n)[:, None]
    idx = np.where(rel > 0, half, 0) + tab[np.abs(rel)]
    add = _t(w["enc_rel_bias"])[torch.as_tensor(idx)].permute(2, 0, 1)
    H, hd = cfg.n_head, cfg.head_dim
    for lw in w["enc_layers"]:
        u = TF.rms_norm(x, (cfg.d_model,), _t(lw["norm1_g"]), cfg.norm_eps)
        q, k, v = (TF.linear(u, _t(lw[m])).view(n, H, hd) for m in ("wq", "wk", "wv"))
        x = x + TF.linear(_attend(q, k, v, add), _t(lw["wo"]))
        u = TF.rms_norm(x, (cfg.d_model,), _t(lw["norm2_g"]), cfg.norm_eps)
        x = x + TF.linear(TF.relu(TF.linear(u, _t(lw["w1"]))), _t(lw["w2"]))
    return TF.rms_norm(x, (cfg.d_model,), _t(w["enc_final_g"]), cfg.norm_eps)


def decode_logits(cfg, w, HE, tokens, mask, distance):
    """All generated-side tokens in one dense forward.  mask bool [N,N] (query, key),
    distance int [N,N]: how far the key lies behind the query.  Returns numpy [N, V]."""
    N = len(tokens)
    H, hd = cfg.n_head, cfg.head_dim
    x = TF.embedding(torch.as_tensor(np.asarray(tokens), dtype=torch.long), _t(w["tok_emb"]))
    d = np.where(mask, distance, 0)
    tab = bucket_table(cfg.rel_buckets, cfg.rel_max_distance, int(d.max()))
    add = _t(w["dec_rel_bias"])[torch.as_tensor(tab[d])].permute(2, 0, 1).clone()
    add.masked_fill_(~torch.as_tensor(mask)[None], float("-inf"))
    n_ctx = HE.shape[0]
    for lw in w["dec_layers"]:
        u = TF.rms_norm(x, (cfg.d_model,), _t(lw["norm1_g"]), cfg.norm_eps)
        q, k, v = (TF.linear(u, _t(lw[m])).view(N, H, hd) for m in ("wq", "wk", "wv"))
        x = x + TF.linear(_attend(q, k, v, add), _t(lw["wo"]))
        u = TF.rms_norm(x, (cfg.d_model,), _t(lw["norm3_g"]), cfg.norm_eps)
        q = TF.linear(u, _t(lw["cq"])).view(N, H, hd)
        k, v = (TF.linear(HE, _t(lw[m])).view(n_ctx, H, hd) for m in ("ck", "cv"))
        x = x + TF.linear(_attend(q, k, v, None), _t(lw["co"]))
        u = TF.rms_norm(x, (cfg.d_model,), _t(lw["norm2_g"]), cfg.norm_eps)
        x = x + TF.linear(TF.relu(TF.linear(u, _t(lw["w1"]))), _t(lw["w2"]))
    x = TF.rms_norm(x, (cfg.d_model,), _t(w["dec_final_g"]), cfg.norm_eps)
    return TF.linear(x, _t(w["lm_head"])).numpy()
