"""Seeded generators for weights and context token ids.

Every tensor is drawn from its own counter-based (Philox) streams keyed by
(seed, tensor id, chunk index), in fixed-size chunks, so the values do not
depend on how many threads fill them.  Matrices are N(0, 0.02); for bf16
workloads they are rounded once to bf16 (round-to-nearest-even) and handed out
as raw 16-bit patterns.  Norm gains/biases stay fp32.
"""

from concurrent.futures import ThreadPoolExecutor
import os

import numpy as np

from .configs import (WorkloadConfig, DTYPE_BF16, FFN_SWIGLU, NORM_LAYERNORM, POS_LEARNED,
                      max_positions)

_CHUNK = 1 << 22
_STD = 0.02


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 bf16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounding = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + rounding) >> 16).astype(np.uint16)


def bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float32 values (exact)."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16, returned as float32."""
    return bits_to_f32(bf16_bits(x))


def _fill_chunk(out_flat, lo, hi, seed, tensor_id, chunk, std, as_bf16):
    bitgen = np.random.Philox(key=[(seed << 32) | tensor_id, chunk])
    g = np.random.Generator(bitgen)
    z = g.standard_normal(hi - lo, dtype=np.float32)
    z *= np.float32(std)
    if as_bf16:
        out_flat[lo:hi] = bf16_bits(z)
    else:
        out_flat[lo:hi] = z


def _normal(shape, seed, tensor_id, as_bf16, pool, std=_STD, mean=0.0):
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16 if as_bf16 else np.float32)
    jobs = []
    for c, lo in enumerate(range(0, n, _CHUNK)):
        hi = min(n, lo + _CHUNK)
        jobs.append(pool.submit(_fill_chunk, out, lo, hi, seed, tensor_id, c, std, as_bf16))
    for j in jobs:
        j.result()
    out = out.reshape(shape)
    if mean != 0.0:
        assert not as_bf16
        out += np.float32(mean)
    return out


def make_weights(cfg: WorkloadConfig, threads: int | None = None) -> dict:
    """Draw all weights of `cfg`.

    Returns a dict: "tok_emb" [V,d], "pos_emb" [max_pos,d] (learned positions only),
    "lm_head" [V,d], "final_norm_g"/"final_norm_b" [d], and "layers": a list of
    dicts with "wqkv" [3d,d], "wo" [d,d], "w1" [ff,d] (GELU up / SwiGLU gate),
    "w_up" [ff,d] (SwiGLU only), "w2" [d,ff], "norm1_g/b", "norm2_g/b" [d].
    All matrices are row-major [out][in]; uint16 bf16 bit patterns when
    cfg.dtype is bf16, float32 otherwise.  Norm vectors are float32; biases are
    present for LayerNorm only.
    """
    as_bf16 = cfg.dtype == DTYPE_BF16
    threads = threads or min(16, os.cpu_count() or 1)
    d, ff, V = cfg.d_model, cfg.d_ff, cfg.vocab
    assert cfg.n_head * cfg.head_dim == d
    random_norm = cfg.norm_init == "random"
    with ThreadPoolExecutor(max_workers=threads) as pool:
        tid = iter(range(1, 1 << 20))

        def mat(*shape):
            return _normal(shape, cfg.seed, next(tid), as_bf16, pool)

        def gain():
            t = next(tid)
            if random_norm:
                return _normal((d,), cfg.seed, t, False, pool, std=0.1, mean=1.0)
            return np.ones(d, dtype=np.float32)

        def bias():
            t = next(tid)
            if cfg.norm_kind != NORM_LAYERNORM:
                return None
            if random_norm:
                return _normal((d,), cfg.seed, t, False, pool, std=0.1)
            return np.zeros(d, dtype=np.float32)

        w = {"tok_emb": mat(V, d)}
        t_pos = next(tid)
        if cfg.pos_kind == POS_LEARNED:
            w["pos_emb"] = _normal((max_positions(cfg), d), cfg.seed, t_pos, as_bf16, pool)
        w["lm_head"] = _normal((V, d), cfg.seed, next(tid), as_bf16, pool, std=cfg.lm_std)
        w["final_norm_g"] = gain()
        w["final_norm_b"] = bias()
        layers = []
        for _ in range(cfg.n_layer):
            lw = {"wqkv": _normal((3 * d, d), cfg.seed, next(tid), as_bf16, pool, std=cfg.qkv_std),
                  "wo": mat(d, d), "w1": mat(ff, d)}
            t_up = next(tid)
            if cfg.ffn_kind == FFN_SWIGLU:
                lw["w_up"] = _normal((ff, d), cfg.seed, t_up, as_bf16, pool)
            lw["w2"] = mat(d, ff)
            lw["norm1_g"], lw["norm1_b"] = gain(), bias()
            lw["norm2_g"], lw["norm2_b"] = gain(), bias()
            layers.append(lw)
        w["layers"] = layers
    return w


def make_context(cfg: WorkloadConfig) -> np.ndarray:
    """Context token ids, int32 [B][L], uniform in [0, vocab)."""
    g = np.random.Generator(np.random.Philox(key=[(cfg.seed << 32) | 0xC0DE, 0]))
    return g.integers(0, cfg.vocab, size=(cfg.batch, cfg.ctx_len), dtype=np.int32)


def make_forced_tokens(cfg: WorkloadConfig, steps: int, salt: int = 1) -> np.ndarray:
    """Arbitrary token ids, int32 [steps][B][S], uniform in [0, vocab): a seeded
    stand-in for "the tokens that were generated", for teacher-forced runs."""
    g = np.random.Generator(np.random.Philox(key=[(cfg.seed << 32) | 0xF0CE, salt]))
    return g.integers(0, cfg.vocab, size=(steps, cfg.batch, cfg.n_sub), dtype=np.int32)


def tie_lm_head(cfg: WorkloadConfig, weights: dict, group_a, group_b, scale: float = 100.0) -> None:
    """Overwrites rows of the vocabulary projection in place so that logits tie exactly: every row
    listed in group_a becomes one seeded vector v (N(0, scale * 0.02)), every row in group_b becomes
    -v.  Whatever the hidden state, one of the two groups then holds the largest logit several
    times over (an input for the tests of the lowest-index rule of Eq. 4)."""
    g = np.random.Generator(np.random.Philox(key=[(cfg.seed << 32) | 0x71E5, 0]))
    v = (g.standard_normal(cfg.d_model, dtype=np.float32) * np.float32(scale * _STD))
    head = weights["lm_head"]
    if head.dtype == np.uint16:
        pos, neg = bf16_bits(v), bf16_bits(-v)
    else:
        pos, neg = v, -v
    for j in group_a:
        head[j] = pos
    for j in group_b:
        head[j] = neg


def make_encdec_weights(cfg, threads: int = 2) -> dict:
    """Weights of an encoder-decoder workload (float32, row-major [out][in]):
    "tok_emb" [V,d] shared by both stacks, "lm_head" [V,d], "enc_rel_bias"/"dec_rel_bias"
    [buckets, H] (one table per stack, used by all its layers), "enc_final_g"/"dec_final_g" [d],
    "enc_layers": dicts with "wq","wk","wv" [H*hd,d], "wo" [d,H*hd], "w1" [ff,d], "w2" [d,ff],
    "norm1_g","norm2_g" [d]; "dec_layers": the same plus "cq","ck","cv","co" (cross-attention) and
    "norm3_g".
    Scales follow the published initialisation of the backbone family, which is what keeps its
    unscaled attention scores (no 1/sqrt(head_dim) factor) of order one: query projections
    N(0, 1/(d*hd)), every other projection N(0, 1/fan_in), embeddings N(0, 1), the vocabulary
    projection N(0, 1/d); biases N(0, 0.5), gains 1 + N(0, 0.1)."""
    d, ff, V, inner = cfg.d_model, cfg.d_ff, cfg.vocab, cfg.n_head * cfg.head_dim
    with ThreadPoolExecutor(max_workers=threads) as pool:
        tid = iter(range(1, 1 << 20))

        def mat(*shape, std):
            return _normal(shape, cfg.seed, next(tid), False, pool, std=std)

        def gain():
            return _normal((d,), cfg.seed, next(tid), False, pool, std=0.1, mean=1.0)

        sq, sd, sf, si = (d * cfg.head_dim) ** -0.5, d ** -0.5, ff ** -0.5, inner ** -0.5

        def layer(cross):
            lw = {"wq": mat(inner, d, std=sq), "wk": mat(inner, d, std=sd), "wv": mat(inner, d, std=sd),
                  "wo": mat(d, inner, std=si), "w1": mat(ff, d, std=sd), "w2": mat(d, ff, std=sf),
                  "norm1_g": gain(), "norm2_g": gain()}
            if cross:
                lw.update({"cq": mat(inner, d, std=sq), "ck": mat(inner, d, std=sd), "cv": mat(inner, d, std=sd),
                           "co": mat(d, inner, std=si), "norm3_g": gain()})
            return lw

        w = {"tok_emb": mat(V, d, std=1.0), "lm_head": mat(V, d, std=sd),
             "enc_rel_bias": mat(cfg.rel_buckets, cfg.n_head, std=0.5),
             "dec_rel_bias": mat(cfg.rel_buckets, cfg.n_head, std=0.5),
             "enc_final_g": gain(), "dec_final_g": gain()}
        w["enc_layers"] = [layer(False) for _ in range(cfg.n_enc_layer)]
        w["dec_layers"] = [layer(True) for _ in range(cfg.n_dec_layer)]
    return w


_ENCDEC_MATRICES = ("wq", "wk", "wv", "wo", "w1", "w2", "cq", "ck", "cv", "co")


def encdec_to_bf16(weights: dict):
    """The encoder-decoder weights once as the bf16 kernels take them and once as the values those
    bit patterns stand for.  Returns (rounded, device): `rounded` has the layout of
    make_encdec_weights with every matrix rounded to bf16 (float32 arrays); `device` holds the same
    matrices as uint16 bf16 bit patterns with the three self-attention projections stacked as
    "wqkv" [3 inner][d] (queries, keys, values) and the key and value projections over the encoder
    states as "ckv" [2 inner][d]; gains and bias tables stay float32 in both."""
    rounded = {k: (bf16_round(v) if k in ("tok_emb", "lm_head") else v) for k, v in weights.items()
               if k not in ("enc_layers", "dec_layers")}
    device = {k: (bf16_bits(v) if k in ("tok_emb", "lm_head") else v) for k, v in weights.items()
              if k not in ("enc_layers", "dec_layers")}
    for group in ("enc_layers", "dec_layers"):
        rounded[group], device[group] = [], []
        for lw in weights[group]:
            r = {k: (bf16_round(v) if k in _ENCDEC_MATRICES else v) for k, v in lw.items()}
            dv = {k: v for k, v in lw.items() if k not in _ENCDEC_MATRICES}
            dv["wqkv"] = bf16_bits(np.concatenate([lw["wq"], lw["wk"], lw["wv"]], axis=0))
            for k in ("wo", "w1", "w2"):
                dv[k] = bf16_bits(lw[k])
            if "cq" in lw:
                dv["cq"] = bf16_bits(lw["cq"])
                dv["ckv"] = bf16_bits(np.concatenate([lw["ck"], lw["cv"]], axis=0))
                dv["co"] = bf16_bits(lw["co"])
            rounded[group].append(r)
            device[group].append(dv)
    return rounded, device
