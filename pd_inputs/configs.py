"""Workload descriptions: model shape + decode parameters + seed.

The five named workloads stand in for the paper's datasets (Table 1: a long
input, a target of tens to hundreds of tokens split into several subsequences);
every subsequence has the same length M and the end-of-sequence token is
disabled, so a run produces exactly S*M tokens per request.
"""

from dataclasses import dataclass, replace

FFN_GELU, FFN_SWIGLU = 0, 1
NORM_LAYERNORM, NORM_RMSNORM = 0, 1
POS_LEARNED, POS_ROPE = 0, 1
DTYPE_F32, DTYPE_BF16 = 0, 1


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    seed: int
    dtype: int          # DTYPE_F32 | DTYPE_BF16 (weights and KV cache; accumulation is fp32)
    n_layer: int
    d_model: int
    n_head: int
    head_dim: int
    d_ff: int
    vocab: int
    ffn_kind: int = FFN_GELU
    norm_kind: int = NORM_LAYERNORM
    pos_kind: int = POS_LEARNED
    rope_base: float = 10000.0
    norm_eps: float = 1e-5
    bos_id: int = 0
    eos_id: int = -1    # < 0: end-of-sequence termination disabled
    # decode parameters
    batch: int = 1      # B independent requests
    ctx_len: int = 128  # L
    n_sub: int = 4      # S = sub^max
    delta_t: int = 2    # delay between subsequence starts
    sub_tokens: int = 16  # M = per-subsequence token limit
    # norm parameters: "identity" (gain 1, bias 0) or "random"
    norm_init: str = "identity"
    # standard deviation of the QKV projection (0.02 everywhere in the named workloads; test
    # cases raise it to make the attention distribution peaky, so that mask errors show)
    qkv_std: float = 0.02
    # standard deviation of the vocabulary projection (0.02 in the named workloads; test cases raise
    # it so that the top-2 logit margins of a whole free-running generation stay clear of rounding)
    lm_std: float = 0.02

    @property
    def time_steps(self) -> int:
        """Time-steps of a full run with EOS disabled: (S-1)*dt + M."""
        return (self.n_sub - 1) * self.delta_t + self.sub_tokens

    def scaled(self, **kw) -> "WorkloadConfig":
        return replace(self, **kw)


def max_positions(cfg: WorkloadConfig) -> int:
    """Rows of the learned position table: largest position index + 1.

    A token of subsequence i (1-based) fed at time-step tau sits at position
    L + (tau-1) + (i-1); the last token of the last subsequence has
    tau = (S-1)*dt + M + 1.
    """
    return cfg.ctx_len + (cfg.n_sub - 1) * (cfg.delta_t + 1) + cfg.sub_tokens + 1


CONFIGS = {
    "cfg1": WorkloadConfig(
        name="cfg1", seed=0, dtype=DTYPE_F32, n_layer=1, d_model=64, n_head=4, head_dim=16,
        d_ff=256, vocab=512, batch=1, ctx_len=128, n_sub=4, delta_t=2, sub_tokens=16),
    "cfg2": WorkloadConfig(
        name="cfg2", seed=1, dtype=DTYPE_BF16, n_layer=6, d_model=768, n_head=12, head_dim=64,
        d_ff=3072, vocab=50265, batch=1, ctx_len=1024, n_sub=8, delta_t=4, sub_tokens=64),
    "cfg3": WorkloadConfig(
        name="cfg3", seed=2, dtype=DTYPE_BF16, n_layer=12, d_model=1024, n_head=16, head_dim=64,
        d_ff=4096, vocab=50265, batch=8, ctx_len=2048, n_sub=16, delta_t=4, sub_tokens=32),
    "cfg4": WorkloadConfig(
        name="cfg4", seed=3, dtype=DTYPE_BF16, n_layer=24, d_model=2048, n_head=16, head_dim=128,
        d_ff=8192, vocab=32000, batch=1, ctx_len=8192, n_sub=32, delta_t=8, sub_tokens=64),
    "cfg5": WorkloadConfig(
        name="cfg5", seed=4, dtype=DTYPE_BF16, n_layer=32, d_model=4096, n_head=32, head_dim=128,
        d_ff=11008, vocab=32000, ffn_kind=FFN_SWIGLU, norm_kind=NORM_RMSNORM, pos_kind=POS_ROPE,
        rope_base=10000.0, batch=4, ctx_len=4096, n_sub=16, delta_t=4, sub_tokens=128),
}


def get_config(name: str) -> WorkloadConfig:
    return CONFIGS[name]


@dataclass(frozen=True)
class EncDecConfig:
    """Encoder-decoder workload (the kind of backbone the paper itself runs, Section 4.3): a stacked
    encoder over the input, a decoder with self-attention over the generated side, cross-attention
    over the encoder states and bucketed relative-position biases."""
    name: str
    seed: int
    n_enc_layer: int
    n_dec_layer: int
    d_model: int
    n_head: int
    head_dim: int       # n_head * head_dim need not equal d_model in this family
    d_ff: int
    vocab: int
    rel_buckets: int = 32
    rel_max_distance: int = 128
    norm_eps: float = 1e-6
    bos_id: int = 0
    eos_id: int = -1
    ctx_len: int = 16
    n_sub: int = 3
    delta_t: int = 1
    sub_tokens: int = 4
    batch: int = 1

    @property
    def time_steps(self) -> int:
        return (self.n_sub - 1) * self.delta_t + self.sub_tokens

    def scaled(self, **kw) -> "EncDecConfig":
        return replace(self, **kw)


def _encdec(name, seed, layers, d, heads, ff):
    return EncDecConfig(name=name, seed=seed, n_enc_layer=layers, n_dec_layer=layers, d_model=d, n_head=heads,
                        head_dim=64, d_ff=ff, vocab=32128, rel_buckets=32, rel_max_distance=128, ctx_len=512,
                        n_sub=8, delta_t=1, sub_tokens=16, batch=1)


# Shapes of the backbone family the paper runs (Section 5.1: the base and the large size; inference
# batch size 1); weights are random, only the dimensions are the family's published ones.
ENCDEC_CONFIGS = {
    "encdec-small": _encdec("encdec-small", 71, 6, 512, 8, 2048),
    "encdec-base": _encdec("encdec-base", 72, 12, 768, 12, 3072),
    "encdec-large": _encdec("encdec-large", 73, 24, 1024, 16, 4096),
}
