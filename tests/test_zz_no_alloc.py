"""pd_generate_static (the entry point for callers that cannot allocate device memory) against
pd_create + pd_generate: same tokens, lengths and step counts, bit for bit, on two calls in a row,
the second with a smaller input (fewer requests, a shorter context, fewer and shorter subsequences, a
narrower model), so that whatever the first call left in the library's static workspace would show."""

import numpy as np
import pytest

import pd_inputs as pi
from pd_inputs import max_positions
from pd_inputs.configs import WorkloadConfig, DTYPE_BF16, DTYPE_F32, FFN_SWIGLU, NORM_RMSNORM, POS_ROPE

pytestmark = pytest.mark.gpu

BIG = WorkloadConfig(name="static-first", seed=91, dtype=DTYPE_BF16, n_layer=2, d_model=256, n_head=2,
                     head_dim=128, d_ff=352, vocab=777, batch=3, ctx_len=200, n_sub=6, delta_t=2,
                     sub_tokens=9, norm_init="random", qkv_std=0.1, ffn_kind=FFN_SWIGLU,
                     norm_kind=NORM_RMSNORM, pos_kind=POS_ROPE)
SMALL = WorkloadConfig(name="static-second", seed=92, dtype=DTYPE_BF16, n_layer=1, d_model=128, n_head=2,
                       head_dim=64, d_ff=256, vocab=517, batch=1, ctx_len=70, n_sub=3, delta_t=1,
                       sub_tokens=4, norm_init="random", qkv_std=0.1)
F32 = WorkloadConfig(name="static-fp32", seed=93, dtype=DTYPE_F32, n_layer=2, d_model=48, n_head=4,
                     head_dim=12, d_ff=80, vocab=203, batch=2, ctx_len=37, n_sub=5, delta_t=2,
                     sub_tokens=6, norm_init="random", qkv_std=0.3)


def reference(cfg, w, ctx):
    from paper_2506_23431_amd import PipelinedDecoder
    dec = PipelinedDecoder(cfg, w, max_batch=cfg.batch, max_ctx=cfg.ctx_len, max_sub=cfg.n_sub,
                           max_sub_tokens=cfg.sub_tokens, max_pos=max_positions(cfg))
    out = dec.generate(ctx, cfg.n_sub, cfg.delta_t, cfg.sub_tokens, cfg.time_steps)
    dec.close()
    return out


def test_static_workspace_generate_matches_pd_generate_twice_in_a_row():
    from paper_2506_23431_amd import binding
    cases = []
    for cfg in (BIG, SMALL, F32, BIG):
        w = pi.make_weights(cfg, threads=4)
        ctx = pi.make_context(cfg)
        cases.append((cfg, w, ctx, reference(cfg, w, ctx)))
    # the calls under test, back to back: large, smaller, the fp32 kernels, large again
    for cfg, w, ctx, want in cases:
        got = binding.generate_static(cfg, w, ctx, cfg.n_sub, cfg.delta_t, cfg.sub_tokens, cfg.time_steps,
                                      max_positions(cfg))
        for name, a, b in zip(("tokens", "lengths", "steps"), want, got):
            assert np.array_equal(a, b), f"{cfg.name}: {name} differ from pd_generate's"
        assert got[2].tolist() == [cfg.time_steps] * cfg.batch
        assert int((got[0] >= 0).sum()) == cfg.batch * cfg.n_sub * cfg.sub_tokens


def test_static_workspace_rejects_what_does_not_fit():
    from paper_2506_23431_amd import binding, PdError
    cfg = pi.get_config("cfg2")          # 162 MB of weights alone
    w = {"tok_emb": None, "pos_emb": None, "lm_head": None, "final_norm_g": None, "final_norm_b": None,
         "layers": [{} for _ in range(cfg.n_layer)]}
    ctx = np.zeros((1, 8), dtype=np.int32)
    with pytest.raises(PdError, match="static workspace"):
        binding.generate_static(cfg, w, ctx, 2, 1, 2, 3, max_positions(cfg))
