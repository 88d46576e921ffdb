"""GPU parity: the HIP library against the CPU oracle, element by element, through the C ABI.
Small and medium workloads that the oracle finishes in seconds: several tiles, ragged tails,
both code paths (fp32-activation kernels and bf16 MFMA kernels), all block variants."""

import numpy as np
import pytest

import pd_inputs as pi
from pd_inputs.configs import (WorkloadConfig, DTYPE_F32, DTYPE_BF16, FFN_SWIGLU, NORM_RMSNORM, POS_ROPE)
from parity_util import oracle_run, make_decoder, compare_teacher_forced

pytestmark = pytest.mark.gpu


def say(msg):
    """Progress line on stdout (run pytest with -s to see the lines of a long case as they come)."""
    print(msg, flush=True)


def small(name, **kw):
    base = dict(name=name, seed=21, dtype=DTYPE_F32, n_layer=2, d_model=48, n_head=4, head_dim=12,
                d_ff=80, vocab=203, batch=2, ctx_len=37, n_sub=5, delta_t=2, sub_tokens=6,
                norm_init="random", qkv_std=0.3)
    base.update(kw)
    if base["dtype"] == DTYPE_BF16 and "qkv_std" not in kw:
        # bf16 rounding of q and k scales with the score magnitude: keep the attention peaky
        # (score std about 1) but within what the 2e-2 logit tolerance can resolve
        base["qkv_std"] = 0.1
    return WorkloadConfig(**base)


LLAMA = dict(ffn_kind=FFN_SWIGLU, norm_kind=NORM_RMSNORM, pos_kind=POS_ROPE)

CASES = {
    # fp32 kernels
    "cfg1": pi.get_config("cfg1"),
    "f32-ragged": small("f32-ragged"),
    "f32-llama": small("f32-llama", seed=22, **LLAMA),
    "f32-dt1": small("f32-dt1", seed=23, delta_t=1, n_sub=6, sub_tokens=4, batch=1),
    # bf16 weights on the fp32-activation kernels (head_dim not a multiple of 32)
    "bf16-simple": small("bf16-simple", seed=24, dtype=DTYPE_BF16, head_dim=12),
    # bf16 MFMA kernels: head_dim 32 / 64 / 128, vocab not a multiple of 16, context not a
    # multiple of the 32-key block, more than 16 rows, rotary + SwiGLU, peaky attention
    "mfma-hd64": small("mfma-hd64", seed=25, dtype=DTYPE_BF16, d_model=128, n_head=2, head_dim=64,
                       d_ff=256, vocab=1003, ctx_len=150, n_sub=5, delta_t=2, sub_tokens=7),
    "mfma-hd32": small("mfma-hd32", seed=26, dtype=DTYPE_BF16, d_model=96, n_head=3, head_dim=32,
                       d_ff=160, vocab=517, ctx_len=75, n_sub=4, delta_t=1, sub_tokens=5, batch=3),
    "mfma-hd96": small("mfma-hd96", seed=32, dtype=DTYPE_BF16, d_model=192, n_head=2, head_dim=96,
                       d_ff=224, vocab=611, ctx_len=110, n_sub=5, delta_t=2, sub_tokens=8, batch=2),
    "mfma-hd128-llama": small("mfma-hd128-llama", seed=27, dtype=DTYPE_BF16, d_model=256, n_head=2,
                              head_dim=128, d_ff=352, vocab=777, ctx_len=200, n_sub=6, delta_t=2,
                              sub_tokens=9, batch=2, **LLAMA),
    "mfma-manyrows": small("mfma-manyrows", seed=28, dtype=DTYPE_BF16, d_model=128, n_head=2,
                           head_dim=64, d_ff=256, vocab=640, ctx_len=97, n_sub=20, delta_t=1,
                           sub_tokens=24, batch=2, n_layer=1),
    # one request, at most 5 rows: every step keeps its activations as packed pairs (rotary, SwiGLU, RMSNorm)
    "mfma-llama-packed": small("mfma-llama-packed", seed=30, dtype=DTYPE_BF16, d_model=256, n_head=2,
                               head_dim=128, d_ff=352, vocab=777, ctx_len=131, n_sub=6, delta_t=2,
                               sub_tokens=9, batch=1, **LLAMA),
    # S = 1: ordinary sequential greedy decoding through the same kernels
    "mfma-sequential": small("mfma-sequential", seed=31, dtype=DTYPE_BF16, d_model=128, n_head=2,
                             head_dim=64, d_ff=256, vocab=1003, ctx_len=90, n_sub=1, delta_t=1,
                             sub_tokens=14, batch=2),
    "mfma-flat": small("mfma-flat", seed=29, dtype=DTYPE_BF16, d_model=128, n_head=2, head_dim=64,
                       d_ff=256, vocab=1000, ctx_len=600, n_sub=4, delta_t=3, sub_tokens=8, batch=1,
                       qkv_std=0.02, norm_init="identity"),
}


@pytest.mark.parametrize("name", list(CASES))
def test_teacher_forced_parity(name):
    cfg = CASES[name]
    say(f"[case] {name}: {cfg}")
    w = pi.make_weights(cfg, threads=4)
    ctx = pi.make_context(cfg)
    outs = oracle_run(cfg, w, ctx)
    dec = make_decoder(cfg, w)
    stats = compare_teacher_forced(cfg, w, ctx, dec, outs, log=say)
    assert stats["rows"] == cfg.batch * (cfg.n_sub * (cfg.sub_tokens + 1) - 1)
    dec.close()


def test_forced_arbitrary_tokens_and_eos():
    """Arbitrary forced tokens (not the model's own), with <eos> among them: subsequences end
    early, their last token is fed once more, exploratory subsequences keep opening."""
    cfg = small("f32-eos", seed=31, eos_id=7, n_sub=6, delta_t=1, sub_tokens=6, batch=2)
    w = pi.make_weights(cfg, threads=4)
    ctx = pi.make_context(cfg)
    force = 8 + pi.make_forced_tokens(cfg, cfg.time_steps) % (cfg.vocab - 8)
    force[2, 0, 0] = 7          # request 0: subsequence 1 ends at step 3
    force[4, 0, 2] = 7          # request 0: subsequence 3 ends at step 5
    force[3, 1, 1] = 7          # request 1: subsequence 2 ends at step 4
    outs = oracle_run(cfg, w, ctx, force=force)
    assert len(outs[0]["result"][0]) == 2 and len(outs[1]["result"][1]) == 2
    dec = make_decoder(cfg, w)
    compare_teacher_forced(cfg, w, ctx, dec, outs, force=force, log=say)
    dec.close()


@pytest.mark.parametrize("name", ["cfg1", "mfma-hd64"])
def test_generate_matches_oracle_until_a_close_call(name):
    """Free-running pd_generate: identical tokens up to the first iteration in which some row's
    top-2 margin is too small to expect the same decision; step counts and lengths always agree
    (EOS is disabled in these workloads)."""
    cfg = CASES[name]
    w = pi.make_weights(cfg, threads=4)
    ctx = pi.make_context(cfg)
    outs = oracle_run(cfg, w, ctx)
    dec = make_decoder(cfg, w)
    toks, lens, steps = dec.generate(ctx, cfg.n_sub, cfg.delta_t, cfg.sub_tokens, cfg.time_steps)
    thr = 1e-3 if cfg.dtype == 0 else 0.05
    for b, o in enumerate(outs):
        assert steps[b] == o["steps"] == cfg.time_steps
        assert lens[b].tolist() == [len(r) for r in o["result"]]
        safe = len(o["trace"])
        for t, rec in enumerate(o["trace"]):
            top2 = np.partition(rec["logits"], -2, axis=1)[:, -2:]
            if (top2[:, 1] - top2[:, 0]).min() < thr:
                safe = t
                break
        checked = 0
        for t in range(safe):
            for i, tok in o["emitted"][t].items():
                j = t - (i - 1) * cfg.delta_t          # token index inside subsequence i
                assert toks[b, i - 1, j] == tok, f"request {b} step {t + 1} subsequence {i}"
                checked += 1
        say(f"[generate] {name} request {b}: {checked} tokens identical before the first close call "
            f"(iteration {safe + 1} of {o['steps']})")
    dec.close()


# --------------------------------------------------------------------------
# Free-running pd_generate over a whole run, token for token.  The vocabulary projection of these
# workloads is drawn with a larger standard deviation and the seeds are chosen (on the CPU, with the
# oracle alone) so that every top-2 margin of the oracle's own run exceeds 0.05: a logit error within
# the 2e-2 tolerance, which the teacher-forced pass asserts first, then cannot change a decision.
# With eos_id >= 0 the model's own argmax ends subsequences: requests stop at different iterations,
# one of them through an exploratory subsequence that comes back empty (Algorithm 1, lines 10-13).
# --------------------------------------------------------------------------
GEN = dict(dtype=DTYPE_BF16, n_layer=2, d_model=128, n_head=2, head_dim=64, d_ff=256, vocab=211, batch=2,
           ctx_len=90, n_sub=3, delta_t=2, sub_tokens=5, qkv_std=0.1, lm_std=0.3)


@pytest.mark.parametrize("seed,eos,steps,lens", [
    (126, -1, [9, 9], [[5, 5, 5], [5, 5, 5]]),
    (114, 195, [4, 9], [[3, 1, 0], [5, 5, 5]]),       # request 0 stops before its third subsequence opens
    (118, 116, [9, 5], [[5, 5, 5], [4, 1, 0]]),       # request 1: the third subsequence is empty
])
def test_generate_whole_run_token_for_token(seed, eos, steps, lens):
    cfg = small(f"gen-{seed}", seed=seed, eos_id=eos, **GEN)
    w = pi.make_weights(cfg, threads=4)
    ctx = pi.make_context(cfg)
    outs = oracle_run(cfg, w, ctx)
    assert [o["steps"] for o in outs] == steps
    assert [[len(r) for r in o["result"]] + [0] * (cfg.n_sub - len(o["result"])) for o in outs] == lens
    margins = [np.diff(np.partition(rec["logits"], -2, axis=1)[:, -2:], axis=1).min()
               for o in outs for rec in o["trace"] if "logits" in rec]
    assert min(margins) > 0.05, "the workload was chosen for clear margins"
    dec = make_decoder(cfg, w)
    compare_teacher_forced(cfg, w, ctx, dec, outs, log=say)          # logits within 2e-2 on every row
    toks, got_lens, got_steps = dec.generate(ctx, cfg.n_sub, cfg.delta_t, cfg.sub_tokens, cfg.time_steps)
    assert got_steps.tolist() == steps and got_lens.tolist() == lens
    for b, o in enumerate(outs):
        for i in range(cfg.n_sub):
            want = o["result"][i] if i < len(o["result"]) else []
            assert toks[b, i, :len(want)].tolist() == want, f"request {b} subsequence {i + 1}"
            assert np.all(toks[b, i, len(want):] == -1)
    say(f"[generate] {cfg.name} eos {eos}: {sum(map(sum, lens))} tokens identical to the oracle's, "
        f"smallest oracle margin {min(margins):.3f}")
    dec.close()


# --------------------------------------------------------------------------
# Exact ties (Eq. 4, lowest index among equal logits).  The vocabulary projection gets two groups of
# identical rows (v and -v, far larger than the other rows), so in every row of every iteration one
# whole group holds the largest logit.  The groups are placed to meet every stage of the argmax:
#   matrix-core path (2100 columns = 132 tiles of 16): 37 and 38 sit in one lane of the projection's
#   epilogue, 45 in the same tile but another lane group, 1061 and 2085 in tiles 66 and 130, which the
#   commit kernel's lane 2 scans after tile 2; 600/601/1500 in other lanes;
#   fp32 path (300 columns, 256 threads): 5 and 261 are scanned by the same thread, 280 by another.
# Free-running generation must return the lowest index of the winning group every time.
# --------------------------------------------------------------------------
TIES = {
    "mfma-ties": (dict(seed=95, dtype=DTYPE_BF16, d_model=128, n_head=2, head_dim=64, d_ff=256, vocab=2100,
                       ctx_len=70, n_sub=4, delta_t=1, sub_tokens=5, batch=2),
                  [37, 38, 45, 1061, 2085], [41, 600, 601, 1500]),
    # 20 rows per step: two row tiles, general activation layout
    "mfma-ties-20-rows": (dict(seed=77, dtype=DTYPE_BF16, d_model=128, n_head=2, head_dim=64, d_ff=256,
                               vocab=2100, ctx_len=40, n_sub=4, delta_t=1, sub_tokens=4, batch=5, n_layer=1),
                          [37, 38, 45, 1061, 2085], [41, 600, 601, 1500]),
    "f32-ties": (dict(seed=84, vocab=300, n_sub=4, delta_t=1, sub_tokens=5, batch=2),
                 [5, 261, 280], [9, 100, 290]),
}


def tie_case(name):
    """Workload with tied logits and the oracle's free run over it.  Rows of the vocabulary projection
    that are identical give logits that are equal as real numbers; whether a BLAS routine returns them
    equal to the last bit depends on where the columns fall in its blocking, so the oracle's choice is
    taken as the lowest index among the logits within 1e-9 of the maximum (fp64 rounding is 1e-15)."""
    from oracle import controller, pipelined
    from oracle.model import OracleModel
    kw, group_a, group_b = TIES[name]
    cfg = small(name, **kw)
    w = pi.make_weights(cfg, threads=4)
    pi.tie_lm_head(cfg, w, group_a, group_b)
    ctx = pi.make_context(cfg)
    model = OracleModel(cfg, w)
    outs, winners = [], set()
    for b in range(cfg.batch):
        dec = pipelined.PerQueryDecoder(model, ctx[b])

        def stepper(G, t, dec=dec):
            out = list(dec(G, t))
            rec = dec.trace[-1]
            for r, i in enumerate(rec["rows"]):
                lg = rec["logits"][r]
                tied = np.flatnonzero(lg >= lg.max() - 1e-9).tolist()
                assert tied in (group_a, group_b), f"{name}: the maximum is not one whole group of duplicates"
                assert np.sort(lg)[-len(tied) - 1] < lg.max() - 1.0, f"{name}: the other logits are too close"
                out[i - 1] = tied[0]
                winners.add(tied[0])
            return out

        result, steps, _ = controller.pipelined_decode(stepper, cfg.delta_t, cfg.time_steps, cfg.n_sub,
                                                       cfg.bos_id, cfg.eos_id, cfg.sub_tokens)
        outs.append({"result": result, "steps": steps})
    assert winners == {group_a[0], group_b[0]}, f"{name}: the run should meet both groups"
    return cfg, w, ctx, outs


@pytest.mark.parametrize("name", list(TIES))
def test_exact_ties_select_the_lowest_index(name):
    cfg, w, ctx, outs = tie_case(name)
    dec = make_decoder(cfg, w)
    assert dec.get_info(binding_mod().PD_INFO_KERNEL_PATH) == (1 if name.startswith("mfma") else 0)
    toks, lens, steps = dec.generate(ctx, cfg.n_sub, cfg.delta_t, cfg.sub_tokens, cfg.time_steps)
    for b, o in enumerate(outs):
        assert steps[b] == o["steps"]
        for i, want in enumerate(o["result"]):
            assert toks[b, i, :len(want)].tolist() == want, f"request {b} subsequence {i + 1}"
    dec.close()


def binding_mod():
    from paper_2506_23431_amd import binding
    return binding


def test_saturated_keys_and_values_are_counted():
    """The 16-bit cache stores keys and values beyond +-65504 saturated; pd_get_info tells the caller
    how many.  A QKV projection drawn 10^5 times larger than usual saturates most of them; the usual
    one none."""
    b = binding_mod()
    for name, kw in (("mfma", dict(d_model=128, n_head=2, head_dim=64, d_ff=256)), ("simple", dict(head_dim=12))):
        for std, expect_some in ((0.1, False), (2.0e4, True)):
            cfg = small(f"{name}-sat", seed=81, dtype=DTYPE_BF16, batch=1, ctx_len=40, n_sub=2, delta_t=1,
                        sub_tokens=2, qkv_std=std, **kw)
            w = pi.make_weights(cfg, threads=4)
            dec = make_decoder(cfg, w)
            dec.generate(pi.make_context(cfg), cfg.n_sub, cfg.delta_t, cfg.sub_tokens, cfg.time_steps)
            n = dec.get_info(b.PD_INFO_KV_SATURATED)
            say(f"[saturation] {cfg.name} qkv std {std}: {n} keys / values stored saturated")
            assert (n > 0) == expect_some
            assert dec.get_info(b.PD_INFO_KV_PAIR_LAYERS) == 0
            dec.close()


MF = dict(dtype=DTYPE_BF16, d_model=128, n_head=2, head_dim=64, d_ff=256, vocab=1003)
DEGENERATE = {
    # one context token, one subsequence, one token
    "f32-minimal": (small("f32-minimal", seed=40, ctx_len=1, n_sub=1, delta_t=1, sub_tokens=1, batch=1), None),
    "mfma-minimal": (small("mfma-minimal", seed=41, ctx_len=1, n_sub=1, delta_t=1, sub_tokens=1, batch=1, **MF), None),
    # delay not shorter than a subsequence: Algorithm 1 stops when the first subsequence has
    # finished and the second was never opened (3 of the 13 scheduled steps)
    "f32-delay-longer-than-subsequence": (small("f32-late", seed=42, n_sub=3, delta_t=5, sub_tokens=3), None),
    "mfma-delay-longer-than-subsequence": (small("mfma-late", seed=43, n_sub=3, delta_t=5, sub_tokens=3, **MF), None),
    # time_max cuts the run short: 4 of 14 steps
    "f32-time-max": (small("f32-tmax", seed=44), 4),
    "mfma-time-max": (small("mfma-tmax", seed=45, **MF), 4),
    # one-token subsequences opened every step: every row is a <bos> row or a draining row
    "mfma-one-token-subsequences": (small("mfma-m1", seed=46, n_sub=7, delta_t=1, sub_tokens=1, ctx_len=33, **MF), None),
    # context of exactly one and exactly two 32-key blocks; 8 rows (packed pairs) then more
    "mfma-context-32": (small("mfma-l32", seed=47, ctx_len=32, n_sub=9, delta_t=1, sub_tokens=10, batch=1, **MF), None),
    "mfma-context-64": (small("mfma-l64", seed=48, ctx_len=64, n_sub=3, delta_t=2, sub_tokens=5, batch=1, **MF), None),
    # the largest step the matrix-core path takes: 8 requests x 16 rows = 128 rows
    "mfma-128-rows": (small("mfma-r128", seed=49, n_sub=16, delta_t=1, sub_tokens=15, batch=8, ctx_len=40,
                            n_layer=1, **MF), 20),
}


@pytest.mark.parametrize("name", list(DEGENERATE))
def test_degenerate_and_extreme_schedules(name):
    cfg, steps = DEGENERATE[name]
    say(f"[case] {name}: {cfg}, steps {steps}")
    w = pi.make_weights(cfg, threads=4)
    ctx = pi.make_context(cfg)
    outs = oracle_run(cfg, w, ctx, steps=steps)
    if name.endswith("delay-longer-than-subsequence"):
        assert all(o["steps"] == cfg.sub_tokens and len(o["result"]) == 1 for o in outs)
    dec = make_decoder(cfg, w)
    stats = compare_teacher_forced(cfg, w, ctx, dec, outs, steps=steps, log=say)
    assert stats["rows"] > 0
    if steps is not None:
        # the run is over after time_max steps: one more step produces nothing and reports all done
        toks, _, done = dec.decode_step(want_done=True)
        assert done and np.all(toks == -1)
    dec.close()


def _random_case(k):
    """Seeded random small workload k: widths, schedule and batch drawn so that the cases cover one
    to five row tiles, packed and general activation layouts, ragged contexts and early stops."""
    rng = np.random.default_rng(1000 + k)
    hd = int(rng.choice([32, 64, 96, 128]))
    nh = int(rng.integers(1, 4))
    llama = bool(rng.integers(0, 2))
    kw = dict(seed=60 + k, dtype=DTYPE_BF16, d_model=hd * nh, n_head=nh, head_dim=hd,
              d_ff=int(rng.choice([96, 160, 224, 320])), vocab=int(rng.integers(130, 900)),
              ctx_len=int(rng.integers(1, 300)), n_sub=int(rng.integers(1, 12)), delta_t=int(rng.integers(1, 6)),
              sub_tokens=int(rng.integers(1, 10)), batch=int(rng.integers(1, 6)), n_layer=int(rng.integers(1, 3)))
    if llama:
        kw.update(LLAMA)
    return small(f"mfma-random-{k}", **kw)


@pytest.mark.parametrize("k", range(12))
def test_random_small_workloads(k):
    cfg = _random_case(k)
    say(f"[case] {cfg}")
    w = pi.make_weights(cfg, threads=4)
    ctx = pi.make_context(cfg)
    outs = oracle_run(cfg, w, ctx)
    dec = make_decoder(cfg, w)
    stats = compare_teacher_forced(cfg, w, ctx, dec, outs, log=say)
    assert stats["rows"] > 0
    dec.close()


def test_more_than_128_rows_per_step():
    """9 requests x 16 rows = 144 rows per step: beyond the 128 rows of the small projection kernels,
    every projection (the vocabulary argmax included) runs in the many-row kernel of the context pass."""
    cfg = small("mfma-r144", seed=50, n_sub=16, delta_t=1, sub_tokens=15, batch=9, ctx_len=40, n_layer=1, **MF)
    w = pi.make_weights(cfg, threads=4)
    ctx = pi.make_context(cfg)
    outs = oracle_run(cfg, w, ctx, log=say)
    dec = make_decoder(cfg, w)
    stats = compare_teacher_forced(cfg, w, ctx, dec, outs, log=say)
    assert stats["rows"] == cfg.batch * (cfg.n_sub * (cfg.sub_tokens + 1) - 1)
    dec.close()


def test_boundary_errors():
    from paper_2506_23431_amd import PdError
    cfg = CASES["cfg1"]
    w = pi.make_weights(cfg, threads=2)
    ctx = pi.make_context(cfg)
    dec = make_decoder(cfg, w)
    with pytest.raises(PdError, match="before pd_prefill_context"):
        dec.B, dec.S = 1, cfg.n_sub
        dec.decode_step()
    with pytest.raises(PdError, match="delta_t"):
        dec.prefill_context(ctx, cfg.n_sub, 0, cfg.sub_tokens, 10)
    with pytest.raises(PdError, match="n_sub"):
        dec.prefill_context(ctx, cfg.n_sub + 1, 1, cfg.sub_tokens, 10)
    with pytest.raises(PdError, match="out of range"):
        bad = ctx.copy(); bad[0, 3] = cfg.vocab
        dec.prefill_context(bad, cfg.n_sub, 1, cfg.sub_tokens, 10)
    with pytest.raises(PdError, match="L ="):
        dec.prefill_context(np.zeros((1, cfg.ctx_len + 1), np.int32), cfg.n_sub, 1, cfg.sub_tokens, 10)
    # time_max bounds the loop: 3 steps, then further steps are no-ops
    toks, lens, steps = dec.generate(ctx, cfg.n_sub, cfg.delta_t, cfg.sub_tokens, 3)
    assert steps[0] == 3 and lens[0].tolist() == [3, 1, 0, 0]
    t, _, done = dec.decode_step()
    assert done and np.all(t == -1)
    dec.close()


def test_cfg2_full_size():
    """BART-base-shaped workload at full size: all 92 iterations, every logit row."""
    cfg = pi.get_config("cfg2")
    say(f"[case] cfg2 full size: {cfg}")
    w = pi.make_weights(cfg)
    ctx = pi.make_context(cfg)
    outs = oracle_run(cfg, w, ctx)
    say("[cfg2] oracle done")
    dec = make_decoder(cfg, w)
    stats = compare_teacher_forced(cfg, w, ctx, dec, outs, log=say)
    assert stats["rows"] == cfg.n_sub * (cfg.sub_tokens + 1) - 1
    dec.close()


# --------------------------------------------------------------------------
# Full-width workloads in the launch configuration the benchmark times: the named
# workloads with 2 layers instead of 12-32 (every kernel's grid, tile shape and key-block
# partition depend on widths, context length, S, dt, M and batch -- not on the depth), a
# mildly peaky attention (QKV std 0.03 instead of 0.02) and a bounded number of iterations
# so that the fp64 oracle finishes in about a minute.
# --------------------------------------------------------------------------
WIDE = {
    # name: (config, iterations)
    "cfg3-wide": (pi.get_config("cfg3").scaled(name="cfg3-wide", n_layer=2, qkv_std=0.03), 40),
    "cfg4-wide": (pi.get_config("cfg4").scaled(name="cfg4-wide", n_layer=2, qkv_std=0.03), 72),
    # dt=1: 17-32 rows per step from iteration 17 on (two row tiles against matrices of 25-34 MB)
    "cfg4-wide-dt1": (pi.get_config("cfg4").scaled(name="cfg4-wide-dt1", n_layer=2, qkv_std=0.03, delta_t=1), 34),
    # dt=1 instead of 4: all 16 rows per request (64 rows in all) are reached within 16 iterations
    "cfg5-wide": (pi.get_config("cfg5").scaled(name="cfg5-wide", n_layer=2, qkv_std=0.03, delta_t=1), 12),
}


@pytest.mark.parametrize("name", list(WIDE))
def test_full_width_parity(name):
    cfg, steps = WIDE[name]
    say(f"[case] {name}: {cfg}, first {steps} iterations")
    w = pi.make_weights(cfg)
    ctx = pi.make_context(cfg)
    say(f"[{name}] weights drawn")
    outs = oracle_run(cfg, w, ctx, steps=steps, log=say)
    say(f"[{name}] oracle done")
    dec = make_decoder(cfg, w)
    # the context pass in 1024-row chunks whatever the default for these widths is, so that the
    # many-row projection kernel is covered at every width
    from paper_2506_23431_amd import binding
    dec.set_option(binding.PD_OPT_PREFILL_CHUNK, 1024)
    stats = compare_teacher_forced(cfg, w, ctx, dec, outs, steps=steps, log=say)
    assert stats["rows"] > 0
    dec.close()


# --------------------------------------------------------------------------
# Pair caches: the first kv_pair_layers layers keep keys and values as high + low halves.
# --------------------------------------------------------------------------
@pytest.mark.parametrize("name,pair_layers", [("mfma-hd128-llama", 1), ("mfma-hd64", 2), ("mfma-hd32", 1),
                                              ("mfma-hd96", 2), ("mfma-manyrows", 1), ("bf16-simple", 1)])
def test_pair_cache_layers(name, pair_layers):
    cfg = CASES[name]
    say(f"[case] {name} with kv_pair_layers = {pair_layers}")
    w = pi.make_weights(cfg, threads=4)
    ctx = pi.make_context(cfg)
    outs = oracle_run(cfg, w, ctx)
    dec = make_decoder(cfg, w, kv_pair_layers=pair_layers)
    stats = compare_teacher_forced(cfg, w, ctx, dec, outs, log=say)
    assert stats["rows"] == cfg.batch * (cfg.n_sub * (cfg.sub_tokens + 1) - 1)
    dec.close()


def test_cfg5_all_layers_short_context():
    """All 32 layers at the cfg5 widths (7B parameters), 1024 context tokens, one request, four
    subsequences: the depth is what the 2-layer full-width case leaves out.  With plain half caches
    the rounding of layer 0's keys and values alone reaches the logits at 1.7e-2 - 2.0e-2 here
    (2.8e-2 over the whole cfg5 workload, measured against the library's fp32 kernels); with layer 0
    kept as pairs the error is several times below the tolerance, which the test asserts so that a
    kernel that ignored the low halves could not pass."""
    cfg = pi.get_config("cfg5").scaled(name="cfg5-deep", ctx_len=1024, batch=1, n_sub=4, delta_t=1,
                                       sub_tokens=3)
    say(f"[case] {cfg.name}: {cfg}")
    w = pi.make_weights(cfg)
    ctx = pi.make_context(cfg)
    say(f"[{cfg.name}] weights drawn")
    outs = oracle_run(cfg, w, ctx, log=say, cache_layers=False)
    say(f"[{cfg.name}] oracle done")
    dec = make_decoder(cfg, w, kv_pair_layers=1)
    stats = compare_teacher_forced(cfg, w, ctx, dec, outs, log=say)
    assert stats["rows"] == cfg.n_sub * (cfg.sub_tokens + 1) - 1
    assert stats["worst"] < 5e-3, stats
    dec.close()


@pytest.mark.parametrize("chunk,ctx_attn", [(256, 1), (160, 1), (48, 1), (256, 2), (160, 2), (48, 2), (0, 2), (40, 2)])
def test_context_pass_in_several_chunks(chunk, ctx_attn):
    """600 context tokens in chunks of 256 (two launches of the many-row kernels and a tail of 88
    rows in the 128-row kernels), 160 (three and a tail of 120), 48 and 40 rows, and all at once: the
    caches the context pass leaves behind must give the oracle's logits whatever the chunking, with the
    decode step's attention kernel (what the library picks at this size) and with the 32-query kernel
    of large context passes (PD_OPT_CONTEXT_ATTN 2; chunks with a ragged last query tile included)."""
    from paper_2506_23431_amd import binding
    cfg = CASES["mfma-flat"]
    w = pi.make_weights(cfg, threads=4)
    ctx = pi.make_context(cfg)
    outs = oracle_run(cfg, w, ctx)
    dec = make_decoder(cfg, w)
    dec.set_option(binding.PD_OPT_PREFILL_CHUNK, chunk)
    dec.set_option(binding.PD_OPT_CONTEXT_ATTN, ctx_attn)
    stats = compare_teacher_forced(cfg, w, ctx, dec, outs, log=say)
    assert stats["rows"] == cfg.batch * (cfg.n_sub * (cfg.sub_tokens + 1) - 1)
    dec.close()


@pytest.mark.parametrize("name,split_act", [("mfma-hd128-llama", 1), ("mfma-flat", 0), ("mfma-hd64", 1),
                                            ("mfma-hd64", 0), ("mfma-manyrows", 1), ("mfma-llama-packed", 1)])
def test_context_attention_kernel_of_large_passes(name, split_act):
    """PD_OPT_CONTEXT_ATTN 2: the 32-query attention kernel that large context passes pick by themselves,
    here on small shapes: head sizes 128 and 64, several requests, contexts that are no multiple of the
    32-key block or of the 32-query block, queries with and without low parts."""
    from paper_2506_23431_amd import binding
    cfg = CASES[name]
    w = pi.make_weights(cfg, threads=4)
    ctx = pi.make_context(cfg)
    outs = oracle_run(cfg, w, ctx)
    dec = make_decoder(cfg, w)
    dec.set_option(binding.PD_OPT_CONTEXT_ATTN, 2)
    dec.set_option(binding.PD_OPT_SPLIT_ACT, split_act)
    stats = compare_teacher_forced(cfg, w, ctx, dec, outs, log=say)
    assert stats["rows"] == cfg.batch * (cfg.n_sub * (cfg.sub_tokens + 1) - 1)
    dec.close()


@pytest.mark.parametrize("name", ["mfma-flat", "mfma-hd128-llama"])
def test_context_pass_activation_precision(name):
    """PD_OPT_CONTEXT_SPLIT_ACT 0: the context pass carries single bf16 activations (half the multiplies);
    on these workloads that stays inside the tolerance, and the default (pairs) is at least as close to the
    oracle."""
    from paper_2506_23431_amd import binding
    cfg = CASES[name]
    w = pi.make_weights(cfg, threads=4)
    ctx = pi.make_context(cfg)
    outs = oracle_run(cfg, w, ctx)
    dec = make_decoder(cfg, w)
    assert dec.get_info(binding.PD_INFO_CONTEXT_PAIRS) == 1
    worst = {}
    for val in (0, 1):
        dec.set_option(binding.PD_OPT_CONTEXT_SPLIT_ACT, val)
        assert dec.get_info(binding.PD_INFO_CONTEXT_PAIRS) == val
        worst[val] = compare_teacher_forced(cfg, w, ctx, dec, outs, log=say)["worst"]
    assert worst[1] <= worst[0] * 1.5
    dec.close()


def test_options_do_not_change_results():
    """HIP-graph replay of the step, other attention split counts, other chunk sizes of the context
    pass (the default here is all 150 rows at once, in the many-row projection kernel) and
    plain-bf16 activations: same tokens as the default path on a workload whose top-2 margins are
    comfortably above the bf16 noise; the graph is replayed for every step of three runs with eager
    work and synchronisations in between, and every replayed run is compared."""
    import torch
    from paper_2506_23431_amd import binding
    cfg = CASES["mfma-hd64"]
    w = pi.make_weights(cfg, threads=4)
    ctx = pi.make_context(cfg)
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        dec = make_decoder(cfg, w)
        args = (ctx, cfg.n_sub, cfg.delta_t, cfg.sub_tokens, cfg.time_steps)
        base = dec.generate(*args)
        for key, val in ((binding.PD_OPT_USE_GRAPH, 1), (binding.PD_OPT_ATTN_SPLITS, 3),
                         (binding.PD_OPT_ATTN_SPLITS, 1), (binding.PD_OPT_ATTN_SPLITS, 7),
                         (binding.PD_OPT_PREFILL_CHUNK, 16), (binding.PD_OPT_PREFILL_CHUNK, 40),
                         (binding.PD_OPT_PREFILL_CHUNK, 128), (binding.PD_OPT_PREFILL_CHUNK, 144),
                         (binding.PD_OPT_PROFILE, 3),        # the attention kernel launched twice per layer
                         (binding.PD_OPT_STREAM_LOADS, 1),   # non-temporal loads of weights, keys and values
                         (binding.PD_OPT_CONTEXT_ATTN, 2)):  # the 32-query attention kernel in the context pass
            dec.set_option(key, val)
            for rep in range(3 if key == binding.PD_OPT_USE_GRAPH else 1):
                got = dec.generate(*args)
                torch.cuda.synchronize()
                for a, b in zip(base, got):
                    assert np.array_equal(a, b), f"option {key}={val} (run {rep}) changed the result"
            dec.set_option(key, 0)
        # plain bf16 activations: larger rounding error, still within the logit tolerance
        dec.set_option(binding.PD_OPT_SPLIT_ACT, 0)
        outs = oracle_run(cfg, w, ctx)
        compare_teacher_forced(cfg, w, ctx, dec, outs, log=say)
        # ... also with a context pass in chunks of 40 rows (three row tiles, each with blocks of its own)
        dec.set_option(binding.PD_OPT_PREFILL_CHUNK, 40)
        compare_teacher_forced(cfg, w, ctx, dec, outs, log=say)
        dec.close()


@pytest.mark.parametrize("name", ["mfma-hd64", "mfma-llama-packed", "mfma-hd128-llama", "mfma-hd32", "mfma-manyrows"])
def test_separate_second_norm_kernel(name):
    """Steps of at most 16 rows, and steps of up to 128 rows against small matrices (mfma-manyrows: 40),
    normally finish the layer's second norm inside the first FFN projection (PD_OPT_FUSE_NORM); with the
    option off they take the separate norm kernel that all other steps use."""
    from paper_2506_23431_amd import binding
    cfg = CASES[name]
    w = pi.make_weights(cfg, threads=4)
    ctx = pi.make_context(cfg)
    outs = oracle_run(cfg, w, ctx)
    dec = make_decoder(cfg, w)
    dec.set_option(binding.PD_OPT_FUSE_NORM, 0)
    stats = compare_teacher_forced(cfg, w, ctx, dec, outs, log=say)
    assert stats["rows"] == cfg.batch * (cfg.n_sub * (cfg.sub_tokens + 1) - 1)
    dec.close()


@pytest.mark.parametrize("name", ["mfma-hd64", "mfma-hd32", "mfma-hd96", "mfma-sequential", "mfma-flat", "rms-learned"])
def test_first_norm_prepared_by_the_previous_layer(name):
    """Value 2 of PD_OPT_FUSE_NORM: the second FFN projection of a layer completes the residual rows and
    hands gain * x with its row sums to the next layer's QKV projection, which finishes that layer's first
    norm in its epilogue (steps of at most 16 rows, no rotary positions): packed pairs, separate low
    parts, LayerNorm with bias and RMSNorm."""
    from paper_2506_23431_amd import binding
    cfg = CASES[name] if name in CASES else small(name, seed=52, dtype=DTYPE_BF16, d_model=160, n_head=5,
                                                   head_dim=32, d_ff=288, vocab=700, ctx_len=61, n_sub=5,
                                                   delta_t=1, sub_tokens=6, batch=2, n_layer=3,
                                                   norm_kind=NORM_RMSNORM)
    w = pi.make_weights(cfg, threads=4)
    ctx = pi.make_context(cfg)
    outs = oracle_run(cfg, w, ctx)
    dec = make_decoder(cfg, w)
    dec.set_option(binding.PD_OPT_FUSE_NORM, 2)
    stats = compare_teacher_forced(cfg, w, ctx, dec, outs, log=say)
    assert stats["rows"] == cfg.batch * (cfg.n_sub * (cfg.sub_tokens + 1) - 1)
    dec.close()


def test_sweep_runs_sequential_and_pipelined():
    """The sweep tool (sequential S = 1 against pipelined schedules with the same token count) runs on
    a two-layer variant of cfg2 and reports the step counts of the schedule's closed form."""
    from paper_2506_23431_amd import sweep
    rows = sweep.main(["--workload", "cfg2", "--layers", "2", "--tokens", "64", "--s-list", "1,4,8",
                       "--dt-list", "1,4"])
    got = {(r["S"], r["dt"]): r for r in rows}
    assert set(got) == {(1, 1), (4, 1), (4, 4), (8, 1), (8, 4)}
    for (S, dt), r in got.items():
        assert r["steps"] == (S - 1) * dt + 64 // S
        assert r["tokens_per_s"] > 0
    assert got[(1, 1)]["speedup_vs_sequential"] == 1.0


def test_ragged_targets_with_eos_match_the_oracle():
    """Targets of uneven shape, drawn the way the ragged sweep draws them (Table 1 averages): every
    subsequence ends with a forced <eos> at its drawn length, later subsequences come back empty,
    requests finish at different times.  Oracle and library get the same forced decisions; every
    logit row and the per-request step counts must agree."""
    from paper_2506_23431_amd import sweep
    dt = 2
    lens = sweep.draw_ragged("cnndm", 3, dt, seed=3)
    lens = [[max(dt, n // 3) for n in l] for l in lens]    # a third of the length: a short oracle run
    assert lens == [[7], [4, 4], [7, 5, 8, 6, 5, 5]]
    S, M, T = sweep.ragged_plan(lens, dt)
    cfg = small("mfma-ragged", seed=33, dtype=DTYPE_BF16, d_model=128, n_head=2, head_dim=64, d_ff=256,
                vocab=1003, ctx_len=70, batch=3, n_sub=S, delta_t=dt, sub_tokens=M, eos_id=1)
    say(f"[case] {cfg.name}: lengths {lens}, S={S} M={M} T={T}")
    w = pi.make_weights(cfg, threads=4)
    ctx = pi.make_context(cfg)
    # forced decisions: <eos> as token number len + 1 of a drawn subsequence and as the first token
    # of every other one; a fixed non-<eos> token everywhere else, so that the lengths are exact
    force = np.full((T, cfg.batch, S), -1, dtype=np.int64)
    for b in range(cfg.batch):
        for i in range(S):
            n = lens[b][i] if i < len(lens[b]) else 0
            t0 = i * dt                                       # 0-based iteration of the first token
            for j in range(n + 1):
                if t0 + j < T:
                    force[t0 + j, b, i] = cfg.eos_id if j == n else 8 + (7 * b + 3 * i + j) % 900
    outs = oracle_run(cfg, w, ctx, force=force)
    for b, o in enumerate(outs):
        assert [len(r) for r in o["result"]][:len(lens[b])] == lens[b]
    assert len({o["steps"] for o in outs}) > 1, "requests should finish at different times"
    dec = make_decoder(cfg, w)
    compare_teacher_forced(cfg, w, ctx, dec, outs, force=force, log=say)
    dec.close()


def test_ragged_sweep_runs():
    from paper_2506_23431_amd import sweep
    rows = sweep.main(["--workload", "cfg2", "--layers", "2", "--ragged", "cnndm", "--dt-list", "2,4",
                       "--targets", "3"])
    assert [r["mode"] for r in rows] == ["sequential", "pipelined", "pipelined"]
    assert all(r["lengths_as_drawn"] for r in rows)
    assert all(r["tokens_per_s"] > 0 for r in rows)


def test_plain_read_bandwidth_measurement():
    """pd_measure_read_bandwidth: sane figure for a 64 MB chunk out of a 1 GiB buffer, errors for bad arguments."""
    import torch
    from paper_2506_23431_amd import binding, PdError
    buf = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    gbs = binding.measure_read_bandwidth(buf.data_ptr(), buf.numel(), 64 << 20, 50)
    say(f"[read] 64 MiB chunks: {gbs:.0f} GB/s")
    assert 1000 < gbs < 8000          # below the 8 TB/s peak, far above anything a broken kernel would show
    with pytest.raises(PdError, match="chunk_bytes"):
        binding.measure_read_bandwidth(buf.data_ptr(), buf.numel(), buf.numel(), 1)
    with pytest.raises(PdError, match="aligned"):
        binding.measure_read_bandwidth(buf.data_ptr() + 4, buf.numel() - 4, 1 << 20, 1)
