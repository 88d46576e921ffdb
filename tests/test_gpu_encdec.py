"""GPU parity of the encoder-decoder form (Eq. 1, Eq. 3, Section 4.3) against oracle/encdec.py:
the library encodes the inputs, then steps Algorithm 1 teacher-forced with the oracle's tokens; every
logit row is compared (2e-2, the bf16 bar) and every token whose oracle margin exceeds 0.05 is the
library's own choice.  Both sides get the same bf16-rounded weights."""

import numpy as np
import pytest

import pd_inputs as pi
from oracle import controller, encdec
from parity_util import compare_teacher_forced

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def E(name, seed, **kw):
    base = dict(n_enc_layer=2, n_dec_layer=2, d_model=128, n_head=2, head_dim=64, d_ff=256, vocab=1003,
                rel_buckets=32, rel_max_distance=128, ctx_len=150, n_sub=5, delta_t=2, sub_tokens=7, batch=2)
    base.update(kw)
    return pi.EncDecConfig(name=name, seed=seed, **base)


CASES = {
    "encdec-hd64": E("encdec-hd64", 61),
    # few buckets and a short reach: distances beyond max_distance on both sides (75 input tokens; grid
    # coordinates up to 31), three heads of 32, rows of three requests
    "encdec-hd32-short-reach": E("encdec-hd32-short-reach", 62, d_model=96, n_head=3, head_dim=32, d_ff=160,
                                 vocab=517, rel_buckets=8, rel_max_distance=20, ctx_len=75, n_sub=6, delta_t=3,
                                 sub_tokens=12, batch=3),
    # one request, at most 5 rows: every decode step keeps its activations as packed pairs
    "encdec-hd128-packed": E("encdec-hd128-packed", 63, d_model=256, n_head=2, head_dim=128, d_ff=352, vocab=777,
                             ctx_len=200, n_sub=6, delta_t=2, sub_tokens=9, batch=1),
    # up to 40 rows per step (three row tiles, each with blocks of its own), input of exactly one 32-key block
    "encdec-manyrows": E("encdec-manyrows", 64, n_enc_layer=1, n_dec_layer=1, vocab=640, ctx_len=32, n_sub=20,
                         delta_t=1, sub_tokens=24, batch=2),
    # S = 1: ordinary greedy decoding with ordinary relative positions; input of one token
    "encdec-sequential": E("encdec-sequential", 65, ctx_len=1, n_sub=1, delta_t=1, sub_tokens=14, batch=2),
    # three encoder layers over a ragged input, deeper decoder
    "encdec-deeper": E("encdec-deeper", 66, n_enc_layer=3, n_dec_layer=4, ctx_len=333, n_sub=4, delta_t=3,
                       sub_tokens=8, batch=1),
}


def oracle_run(cfg, rounded, ctx, force=None):
    model = encdec.EncDecModel(cfg, rounded)
    outs = []
    for b in range(cfg.batch):
        dec = encdec.EncDecPerQueryDecoder(model, ctx[b], force=None if force is None else force[:, b, :])
        result, n_steps, emitted = controller.pipelined_decode(
            dec, cfg.delta_t, cfg.time_steps, cfg.n_sub, cfg.bos_id, cfg.eos_id, cfg.sub_tokens)
        outs.append({"result": result, "steps": n_steps, "emitted": emitted, "trace": dec.trace})
    return outs


def make(cfg):
    from paper_2506_23431_amd.binding import EncDecPipelinedDecoder
    rounded, device = pi.encdec_to_bf16(pi.make_encdec_weights(cfg))
    ctx = pi.make_context(cfg)
    dec = EncDecPipelinedDecoder(cfg, device, max_batch=cfg.batch, max_ctx=cfg.ctx_len, max_sub=cfg.n_sub,
                                 max_sub_tokens=cfg.sub_tokens)
    return rounded, ctx, dec


@pytest.mark.parametrize("name", list(CASES))
def test_encoder_decoder_parity(name):
    cfg = CASES[name]
    say(f"[encdec] {name}: {cfg}")
    rounded, ctx, dec = make(cfg)
    outs = oracle_run(cfg, rounded, ctx)
    stats = compare_teacher_forced(cfg, None, ctx, dec, outs, tol=2e-2, log=say)
    assert stats["rows"] == cfg.batch * (cfg.n_sub * (cfg.sub_tokens + 1) - 1)
    assert stats["exact"] > 0
    dec.close()


@pytest.mark.parametrize("name", sorted(pi.ENCDEC_CONFIGS) + ["encdec-base-x4"])
def test_backbone_shaped_models_at_full_size(name):
    """The backbone-shaped models the sweep measures (Section 5.1: base and large size, and a smaller one;
    random weights): 6 + 6 to 24 + 24 layers, 512 input tokens, vocabulary 32128, one request, 8
    subsequences of 16 tokens.  The encoder pass runs the many-row kernels, the decode steps the packed
    ones, the two larger models with streamed weight loads.  The base size also with four requests at
    once: 32 rows per step, two row tiles."""
    cfg = (pi.ENCDEC_CONFIGS["encdec-base"].scaled(name="encdec-base-x4", batch=4) if name.endswith("-x4")
           else pi.ENCDEC_CONFIGS[name])
    say(f"[encdec] {name}: {cfg}")
    rounded, ctx, dec = make(cfg)
    outs = oracle_run(cfg, rounded, ctx)
    stats = compare_teacher_forced(cfg, None, ctx, dec, outs, tol=2e-2, log=say)
    assert stats["rows"] == cfg.batch * (cfg.n_sub * (cfg.sub_tokens + 1) - 1)
    assert stats["exact"] > 0
    dec.close()


@pytest.mark.parametrize("name", ["encdec-hd64", "encdec-hd32-short-reach", "encdec-hd128-packed", "encdec-manyrows"])
def test_encoder_decoder_teacher_forced_forward(name):
    """Section 3.3 on the encoder-decoder form: whole training targets in one pass (the time half of Fig. 3b's
    matrix is the attention kernel's own check here, and distances reach beyond max_distance in the second
    case); logits, loss terms and loss against oracle/training.py."""
    from oracle import training
    cfg = CASES[name].scaled(eos_id=1)
    rounded, ctx, dec = make(cfg)
    model = encdec.EncDecModel(cfg, rounded)
    g = np.random.Generator(np.random.Philox(key=[cfg.seed, 0x7EAC]))
    targets = []
    for _ in range(cfg.batch):
        Y = [[int(t) for t in g.integers(2, cfg.vocab, size=int(g.integers(1, cfg.sub_tokens)))]
             for _ in range(int(g.integers(2, cfg.n_sub)))]
        while sum(len(y) + 2 for y in Y) + 2 > 120:
            Y.pop()
        targets.append(training.training_target(Y, cfg.bos_id, cfg.eos_id))
    dec.prefill_context(ctx, cfg.n_sub, cfg.delta_t, cfg.sub_tokens, cfg.time_steps)
    logits, nll, loss = dec.teacher_forced(targets)
    worst = worst_nll = 0.0
    for b, tgt in enumerate(targets):
        want_logits, want_nll, want_loss = training.teacher_forced_encdec(model, ctx[b], tgt, cfg.delta_t)
        err = np.abs(logits[b].cpu().numpy().astype(np.float64) - want_logits).max()
        assert np.isfinite(err) and err <= 2e-2, f"request {b}: max|logit diff| = {err:.3e}"
        e2 = np.abs(nll[b] - want_nll).max()
        assert e2 <= 4e-2 and np.array_equal(nll[b] == 0, want_nll == 0)
        assert abs(loss[b] - want_loss) <= 4e-2 * int((want_nll != 0).sum())
        worst, worst_nll = max(worst, err), max(worst_nll, e2)
    say(f"[teacher-forced] {name}: {sum(len(x) for x in nll)} rows, max|logit diff| = {worst:.3e}, "
        f"max|term diff| = {worst_nll:.3e}")
    # the context decodes as before afterwards
    outs = oracle_run(cfg.scaled(eos_id=-1), rounded, ctx)
    compare_teacher_forced(cfg.scaled(eos_id=-1), None, ctx, dec, outs, tol=2e-2, log=say)
    dec.close()


def _random_case(k):
    """Seeded random small encoder-decoder workload k: head sizes 32 / 64 / 96 / 128, one to three heads, bucket
    counts and reaches on both sides of the distances that occur, ragged inputs, one to five row tiles per
    step, delays longer than a subsequence (Algorithm 1 then stops early)."""
    rng = np.random.default_rng(2000 + k)
    hd = int(rng.choice([32, 64, 96, 128]))
    nh = int(rng.integers(1, 4))
    buckets = int(rng.choice([4, 8, 16, 32]))
    return E(f"encdec-random-{k}", 80 + k, n_enc_layer=int(rng.integers(1, 3)), n_dec_layer=int(rng.integers(1, 3)),
             d_model=hd * nh, n_head=nh, head_dim=hd, d_ff=int(rng.choice([96, 160, 224, 320])),
             vocab=int(rng.integers(130, 900)), rel_buckets=buckets,
             rel_max_distance=int(rng.integers(buckets // 2 + 1, 129)), ctx_len=int(rng.integers(1, 300)),
             n_sub=int(rng.integers(1, 12)), delta_t=int(rng.integers(1, 6)), sub_tokens=int(rng.integers(1, 10)),
             batch=int(rng.integers(1, 6)))


@pytest.mark.parametrize("k", range(10))
def test_encoder_decoder_random_small_workloads(k):
    cfg = _random_case(k)
    say(f"[case] {cfg}")
    rounded, ctx, dec = make(cfg)
    outs = oracle_run(cfg, rounded, ctx)
    stats = compare_teacher_forced(cfg, None, ctx, dec, outs, tol=2e-2, log=say)
    assert stats["rows"] > 0
    dec.close()


def test_encoder_decoder_forced_tokens_and_eos():
    """Arbitrary forced tokens (the model's own choices never enter the history) with <eos> among them:
    subsequences end early, requests end at different steps."""
    cfg = CASES["encdec-hd64"].scaled(name="encdec-eos", seed=67, eos_id=5, vocab=40)
    rounded, ctx, dec = make(cfg)
    force = pi.make_forced_tokens(cfg, cfg.time_steps)
    outs = oracle_run(cfg, rounded, ctx, force=force)
    assert len({o["steps"] for o in outs}) > 1 or any(len(r) < cfg.sub_tokens for o in outs for r in o["result"])
    compare_teacher_forced(cfg, None, ctx, dec, outs, force=force, tol=2e-2, log=say)
    dec.close()


def test_encoder_decoder_generate_and_options():
    """pd_generate equals stepping the same context one call at a time; graph replay, other attention
    split counts and plain-bf16 activations leave the tokens of a workload with clear margins alone; a
    second prefill with other inputs on the same context gives what a fresh context gives."""
    import torch
    from paper_2506_23431_amd import binding
    cfg = CASES["encdec-hd64"]
    st = torch.cuda.Stream()          # graph capture needs a stream of its own
    torch.cuda.set_stream(st)
    rounded, ctx, dec = make(cfg)
    args = (ctx, cfg.n_sub, cfg.delta_t, cfg.sub_tokens, cfg.time_steps)
    base = dec.generate(*args)
    dec.prefill_context(*args)
    done, got = False, np.full((cfg.batch, cfg.n_sub, cfg.sub_tokens), -1, dtype=np.int32)
    fill = np.zeros((cfg.batch, cfg.n_sub), dtype=int)
    while not done:
        toks, _, done = dec.decode_step()
        for b, i in zip(*np.nonzero(toks >= 0)):
            got[b, i, fill[b, i]] = toks[b, i]
            fill[b, i] += 1
    assert np.array_equal(got, base[0]) and np.array_equal(fill, base[1])
    for key, val in ((binding.PD_OPT_USE_GRAPH, 1), (binding.PD_OPT_ATTN_SPLITS, 3), (binding.PD_OPT_ATTN_SPLITS, 1),
                     (binding.PD_OPT_FUSE_NORM, 0)):
        dec.set_option(key, val)
        for rep in range(3 if key == binding.PD_OPT_USE_GRAPH else 1):
            again = dec.generate(*args)
            torch.cuda.synchronize()
            for a, b in zip(base, again):
                assert np.array_equal(a, b), f"option {key}={val} (run {rep}) changed the result"
        dec.set_option(key, 1 if key == binding.PD_OPT_FUSE_NORM else 0)
    other = (ctx[::-1].copy(),) + args[1:]
    second = dec.generate(*other)
    dec.close()
    _, _, fresh = make(cfg)
    first = fresh.generate(*other)
    for a, b in zip(first, second):
        assert np.array_equal(a, b)
    fresh.close()
    torch.cuda.set_stream(torch.cuda.default_stream())
