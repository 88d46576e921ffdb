"""GPU parity of the teacher-forced forward (Section 3.3, Eq. 5-6, Fig. 3b) against oracle/training.py:
logits of every target token, the loss term of every token with a successor, and the loss."""

import numpy as np
import pytest

import pd_inputs as pi
from oracle import training
from oracle.model import OracleModel
from parity_util import make_decoder
from test_gpu_parity import CASES, small, DTYPE_BF16

pytestmark = pytest.mark.gpu

TOL = 2e-2          # logits, the bf16 bar; a loss term is a difference of two such quantities


def say(*a):
    print(*a, flush=True)


def draw_targets(cfg, n_req, salt=0, row_cap=120):
    """Per request a training target (Eq. 5): 2 .. n_sub - 1 subsequences of 1 .. M - 1 tokens between <bos>
    and <eos>, then the empty one; ids avoid <bos> and <eos>; at most row_cap tokens in all (one pass of rows
    of the small test configurations)."""
    g = np.random.Generator(np.random.Philox(key=[cfg.seed, 0x7EAC + salt]))
    eos = cfg.eos_id if cfg.eos_id >= 0 else 1
    out = []
    for _ in range(n_req):
        n = int(g.integers(2, cfg.n_sub)) if cfg.n_sub > 2 else 1
        Y = [[int(t) for t in g.integers(2, cfg.vocab, size=int(g.integers(1, cfg.sub_tokens)))] for _ in range(n)]
        while sum(len(y) + 2 for y in Y) + 2 > row_cap:
            Y.pop()
        out.append(training.training_target(Y, cfg.bos_id, eos))
    return out


def check(cfg, targets, w=None, ctx=None, dec=None):
    w = pi.make_weights(cfg, threads=4) if w is None else w
    ctx = pi.make_context(cfg) if ctx is None else ctx
    own = dec is None
    dec = make_decoder(cfg, w) if own else dec
    dec.prefill_context(ctx, cfg.n_sub, cfg.delta_t, cfg.sub_tokens, cfg.time_steps)
    logits, nll, loss = dec.teacher_forced(targets)
    model = OracleModel(cfg, w)
    worst = worst_nll = 0.0
    rows = terms = 0
    for b, tgt in enumerate(targets):
        want_logits, want_nll, want_loss = training.teacher_forced(model, ctx[b], tgt, cfg.delta_t)
        got = logits[b].cpu().numpy().astype(np.float64)
        assert got.shape == want_logits.shape
        err = np.abs(got - want_logits).max()
        assert np.isfinite(err) and err <= TOL, f"request {b}: max|logit diff| = {err:.3e}"
        worst = max(worst, err)
        e2 = np.abs(nll[b] - want_nll).max()
        assert e2 <= 2 * TOL, f"request {b}: max|loss term diff| = {e2:.3e}"
        assert np.array_equal(nll[b] == 0, want_nll == 0), "terms exactly where a token has a successor"
        worst_nll = max(worst_nll, e2)
        n_terms = int((want_nll != 0).sum())
        assert abs(loss[b] - want_loss) <= 2 * TOL * n_terms
        assert loss[b] == pytest.approx(float(np.sum(nll[b].astype(np.float64))), abs=1e-9), "terms added in row order, in fp64"
        rows += len(want_nll)
        terms += n_terms
    say(f"[teacher-forced] {cfg.name}: {len(targets)} requests, {rows} rows, {terms} loss terms, "
        f"max|logit diff| = {worst:.3e}, max|term diff| = {worst_nll:.3e}")
    if own:
        dec.close()
    return worst


@pytest.mark.parametrize("name", ["mfma-hd64", "mfma-hd128-llama", "mfma-hd32", "mfma-hd96", "mfma-manyrows"])
def test_teacher_forced_parity(name):
    cfg = CASES[name]
    check(cfg, draw_targets(cfg, cfg.batch))


def test_fig_3b_shape_and_single_subsequence():
    """Fig. 3b's shape ([bos A B C eos], [bos D E eos], [bos eos]) at delta_t = 1, and one subsequence alone,
    where the matrix is the ordinary causal one."""
    cfg = small("tf-fig3b", seed=71, dtype=DTYPE_BF16, d_model=128, n_head=2, head_dim=64, d_ff=256, vocab=500,
                ctx_len=40, n_sub=3, delta_t=1, sub_tokens=4, batch=2)
    fig = [[cfg.bos_id, 10, 11, 12, 1], [cfg.bos_id, 13, 14, 1], [cfg.bos_id, 1]]
    check(cfg, [fig, [[cfg.bos_id, 20, 21, 22, 23, 1]]])


def test_more_rows_than_one_row_group_and_decoding_afterwards():
    """240 .. 300 target tokens per request (the many-row projection kernels), and the context still decodes
    as before afterwards."""
    cfg = small("tf-many", seed=72, dtype=DTYPE_BF16, d_model=128, n_head=2, head_dim=64, d_ff=256, vocab=640,
                ctx_len=300, n_sub=24, delta_t=2, sub_tokens=14, batch=2, n_layer=2)
    w = pi.make_weights(cfg, threads=4)
    ctx = pi.make_context(cfg)
    dec = make_decoder(cfg, w)
    args = (ctx, cfg.n_sub, cfg.delta_t, cfg.sub_tokens, cfg.time_steps)
    before = dec.generate(*args)
    g = np.random.Generator(np.random.Philox(key=[cfg.seed, 5]))
    targets = [training.training_target([[int(t) for t in g.integers(2, cfg.vocab, size=int(g.integers(9, 13)))]
                                         for _ in range(22)], cfg.bos_id, 1) for _ in range(cfg.batch)]
    assert all(sum(len(s) for s in t) > 256 for t in targets)
    check(cfg, targets, w=w, ctx=ctx, dec=dec)
    dec.prefill_context(*args)
    dec.teacher_forced(targets)
    dec.decode_steps(3)                      # the context restarts at t = 0 after the forward
    dec.reset_decode()
    after = dec.generate(*args)
    for a, b in zip(before, after):
        assert np.array_equal(a, b)
    dec.close()


def test_teacher_forced_rejects_what_it_cannot_run():
    from paper_2506_23431_amd.binding import PdError
    cfg = CASES["mfma-hd64"]
    w = pi.make_weights(cfg, threads=4)
    ctx = pi.make_context(cfg)
    dec = make_decoder(cfg, w)
    with pytest.raises(PdError, match="before pd_prefill_context"):
        dec.B, dec.S = cfg.batch, cfg.n_sub
        dec.teacher_forced([[[0, 1]]] * cfg.batch)
    dec.prefill_context(ctx, cfg.n_sub, cfg.delta_t, cfg.sub_tokens, cfg.time_steps)
    with pytest.raises(PdError, match="max_len"):
        dec.teacher_forced([[[0] * (cfg.sub_tokens + 3)]] * cfg.batch)
    with pytest.raises(PdError, match="follows an empty one"):
        arr = [[[0, 5, 1], [], [0, 1]]] * cfg.batch
        dec.teacher_forced([[s if s else [] for s in t] for t in arr])
    with pytest.raises(PdError, match="out of range"):
        dec.teacher_forced([[[0, cfg.vocab, 1]]] * cfg.batch)
    dec.close()
    f32 = CASES["cfg1"] if "cfg1" in CASES else None
    if f32 is not None:
        d2 = make_decoder(f32, pi.make_weights(f32, threads=2))
        d2.prefill_context(pi.make_context(f32), f32.n_sub, f32.delta_t, f32.sub_tokens, f32.time_steps)
        with pytest.raises(PdError, match="matrix-core"):
            d2.teacher_forced([[[0, 1]]] * f32.batch)
        d2.close()


def test_teacher_forced_at_the_full_size_of_cfg2():
    """The 768-wide workload at full size (6 layers, 12 heads of 64, vocabulary 50265, 1024 context tokens):
    one training target of 7 subsequences of 40 .. 63 tokens and the empty one, about 360 rows in one pass."""
    cfg = pi.get_config("cfg2")
    g = np.random.Generator(np.random.Philox(key=[cfg.seed, 9]))
    Y = [[int(t) for t in g.integers(2, cfg.vocab, size=int(g.integers(40, 64)))] for _ in range(7)]
    target = training.training_target(Y, cfg.bos_id, 1)
    assert sum(len(s) for s in target) > 300
    worst = check(cfg, [target])
    assert worst < 5e-3
