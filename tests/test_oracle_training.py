"""Pins for oracle/training.py (Section 3.3, Eq. 5-6, Fig. 3b).  CPU only."""

import numpy as np
import pytest
import torch

import pd_inputs as pi
from oracle import controller, pipelined, training
from oracle.model import OracleModel
from test_oracle_pins import tiny
from torch_dense import dense_logits


def setup(kind, **kw):
    kw = dict(dict(n_sub=6, delta_t=3, sub_tokens=8), **kw)      # sizes the learned position table
    cfg = tiny(kind, **kw)
    w = pi.make_weights(cfg, threads=2)
    ctx = pi.make_context(cfg)[0]
    return cfg, w, ctx, OracleModel(cfg, w)


def draw_target(cfg, lengths, seed=0):
    """Subsequences of the given lengths with ids that avoid <bos> and <eos>."""
    g = np.random.Generator(np.random.Philox(key=[cfg.seed, seed]))
    return [[int(t) for t in g.integers(2, cfg.vocab, size=n)] for n in lengths]


def test_target_of_fig_3b():
    """Fig. 3b's example: subsequences [A, B, C] and [D, E] become [bos, A, B, C, eos], [bos, D, E, eos]
    and the empty [bos, eos] (Eq. 5); Eq. 6 then has 4 + 3 + 1 = 8 terms."""
    A, B, C, D, E, bos, eos = 10, 11, 12, 13, 14, 0, 1
    tgt = training.training_target([[A, B, C], [D, E]], bos, eos)
    assert tgt == [[bos, A, B, C, eos], [bos, D, E, eos], [bos, eos]]
    cfg, w, ctx, model = setup("gelu", eos_id=eos)
    _, nll, loss = training.teacher_forced(model, ctx, tgt, 1)
    assert nll.shape == (11,) and int((nll > 0).sum()) == 8
    assert np.all(nll[[4, 8, 10]] == 0.0), "the closing <eos> of a subsequence has no term"
    assert loss == pytest.approx(nll.sum())


@pytest.mark.parametrize("kind,lengths,dt", [("gelu", [3, 2], 1), ("llama", [4, 2, 3], 2), ("bf16", [5, 3, 4, 3], 3)])
def test_loss_terms_are_the_distributions_of_algorithm_1(kind, lengths, dt):
    """Algorithm 1 run with the target's tokens forced produces, step by step, the distribution of every
    next token through the incremental decoder (explicit visible set per query, caches appended as the
    run goes); -log of the target's probability there is the same number the one-pass forward gives."""
    cfg, w, ctx, model = setup(kind, eos_id=1)
    Y = draw_target(cfg, lengths)
    tgt = training.training_target(Y, cfg.bos_id, cfg.eos_id)
    n = len(tgt)
    # the step that produces a subsequence's <eos> feeds its token before it: tau = (i-1) dt + len - 1
    T = max(i * dt + len(s) - 1 for i, s in enumerate(tgt))
    force = np.full((T, n), -1, dtype=np.int64)
    for i, s in enumerate(tgt):
        for j in range(1, len(s)):
            force[i * dt + j - 1, i] = s[j]              # token j is appended by the step that feeds token j - 1
    dec = pipelined.PerQueryDecoder(model, ctx, force=force)
    result, steps, _ = controller.pipelined_decode(dec, dt, 10 ** 6, n, cfg.bos_id, cfg.eos_id, 10 ** 6)
    assert result == Y + [[]] and steps == T, "the forced run reproduces the target and stops with the empty subsequence"
    logits, nll, loss = training.teacher_forced(model, ctx, tgt, dt)
    offset = np.concatenate([[0], np.cumsum([len(s) for s in tgt])])
    seen = 0
    for rec in dec.trace:
        for r, i in enumerate(rec["rows"]):
            j = rec["t"] - ((i - 1) * dt + 1)
            row = offset[i - 1] + j
            np.testing.assert_allclose(rec["logits"][r], logits[row], rtol=0, atol=1e-10)
            seen += 1
    # every token whose time lies inside the run is fed exactly once, closing <eos> tokens included; the
    # ones behind the last step (the loop has ended) are keys no token with a loss term can see
    inside = sum(1 for i, s in enumerate(tgt) for j in range(len(s)) if i * dt + 1 + j <= T)
    assert seen == inside and inside > sum(len(s) - 1 for s in tgt) - 1
    assert any(i * dt + len(s) <= T for i, s in enumerate(tgt)), "some closing <eos> is fed as a key"
    assert loss > 0


@pytest.mark.parametrize("kind,lengths,dt", [("gelu", [6], 1), ("llama", [3, 4, 2], 2), ("bf16", [4, 4, 4], 1)])
def test_loss_against_library_cross_entropy(kind, lengths, dt):
    """The independent PyTorch model under a mask and positions enumerated here, with the library's own
    cross-entropy.  One subsequence: the ordinary language-model loss of [input, bos, Y, eos] on the
    generated part."""
    cfg, w, ctx, model = setup(kind, eos_id=1)
    tgt = training.training_target(draw_target(cfg, lengths, seed=1), cfg.bos_id, cfg.eos_id)
    if len(lengths) == 1:
        tgt = tgt[:1]                                       # exactly one subsequence: plain causal LM
    L = len(ctx)
    fed = [(i, i * dt + j, tok) for i, s in enumerate(tgt) for j, tok in enumerate(s)]     # 0-based i, tau - 1
    N = len(fed)
    mask = np.zeros((L + N, L + N), dtype=bool)
    mask[:L, :L] = np.tril(np.ones((L, L), dtype=bool))
    mask[L:, :L] = True
    for a, (iq, tq, _) in enumerate(fed):
        for b, (ik, tk, _) in enumerate(fed):
            mask[L + a, L + b] = ik <= iq and tk <= tq
    pos = list(range(L)) + [L + t + i for i, t, _ in fed]
    if len(tgt) == 1:
        assert np.array_equal(mask, np.tril(np.ones((L + N, L + N), dtype=bool))) and pos == list(range(L + N))
    lg = dense_logits(cfg, w, list(ctx) + [f[2] for f in fed], pos, mask)[L:]
    rows, nxt = [], []
    r = 0
    for s in tgt:
        for j in range(len(s)):
            if j + 1 < len(s):
                rows.append(r)
                nxt.append(s[j + 1])
            r += 1
    want = torch.nn.functional.cross_entropy(torch.as_tensor(lg[rows]), torch.as_tensor(nxt), reduction="none").numpy()
    logits, nll, loss = training.teacher_forced(model, ctx, tgt, dt)
    np.testing.assert_allclose(logits, lg, rtol=0, atol=1e-10)
    np.testing.assert_allclose(nll[rows], want, rtol=0, atol=1e-10)
    assert loss == pytest.approx(float(want.sum()), abs=1e-9)


def test_planted_mistakes_change_the_loss():
    cfg, w, ctx, model = setup("gelu", eos_id=1)
    tgt = training.training_target(draw_target(cfg, [4, 3, 3], seed=2), cfg.bos_id, cfg.eos_id)
    _, nll, loss = training.teacher_forced(model, ctx, tgt, 1)
    # (a) the closing <eos> tokens left out of the keys: later tokens of higher subsequences change
    from oracle import matrix_form
    coords = [c for c in matrix_form.coordinates([s[:-1] for s in tgt], 1)]
    L = len(ctx)
    tokens = np.concatenate([ctx, [c[2] for c in coords]])
    pos = np.concatenate([np.arange(L), [L + (t - 1) + (i - 1) for i, t, _ in coords]])
    lg = matrix_form.dense_forward(model, tokens, pos, matrix_form.attention_matrix(L, coords))[L:]
    full_rows = [r for r, (s, j) in enumerate((s, j) for s in tgt for j in range(len(s))) if j + 1 < len(s)]
    ref, _, _ = training.teacher_forced(model, ctx, tgt, 1)
    assert np.abs(lg - ref[full_rows]).max() > 1e-3
    # (b) another delay moves the coordinates: another loss
    assert abs(training.teacher_forced(model, ctx, tgt, 2)[2] - loss) > 1e-6
    # (c) targets shifted by one token
    shifted = [s[:1] + s[2:] + s[1:2] for s in tgt]
    assert abs(training.teacher_forced(model, ctx, shifted, 1)[2] - loss) > 1e-6


def test_gpu_cases_can_see_a_wrong_matrix():
    """The GPU parity cases compare logits at 2e-2.  With either half of Fig. 3b's matrix dropped (a token
    seeing later tokens of lower subsequences, or tokens of higher subsequences), the oracle's own logits on
    such a case move by far more than that, so a kernel with that mistake cannot pass."""
    from oracle import matrix_form
    from test_gpu_parity import CASES
    from test_gpu_teacher_forced import draw_targets
    cfg = CASES["mfma-hd64"]
    w = pi.make_weights(cfg, threads=2)
    ctx = pi.make_context(cfg)[0]
    model = OracleModel(cfg, w)
    tgt = draw_targets(cfg, 1)[0]
    right, _, _ = training.teacher_forced(model, ctx, tgt, cfg.delta_t)
    L = len(ctx)
    coords = matrix_form.coordinates(tgt, cfg.delta_t)
    tokens = np.concatenate([ctx, [c[2] for c in coords]])
    pos = np.concatenate([np.arange(L), [L + (t - 1) + (i - 1) for i, t, _ in coords]])
    for drop in ("time", "subsequence"):
        mask = matrix_form.attention_matrix(L, coords)
        for a, (iq, tq, _) in enumerate(coords):
            for b, (ik, tk, _) in enumerate(coords):
                mask[L + a, L + b] = (ik <= iq) if drop == "time" else (tk <= tq)
        wrong = matrix_form.dense_forward(model, tokens, pos, mask)[L:]
        assert np.abs(wrong - right).max() > 0.06, drop         # three times the bar


# --------------------------------------------------------------------------
# encoder-decoder form
# --------------------------------------------------------------------------
ED = pi.EncDecConfig(name="encdec-train", seed=57, n_enc_layer=2, n_dec_layer=2, d_model=32, n_head=4, head_dim=6,
                     d_ff=48, vocab=83, rel_buckets=8, rel_max_distance=20, ctx_len=17, eos_id=1)


def ed_setup():
    from oracle import encdec
    w = pi.make_encdec_weights(ED)
    g = np.random.Generator(np.random.Philox(key=[(ED.seed << 32) | 0xC0DE, 1]))
    return encdec.EncDecModel(ED, w), w, g.integers(0, ED.vocab, size=ED.ctx_len)


@pytest.mark.parametrize("lengths,dt", [([3, 2], 1), ([4, 2, 3], 2), ([5, 3, 4, 3], 3)])
def test_encdec_loss_terms_are_the_distributions_of_algorithm_1(lengths, dt):
    from oracle import encdec
    model, w, ctx = ed_setup()
    tgt = training.training_target(draw_target(ED, lengths), ED.bos_id, ED.eos_id)
    n = len(tgt)
    T = max(i * dt + len(s) - 1 for i, s in enumerate(tgt))
    force = np.full((T, n), -1, dtype=np.int64)
    for i, s in enumerate(tgt):
        for j in range(1, len(s)):
            force[i * dt + j - 1, i] = s[j]
    dec = encdec.EncDecPerQueryDecoder(model, ctx, force=force)
    result, steps, _ = controller.pipelined_decode(dec, dt, 10 ** 6, n, ED.bos_id, ED.eos_id, 10 ** 6)
    assert result == [s[1:-1] for s in tgt] and steps == T
    logits, nll, loss = training.teacher_forced_encdec(model, ctx, tgt, dt)
    offset = np.concatenate([[0], np.cumsum([len(s) for s in tgt])])
    seen = 0
    for rec in dec.trace:
        for r, i in enumerate(rec["rows"]):
            row = offset[i - 1] + rec["t"] - ((i - 1) * dt + 1)
            np.testing.assert_allclose(rec["logits"][r], logits[row], rtol=0, atol=1e-10)
            seen += 1
    assert seen == sum(1 for i, s in enumerate(tgt) for j in range(len(s)) if i * dt + 1 + j <= T)
    assert int((nll > 0).sum()) == sum(len(s) - 1 for s in tgt) and loss == pytest.approx(nll.sum())


def test_encdec_loss_against_library_cross_entropy():
    from torch_encdec import encode as torch_encode, decode_logits
    model, w, ctx = ed_setup()
    dt = 2
    tgt = training.training_target(draw_target(ED, [4, 3, 2], seed=3), ED.bos_id, ED.eos_id)
    fed = [(i, i * dt + j, tok) for i, s in enumerate(tgt) for j, tok in enumerate(s)]
    N = len(fed)
    mask = np.zeros((N, N), dtype=bool)
    dist = np.zeros((N, N), dtype=np.int64)
    for a, (iq, tq, _) in enumerate(fed):
        for b, (ik, tk, _) in enumerate(fed):
            mask[a, b] = ik <= iq and tk <= tq
            dist[a, b] = abs(tq - tk) + abs(iq - ik)
    lg = decode_logits(ED, w, torch_encode(ED, w, ctx), [f[2] for f in fed], mask, dist)
    rows, nxt, r = [], [], 0
    for s in tgt:
        for j in range(len(s)):
            if j + 1 < len(s):
                rows.append(r)
                nxt.append(s[j + 1])
            r += 1
    want = torch.nn.functional.cross_entropy(torch.as_tensor(np.asarray(lg)[rows]), torch.as_tensor(nxt),
                                             reduction="none").numpy()
    logits, nll, loss = training.teacher_forced_encdec(model, ctx, tgt, dt)
    np.testing.assert_allclose(logits, np.asarray(lg), rtol=0, atol=1e-10)
    np.testing.assert_allclose(nll[rows], want, rtol=0, atol=1e-10)
    assert loss == pytest.approx(float(want.sum()), abs=1e-9)
