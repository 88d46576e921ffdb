"""Pins for the CPU oracle: everything here checks oracle/ against something other
than itself -- the paper's worked example (Fig. 2), closed forms of Section 3.2,
an independent PyTorch dense transformer, brute-force enumeration of the
dependency rule -- and checks that planted mistakes are caught.  CPU only."""

import itertools
import math
import os

import numpy as np
import pytest

import pd_inputs as pi
from pd_inputs.configs import (WorkloadConfig, DTYPE_F32, DTYPE_BF16, FFN_GELU, FFN_SWIGLU,
                               NORM_LAYERNORM, NORM_RMSNORM, POS_LEARNED, POS_ROPE)
from oracle import controller, pipelined, matrix_form, splitk
from oracle.model import OracleModel
from torch_dense import dense_logits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny(kind="gelu", **kw):
    base = dict(name="tiny-" + kind, seed=11, dtype=DTYPE_F32, n_layer=2, d_model=32, n_head=4,
                head_dim=8, d_ff=64, vocab=97, batch=1, ctx_len=9, n_sub=3, delta_t=2,
                sub_tokens=4, norm_init="random")
    if kind == "llama":
        base.update(ffn_kind=FFN_SWIGLU, norm_kind=NORM_RMSNORM, pos_kind=POS_ROPE, d_ff=48,
                    seed=12)
    if kind == "bf16":
        base.update(dtype=DTYPE_BF16, seed=13)
    base.update(kw)
    return WorkloadConfig(**base)


def setup(cfg):
    w = pi.make_weights(cfg, threads=2)
    ctx = pi.make_context(cfg)[0]
    return OracleModel(cfg, w), w, ctx


def run(cfg, model, ctx, **kw):
    args = dict(n_sub=cfg.n_sub, delta_t=cfg.delta_t, sub_tokens=cfg.sub_tokens,
                time_max=kw.pop("time_max", 10 ** 6), bos_id=cfg.bos_id, eos_id=cfg.eos_id)
    args.update(kw)
    return pipelined.generate(model, ctx, **args)


# --------------------------------------------------------------------------
# Eq. 4 with ties: the most probable token, the lowest index among equals
# --------------------------------------------------------------------------

def _argmax_by_hand(v):
    best, bi = None, -1
    for j, x in enumerate(v):            # ascending scan, strict comparison: the first maximum stays
        if best is None or x > best:
            best, bi = x, j
    return bi


def test_argmax_takes_the_lowest_index_among_equal_maxima():
    from oracle import primitives as P
    rng = np.random.default_rng(5)
    for n in (1, 2, 17, 300, 2100):
        for _ in range(20):
            v = rng.standard_normal(n)
            k = int(rng.integers(1, min(n, 6) + 1))
            where = rng.choice(n, size=k, replace=False)
            v[where] = v.max() + 1.0                      # k exact copies of the maximum
            assert P.argmax_lowest(v) == int(where.min()) == _argmax_by_hand(v)
    assert P.argmax_lowest(np.zeros(9)) == 0              # everything ties
    assert P.argmax_lowest(np.array([-np.inf, 3.0, 3.0, -np.inf])) == 1


def test_tied_logits_select_the_lowest_index_through_a_whole_run():
    """A vocabulary projection with duplicated rows: in every row of every iteration one of two
    groups of identical rows holds the largest logit several times over; the free-running oracle
    must append the lowest index of that group each time."""
    cfg = tiny(seed=16, d_model=128, n_head=2, head_dim=64, d_ff=96, vocab=2100, n_sub=3, delta_t=1, sub_tokens=4)
    w = pi.make_weights(cfg, threads=2)
    group_a, group_b = [37, 38, 45, 1061, 2085], [41, 600, 601, 1500]
    pi.tie_lm_head(cfg, w, group_a, group_b)
    out = run(cfg, OracleModel(cfg, w), pi.make_context(cfg)[0])
    seen = set()
    for rec, em in zip(out["trace"], out["emitted"]):
        for r, i in enumerate(rec["rows"]):
            lg = rec["logits"][r]
            tied = np.flatnonzero(lg == lg.max())
            assert tied.tolist() in (group_a, group_b), "the maximum is not one whole group of duplicates"
            assert np.sort(lg)[-len(tied) - 1] < lg.max() - 0.05
            if i in em:
                assert em[i] == tied.min() == _argmax_by_hand(lg)
                seen.add(int(em[i]))
    assert seen == {37, 41}, "the run should meet both groups"


# --------------------------------------------------------------------------
# Fig. 2 / Section 3.1: the worked example, with a scripted decoder
# --------------------------------------------------------------------------

def _read_fig2():
    names, script, steps, result = {}, {}, [], []
    for line in open(os.path.join(GOLDEN, "fig2_schedule.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        key, _, rest = line.partition(":")
        if key == "token":
            n, v = rest.split()
            names[n] = int(v)
        elif key == "script":
            i, *toks = rest.split()
            script[int(i)] = [names[t] for t in toks]
        elif key == "step":
            t, *pairs = rest.split()
            steps.append({int(p.split("=")[0]): names[p.split("=")[1]] for p in pairs})
        elif key == "result":
            i, *toks = rest.split()
            result.append([names[t] for t in toks])
    return names, script, steps, result


def test_fig2_schedule_with_scripted_decoder():
    names, script, steps, result = _read_fig2()

    def scripted(G, t):
        return [script[i][len(g) - 1] if len(g) - 1 < len(script[i]) else names["eos"]
                for i, g in enumerate(G, start=1)]

    res, n_steps, emitted = controller.pipelined_decode(
        scripted, delta_t=1, time_max=50, sub_max=20, bos_id=names["bos"], eos_id=names["eos"])
    assert n_steps == 4                      # "only costs 4 time-steps"
    assert emitted == steps                  # 1, 2, 2(+eos of the exploratory one), then all eos
    assert [len(e) for e in emitted][:3] == [1, 2, 3]
    assert res == result


def test_fig2_dependency_sets():
    """'D' depends only on 'A' and two <bos> tokens (Section 3.2); 'E' additionally on B and D
    but not on C, which is produced in the same iteration as E."""
    names, script, _, _ = _read_fig2()
    cfg = tiny(vocab=32, n_sub=20, delta_t=1, sub_tokens=50)
    model, _, ctx = setup(cfg)
    force = np.full((8, 20), names["eos"], dtype=np.int64)
    for i, toks in script.items():
        for j, tok in enumerate(toks):
            force[(i - 1) + j][i - 1] = tok
    out = pipelined.generate(model, ctx, n_sub=20, delta_t=1, sub_tokens=50, time_max=50,
                             bos_id=names["bos"], eos_id=names["eos"], force=force)
    assert out["steps"] == 4
    tok_at = {}
    for rec in out["trace"]:
        for i, tok in zip(rec["rows"], rec["tokens_in"]):
            tok_at[(i, rec["t"])] = tok
    inv = {v: k for k, v in names.items()}

    def deps(i, t):
        rec = out["trace"][t - 1]
        return sorted(inv[tok_at[c]] + str(c[0]) for c in rec["vis"][rec["rows"].index(i)])

    # the query that emits D is <bos> of subsequence 2, fed in iteration 2
    assert deps(2, 2) == sorted(["bos1", "A1", "bos2"])
    # the query that emits E is D, fed in iteration 3
    assert deps(2, 3) == sorted(["bos1", "A1", "B1", "bos2", "D2"])
    # subsequence 1 never sees subsequence 2
    assert deps(1, 3) == sorted(["bos1", "A1", "B1"])


# --------------------------------------------------------------------------
# Section 3.2 closed forms: k = ceil(t/dt); token (i, j) is generated at (i-1)dt + j
# --------------------------------------------------------------------------

@pytest.mark.parametrize("S,dt,M", [(4, 2, 16), (8, 4, 64), (16, 4, 32), (32, 8, 64), (5, 1, 3),
                                    (3, 7, 2), (1, 3, 5)])
def test_schedule_closed_forms(S, dt, M):
    ks = []

    def dec(G, t):
        ks.append(len(G))
        return [1000 * i + len(g) for i, g in enumerate(G, start=1)]   # token encodes (i, j)

    res, steps, emitted = controller.pipelined_decode(dec, dt, 10 ** 6, S, bos_id=0,
                                                      sub_tokens=M)
    if M + 1 > dt or S == 1:     # pipelines overlap (or nothing to overlap): the run is complete
        assert steps == (S - 1) * dt + M
        assert sum(len(r) for r in res) == S * M
        for t, k in enumerate(ks, start=1):
            assert k == min(S, math.ceil(t / dt))
        for t, em in enumerate(emitted, start=1):
            for i, tok in em.items():
                j = tok - 1000 * i
                assert t == (i - 1) * dt + j
    else:
        # every open subsequence finishes before the next one opens: the loop stops early
        assert steps == M and len(res) == 1


def test_early_stop_counts_only_opened_subsequences():
    # dt larger than the subsequence: after M steps the only open subsequence is complete
    res, steps, _ = controller.pipelined_decode(lambda G, t: [5] * len(G), 5, 100, 4, bos_id=0,
                                                sub_tokens=2)
    assert steps == 2 and res == [[5, 5]]


def test_time_max_bounds_the_loop():
    res, steps, _ = controller.pipelined_decode(lambda G, t: [5] * len(G), 1, 3, 10, bos_id=0)
    assert steps == 3 and [len(r) for r in res] == [3, 2, 1]


# --------------------------------------------------------------------------
# Dependency rule, enumerated by brute force
# --------------------------------------------------------------------------

@pytest.mark.parametrize("S,dt,M,L", [(3, 2, 4, 5), (4, 1, 3, 0), (3, 3, 5, 2), (5, 2, 2, 1)])
def test_visible_sets_match_brute_force(S, dt, M, L):
    cfg = tiny(vocab=40, n_sub=S, delta_t=dt, sub_tokens=M, ctx_len=max(L, 1), n_layer=1)
    model, _, ctx = setup(cfg)
    ctx = ctx[:L]
    out = pipelined.generate(model, ctx, n_sub=S, delta_t=dt, sub_tokens=M, time_max=10 ** 6,
                             bos_id=0)
    # every token that is ever fed: <bos> at (i-1)dt+1, then one per step, M generated in all
    first = {i: (i - 1) * dt + 1 for i in range(1, S + 1)}
    last = {i: first[i] + M for i in range(1, S + 1)}
    for rec in out["trace"]:
        t = rec["t"]
        for r, i in enumerate(rec["rows"]):
            brute = {(ii, tau) for ii in range(1, S + 1) for tau in range(first[ii], last[ii] + 1)
                     if ii <= i and tau <= t}
            assert set(rec["vis"][r]) == brute
            closed = sum(max(0, min(t, last[ii]) - first[ii] + 1) for ii in range(1, i + 1))
            assert len(rec["vis"][r]) == closed
            assert rec["positions"][r] == L + (t - 1) + (i - 1)


def test_manhattan_distance_is_position_difference():
    """Section 4.3: relative distance |t1-t2| + |i1-i2|.  On visible pairs it equals p_q - p_k."""
    L = 7
    for iq, tq, ik, tk in itertools.product(range(1, 6), range(1, 9), range(1, 6), range(1, 9)):
        if ik <= iq and tk <= tq:
            d = abs(tq - tk) + abs(iq - ik)
            assert d == pipelined.position(L, iq, tq) - pipelined.position(L, ik, tk) >= 0


# --------------------------------------------------------------------------
# Special cases that reduce to a textbook routine (independent PyTorch model)
# --------------------------------------------------------------------------

def _greedy_textbook(cfg, w, ctx, n_new):
    """Ordinary greedy decoding of a causal LM on prompt = context + <bos>: full recompute."""
    seq = list(ctx) + [cfg.bos_id]
    all_logits = []
    for _ in range(n_new):
        lg = dense_logits(cfg, w, seq, np.arange(len(seq)))[-1]
        all_logits.append(lg)
        seq.append(int(np.argmax(lg)))
    return seq[len(ctx) + 1:], np.stack(all_logits)


@pytest.mark.parametrize("kind", ["gelu", "llama", "bf16"])
def test_single_subsequence_is_ordinary_greedy_decoding(kind):
    cfg = tiny(kind, n_sub=1, sub_tokens=6)
    model, w, ctx = setup(cfg)
    out = run(cfg, model, ctx)
    toks, logits = _greedy_textbook(cfg, w, ctx, 6)
    assert out["result"] == [toks]
    mine = np.stack([rec["logits"][0] for rec in out["trace"]])
    np.testing.assert_allclose(mine, logits, rtol=0, atol=1e-10)


@pytest.mark.parametrize("kind", ["gelu", "llama"])
def test_first_subsequence_is_always_ordinary_greedy_decoding(kind):
    cfg = tiny(kind, n_sub=3, delta_t=2, sub_tokens=5)
    model, w, ctx = setup(cfg)
    out = run(cfg, model, ctx)
    toks, logits = _greedy_textbook(cfg, w, ctx, 5)
    assert out["result"][0] == toks
    mine = np.stack([rec["logits"][rec["rows"].index(1)] for rec in out["trace"][:5]])
    np.testing.assert_allclose(mine, logits, rtol=0, atol=1e-10)


@pytest.mark.parametrize("kind", ["gelu", "llama"])
def test_no_overlap_is_plain_causal_decoding_with_explicit_positions(kind):
    """Subsequences opened M+1 steps apart: each one (incl. its last token) is complete before
    the next opens, so every query sees everything before it; only the position ids are unusual.
    Algorithm 1 itself would stop after the first subsequence here (all opened ones are complete),
    so the decoder is driven by a loop without that test."""
    S, M = 3, 3
    cfg = tiny(kind, n_sub=S, delta_t=M + 1, sub_tokens=M)
    model, w, ctx = setup(cfg)
    dec = pipelined.PerQueryDecoder(model, ctx)
    G = []
    for t in range(1, S * (M + 1) + 1):
        if (t - 1) % (M + 1) == 0:
            G.append([cfg.bos_id])
        new = dec(G, t)
        for i, g in enumerate(G):
            if len(g) - 1 < M:
                g.append(new[i])
    L = len(ctx)
    seq, pos, got, want = list(ctx), list(range(L)), [], []
    for i in range(1, S + 1):
        for j in range(M + 1):               # <bos> and M tokens are fed; the last one drains
            tau = (i - 1) * (M + 1) + 1 + j
            seq.append(G[i - 1][j])
            pos.append(pipelined.position(L, i, tau))
            assert pos[-1] == L + (tau - 1) + (i - 1)
            rec = dec.trace[tau - 1]
            assert rec["rows"] == [i]
            if j < M:
                got.append(rec["logits"][0])
                want.append(dense_logits(cfg, w, seq, pos)[-1])
                assert int(np.argmax(want[-1])) == G[i - 1][j + 1]
    np.testing.assert_allclose(np.stack(got), np.stack(want), rtol=0, atol=1e-10)


@pytest.mark.parametrize("kind,S,dt,M", [("gelu", 3, 2, 4), ("llama", 4, 1, 3), ("bf16", 3, 3, 5)])
def test_any_schedule_equals_dense_model_under_enumerated_mask(kind, S, dt, M):
    """Final check of the logits on overlapping schedules: rebuild the complete run as ONE dense
    forward of the PyTorch model over all fed tokens, under a mask enumerated directly from the
    rule (i_k <= i_q and tau_k <= tau_q, plus all context), and compare every produced logit row."""
    cfg = tiny(kind, n_sub=S, delta_t=dt, sub_tokens=M)
    model, w, ctx = setup(cfg)
    out = run(cfg, model, ctx)
    L = len(ctx)
    fed = [(i, rec["t"], tok) for rec in out["trace"] for i, tok in zip(rec["rows"], rec["tokens_in"])]
    n = len(fed)
    mask = np.zeros((L + n, L + n), dtype=bool)
    for a in range(L):
        mask[a, :a + 1] = True
    for a, (iq, tq, _) in enumerate(fed):
        mask[L + a, :L] = True
        for b, (ik, tk, _) in enumerate(fed):
            mask[L + a, L + b] = ik <= iq and tk <= tq
    tokens = list(ctx) + [f[2] for f in fed]
    pos = list(range(L)) + [L + (t - 1) + (i - 1) for i, t, _ in fed]
    want = dense_logits(cfg, w, tokens, pos, mask)[L:]
    got = np.concatenate([rec["logits"] for rec in out["trace"]])
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-10)
    assert n == S * (M + 1) - 1              # the very last token is never fed


# --------------------------------------------------------------------------
# Corollaries and the two formulations
# --------------------------------------------------------------------------

def test_lower_subsequences_do_not_depend_on_higher_ones():
    cfg = tiny("gelu", n_sub=4, delta_t=1, sub_tokens=4)
    model, _, ctx = setup(cfg)
    a = run(cfg, model, ctx)
    b = run(cfg.scaled(n_sub=2), model, ctx, n_sub=2)
    assert a["result"][:2] == b["result"]
    for ra, rb in zip(a["trace"], b["trace"]):
        for i in rb["rows"]:
            np.testing.assert_allclose(ra["logits"][ra["rows"].index(i)],
                                       rb["logits"][rb["rows"].index(i)], rtol=0, atol=1e-12)


@pytest.mark.parametrize("kind,S,dt,M", [("gelu", 3, 2, 4), ("llama", 3, 1, 3)])
def test_per_query_loop_equals_matrix_masked_form(kind, S, dt, M):
    cfg = tiny(kind, n_sub=S, delta_t=dt, sub_tokens=M)
    model, _, ctx = setup(cfg)
    f1 = run(cfg, model, ctx)
    dec = matrix_form.MatrixDecoder(model, ctx, dt)
    res, steps, emitted = controller.pipelined_decode(dec, dt, 10 ** 6, S, cfg.bos_id, -1, M)
    assert res == f1["result"] and steps == f1["steps"] and emitted == f1["emitted"]
    for r1, r2 in zip(f1["trace"], dec.trace):
        for r, i in enumerate(r1["rows"]):
            assert r2["last_tau"][i] == r1["t"]
            np.testing.assert_allclose(r1["logits"][r], r2["logits"][i], rtol=0, atol=1e-10)


def test_matrix_form_with_eos_and_forced_tokens():
    cfg = tiny("gelu", n_sub=3, delta_t=1, sub_tokens=6, vocab=50)
    model, _, ctx = setup(cfg)
    eos = 7
    force = 8 + pi.make_forced_tokens(cfg, 12)[:, 0, :].astype(np.int64) % (cfg.vocab - 8)
    force[2, 0] = eos                        # subsequence 1 ends in iteration 3
    f1 = pipelined.generate(model, ctx, 3, 1, 6, 100, cfg.bos_id, eos_id=eos, force=force)
    dec = matrix_form.MatrixDecoder(model, ctx, 1, force=force)
    res, steps, emitted = controller.pipelined_decode(dec, 1, 100, 3, cfg.bos_id, eos, 6)
    assert res == f1["result"] and steps == f1["steps"]
    assert len(res[0]) == 2                  # two tokens, then <eos>
    # iteration 4 feeds the <eos> of subsequence 1 once (draining row), then never again
    assert 1 in f1["trace"][3]["rows"] and all(1 not in r["rows"] for r in f1["trace"][4:])
    for r1, r2 in zip(f1["trace"], dec.trace):
        for r, i in enumerate(r1["rows"]):
            np.testing.assert_allclose(r1["logits"][r], r2["logits"][i], rtol=0, atol=1e-10)


def test_row_order_within_a_step_is_irrelevant():
    cfg = tiny("gelu", n_sub=4, delta_t=1, sub_tokens=4)
    model, _, ctx = setup(cfg)
    a = run(cfg, model, ctx)
    b = run(cfg, model, ctx, row_order=lambda rows: rows[::-1])
    assert a["result"] == b["result"]
    for ra, rb in zip(a["trace"], b["trace"]):
        for i in ra["rows"]:
            np.testing.assert_allclose(ra["logits"][ra["rows"].index(i)],
                                       rb["logits"][rb["rows"].index(i)], rtol=0, atol=1e-12)


def test_split_k_merge_is_exact():
    rng = np.random.default_rng(5)
    K, V, q = rng.standard_normal((37, 8)) * 3, rng.standard_normal((37, 8)), rng.standard_normal(8)
    want = splitk.attention(q, K, V, 0.35)
    for cuts in ([0, 37], [0, 1, 37], [0, 0, 5, 5, 36, 37], [0, 10, 20, 30, 37], list(range(38))):
        parts = [splitk.partial(q, K[a:b], V[a:b], 0.35) for a, b in zip(cuts[:-1], cuts[1:])]
        np.testing.assert_allclose(splitk.merge(parts), want, rtol=1e-12, atol=1e-14)
    # also equals SciPy's softmax
    from scipy.special import softmax
    np.testing.assert_allclose(want, softmax(K @ q * 0.35) @ V, rtol=1e-12)


# --------------------------------------------------------------------------
# End-of-sequence semantics on the small fp32 workload
# --------------------------------------------------------------------------

def test_eos_ends_a_subsequence_and_its_last_token_stays_visible():
    cfg = pi.get_config("cfg1")
    model, _, ctx = setup(cfg)
    free = run(cfg, model, ctx)
    eos = free["result"][1][5]               # a token subsequence 2 is seen to emit mid-way
    out = run(cfg.scaled(eos_id=eos), model, ctx, eos_id=eos)
    first_hit = free["result"][1].index(eos)
    assert out["result"][1] == free["result"][1][:first_hit]
    t_end = cfg.delta_t + first_hit + 1      # iteration in which subsequence 2 emitted <eos>
    assert 2 in out["trace"][t_end]["rows"]                       # fed once more (draining) ...
    assert all(2 not in r["rows"] for r in out["trace"][t_end + 1:])   # ... then never again
    rec = out["trace"][t_end + 1]
    for r, i in enumerate(rec["rows"]):       # and its <eos> stays visible to later subsequences
        assert ((2, t_end + 1) in rec["vis"][r]) == (i >= 2)


# --------------------------------------------------------------------------
# Planted mistakes must be caught by the pins above
# --------------------------------------------------------------------------

def _expect_failure(test, *args):
    with pytest.raises(AssertionError):
        test(*args)


def test_planted_mistakes_are_caught(monkeypatch):
    orig_vis = pipelined.PerQueryDecoder.visible
    # (a) strict inequality on the subsequence index: a query no longer sees its own subsequence
    monkeypatch.setattr(pipelined.PerQueryDecoder, "visible",
                        lambda self, i, t: [n for n in orig_vis(self, i, t) if self.gen_sub[n] < i])
    _expect_failure(test_fig2_dependency_sets)
    _expect_failure(test_single_subsequence_is_ordinary_greedy_decoding, "gelu")
    # (b) same-step tokens of lower subsequences hidden
    monkeypatch.setattr(pipelined.PerQueryDecoder, "visible",
                        lambda self, i, t: [n for n in orig_vis(self, i, t)
                                            if self.gen_tau[n] < t or self.gen_sub[n] == i])
    _expect_failure(test_fig2_dependency_sets)
    _expect_failure(test_any_schedule_equals_dense_model_under_enumerated_mask, "gelu", 3, 2, 4)
    # (c) every cached token visible (sequential-style dependency)
    monkeypatch.setattr(pipelined.PerQueryDecoder, "visible",
                        lambda self, i, t: list(range(len(self.gen_sub))))
    _expect_failure(test_fig2_dependency_sets)
    _expect_failure(test_visible_sets_match_brute_force, 3, 2, 4, 5)
    monkeypatch.setattr(pipelined.PerQueryDecoder, "visible", orig_vis)
    # (d) wrong position law
    monkeypatch.setattr(pipelined, "position", lambda L, i, tau: L + (tau - 1))
    _expect_failure(test_no_overlap_is_plain_causal_decoding_with_explicit_positions, "gelu")
    _expect_failure(test_manhattan_distance_is_position_difference)
    monkeypatch.undo()
    # (e) missing 1/sqrt(hd), transposed weight, dropped residual
    from oracle import model as om
    orig_after = om.OracleModel.after_attention
    monkeypatch.setattr(om.OracleModel, "after_attention",
                        lambda self, lw, x, attn: orig_after(self, lw, x, attn) - x)
    _expect_failure(test_single_subsequence_is_ordinary_greedy_decoding, "llama")
    monkeypatch.undo()
    orig_rope = om.P.rope
    monkeypatch.setattr(om.P, "rope", lambda x, pos, base: orig_rope(x, pos, base * 2))
    _expect_failure(test_single_subsequence_is_ordinary_greedy_decoding, "llama")
    monkeypatch.undo()
    # (g) the argmax keeps the last of several equal maxima instead of the first
    from oracle import primitives as prim
    monkeypatch.setattr(prim, "argmax_lowest", lambda v: int(len(v) - 1 - np.argmax(np.asarray(v)[::-1])))
    _expect_failure(test_argmax_takes_the_lowest_index_among_equal_maxima)
    _expect_failure(test_tied_logits_select_the_lowest_index_through_a_whole_run)
    monkeypatch.undo()
    # (f) controller opens subsequences one iteration late
    orig = controller.pipelined_decode
    monkeypatch.setattr(controller, "pipelined_decode",
                        lambda decoder, delta_t, *a, **k: orig(decoder, delta_t + 1, *a, **k))
    _expect_failure(test_fig2_schedule_with_scripted_decoder)
