"""Pins for the encoder-decoder form of the oracle (oracle/encdec.py; Eq. 1, Eq. 3, Section 4.3):
the bucket function against its definition, the model against an independent dense encoder-decoder
written with PyTorch library ops, the per-query loop against the matrix-masked form.  CPU only."""

import numpy as np
import pytest

import pd_inputs as pi
from oracle import controller, encdec
from torch_encdec import bucket_table, encode as torch_encode, decode_logits

CFG = pi.EncDecConfig(name="encdec-tiny", seed=51, n_enc_layer=2, n_dec_layer=2, d_model=32, n_head=4,
                      head_dim=6, d_ff=48, vocab=83, rel_buckets=8, rel_max_distance=20, ctx_len=23,
                      n_sub=4, delta_t=2, sub_tokens=5)


def setup(cfg):
    w = pi.make_encdec_weights(cfg)
    g = np.random.Generator(np.random.Philox(key=[(cfg.seed << 32) | 0xC0DE, 1]))
    ctx = g.integers(0, cfg.vocab, size=cfg.ctx_len)
    return encdec.EncDecModel(cfg, w), w, ctx


def run(cfg, decoder):
    return controller.pipelined_decode(decoder, cfg.delta_t, 10 ** 6, cfg.n_sub, cfg.bos_id, cfg.eos_id,
                                       cfg.sub_tokens)


# --------------------------------------------------------------------------
# relative-position buckets
# --------------------------------------------------------------------------

def test_bucket_values_follow_the_definition():
    b = lambda n: int(encdec.bucket_behind(np.array([n]), 32, 128)[0])
    # below max_exact = 16 every distance has its own bucket
    assert [b(n) for n in range(16)] == list(range(16))
    # beyond: 16 + floor(log(n / 16) / log(128 / 16) * 16), worked by hand
    assert (b(16), b(17), b(19), b(32), b(64), b(127)) == (16, 16, 17, 21, 26, 31)
    assert b(128) == 31 and b(1000) == 31                      # the last bucket takes everything beyond
    for buckets, far in ((32, 128), (8, 20), (16, 64)):
        n = np.arange(0, 4 * far)
        got = encdec.bucket_behind(n, buckets, far)
        assert np.all(np.diff(got) >= 0) and got.min() == 0 and got.max() == buckets - 1
        assert np.array_equal(got, bucket_table(buckets, far, 4 * far - 1)), "boundaries in closed form"


def test_bidirectional_buckets_mirror_the_sign():
    rel = np.arange(-300, 301)
    got = encdec.bucket_bidirectional(rel, 32, 128)
    behind = encdec.bucket_behind(np.abs(rel), 16, 128)
    assert np.array_equal(got[rel <= 0], behind[rel <= 0])
    assert np.array_equal(got[rel > 0], 16 + behind[rel > 0])
    assert got.max() == 31


# --------------------------------------------------------------------------
# the model against the independent dense encoder-decoder
# --------------------------------------------------------------------------

def test_encoder_states_match_the_dense_model():
    model, w, ctx = setup(CFG)
    np.testing.assert_allclose(model.encode(ctx), torch_encode(CFG, w, ctx).numpy(), rtol=0, atol=1e-10)


def test_single_subsequence_is_ordinary_encoder_decoder_greedy_decoding():
    """S = 1: the Manhattan distance is the ordinary distance between positions and the dependency
    rule is the causal one, so the run must equal textbook greedy decoding of the dense model."""
    cfg = CFG.scaled(n_sub=1, sub_tokens=9)
    model, w, ctx = setup(cfg)
    dec = encdec.EncDecPerQueryDecoder(model, ctx)
    result, steps, _ = run(cfg, dec)
    HE = torch_encode(cfg, w, ctx)
    seq = [cfg.bos_id]
    for j in range(cfg.sub_tokens):
        n = len(seq)
        pos = np.arange(n)
        lg = decode_logits(cfg, w, HE, seq, pos[None, :] <= pos[:, None], pos[:, None] - pos[None, :])[-1]
        np.testing.assert_allclose(dec.trace[j]["logits"][0], lg, rtol=0, atol=1e-10)
        seq.append(int(np.argmax(lg)))
    assert result == [seq[1:]] and steps == cfg.sub_tokens


@pytest.mark.parametrize("S,dt,M", [(4, 2, 5), (5, 1, 4), (3, 3, 7)])
def test_any_schedule_equals_one_dense_forward_under_the_enumerated_rule(S, dt, M):
    """The whole run rebuilt as ONE dense forward over every fed token: mask enumerated from the
    dependency rule of Section 3.2, distances |t1 - t2| + |i1 - i2| enumerated from Section 4.3."""
    cfg = CFG.scaled(n_sub=S, delta_t=dt, sub_tokens=M)
    model, w, ctx = setup(cfg)
    dec = encdec.EncDecPerQueryDecoder(model, ctx)
    result, steps, emitted = run(cfg, dec)
    fed = [(i, rec["t"]) for rec in dec.trace for i in rec["rows"]]
    tokens = []
    for i, t in fed:
        j = t - ((i - 1) * dt + 1)                       # index inside subsequence i (0 = <bos>)
        tokens.append(cfg.bos_id if j == 0 else result[i - 1][j - 1])
    n = len(fed)
    mask = np.zeros((n, n), dtype=bool)
    dist = np.zeros((n, n), dtype=np.int64)
    for a, (iq, tq) in enumerate(fed):
        for b, (ik, tk) in enumerate(fed):
            mask[a, b] = ik <= iq and tk <= tq
            dist[a, b] = abs(tq - tk) + abs(iq - ik)
    want = decode_logits(cfg, w, torch_encode(cfg, w, ctx), tokens, mask, dist)
    row = 0
    for rec in dec.trace:
        for r in range(len(rec["rows"])):
            np.testing.assert_allclose(rec["logits"][r], want[row], rtol=0, atol=1e-10)
            row += 1
    assert row == n == S * (M + 1) - 1


def test_per_query_loop_equals_matrix_masked_form():
    model, w, ctx = setup(CFG)
    f1 = encdec.EncDecPerQueryDecoder(model, ctx)
    f2 = encdec.EncDecMatrixDecoder(model, ctx, CFG.delta_t)
    r1, s1, _ = run(CFG, f1)
    r2, s2, _ = run(CFG, f2)
    assert r1 == r2 and s1 == s2 == CFG.time_steps
    for a, b in zip(f1.trace, f2.trace):
        for r, i in enumerate(a["rows"]):
            if i in b["logits"]:
                np.testing.assert_allclose(a["logits"][r], b["logits"][i], rtol=0, atol=1e-9)


def test_lower_subsequences_do_not_depend_on_higher_ones():
    model, w, ctx = setup(CFG)
    big = encdec.EncDecPerQueryDecoder(model, ctx)
    r4, _, _ = run(CFG, big)
    small = encdec.EncDecPerQueryDecoder(model, ctx)
    r2, _, _ = run(CFG.scaled(n_sub=2), small)
    assert r4[:2] == r2
    for a, b in zip(big.trace, small.trace):
        for r, i in enumerate(b["rows"]):
            np.testing.assert_allclose(a["logits"][a["rows"].index(i)], b["logits"][r], rtol=0, atol=1e-12)


def test_planted_mistakes_are_caught(monkeypatch):
    def expect_failure(test, *args):
        with pytest.raises(AssertionError):
            test(*args)
    # distance without the subsequence term
    monkeypatch.setattr(encdec, "manhattan", lambda i_q, t_q, i_k, t_k: abs(t_q - t_k))
    expect_failure(test_any_schedule_equals_one_dense_forward_under_the_enumerated_rule, 4, 2, 5)
    monkeypatch.undo()
    # a 1/sqrt(head_dim) factor on the scores, which this backbone does not have
    monkeypatch.setattr(encdec.EncDecModel, "heads",
                        lambda self, y: y.reshape(y.shape[0], self.c.n_head, self.c.head_dim) / self.c.head_dim ** 0.25)
    expect_failure(test_single_subsequence_is_ordinary_encoder_decoder_greedy_decoding)
    monkeypatch.undo()
    # buckets off by one beyond max_exact
    orig = encdec.bucket_behind
    monkeypatch.setattr(encdec, "bucket_behind",
                        lambda n, buckets, far: np.minimum(orig(n, buckets, far) + (np.asarray(n) >= buckets // 2),
                                                           buckets - 1))
    expect_failure(test_bucket_values_follow_the_definition)
    expect_failure(test_single_subsequence_is_ordinary_encoder_decoder_greedy_decoding)
    monkeypatch.undo()
    # encoder buckets that drop the sign (keys ahead of the query treated like keys behind it)
    orig_bi = encdec.bucket_bidirectional
    monkeypatch.setattr(encdec, "bucket_bidirectional",
                        lambda rel, buckets, far: orig_bi(-np.abs(rel), buckets, far))
    expect_failure(test_encoder_states_match_the_dense_model)
