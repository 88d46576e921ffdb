"""CPU-only checks of the C-ABI library: it loads, exports every function include/pd.h declares,
sizes workspaces and rejects bad arguments with error codes (no GPU call is reached)."""

import ctypes as C
import os
import re

import numpy as np
import pytest

import pd_inputs as pi
from pd_inputs import max_positions

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2506_23431_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2506_23431_amd.build import build
        build(verbose=False)
    return binding.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "pd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pd_[a-z_]+)\s*\(", text)))


def config_struct(cfg, **kw):
    from paper_2506_23431_amd.binding import PdConfig
    f = dict(n_layer=cfg.n_layer, d_model=cfg.d_model, n_head=cfg.n_head, head_dim=cfg.head_dim,
             d_ff=cfg.d_ff, vocab=cfg.vocab, ffn_kind=cfg.ffn_kind, norm_kind=cfg.norm_kind,
             pos_kind=cfg.pos_kind, rope_base=cfg.rope_base, norm_eps=cfg.norm_eps, dtype=cfg.dtype,
             bos_id=cfg.bos_id, eos_id=cfg.eos_id, max_batch=cfg.batch, max_ctx=cfg.ctx_len,
             max_sub=cfg.n_sub, max_sub_tokens=cfg.sub_tokens, max_pos=max_positions(cfg))
    f.update(kw)
    return PdConfig(**f)


def test_every_declared_function_is_exported(lib):
    names = declared_functions()
    assert {"pd_prefill_context", "pd_decode_step", "pd_generate"} <= set(names)
    for n in names:
        assert getattr(lib, n) is not None, n
    from paper_2506_23431_amd import binding
    assert sorted(binding.EXPORTS) == names


def test_workspace_sizes(lib):
    sizes = {}
    for name in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5"):
        cfg = pi.get_config(name)
        n = lib.pd_workspace_bytes(C.byref(config_struct(cfg)))
        assert n > 0 and n % 256 == 0
        sizes[name] = n
        # at least the two KV caches of every layer
        kv = 2 * cfg.n_layer * cfg.batch * cfg.d_model * (cfg.ctx_len + cfg.n_sub * (cfg.sub_tokens + 1)) \
            * (4 if cfg.dtype == 0 else 2)
        assert n >= kv
    assert sizes["cfg1"] < sizes["cfg2"] < sizes["cfg4"] < sizes["cfg5"] < 64 << 30
    # a pair layer adds exactly one more key cache and one more value cache of that layer
    cfg = pi.get_config("cfg5")
    kv_cap = (cfg.ctx_len + cfg.n_sub * (cfg.sub_tokens + 1) + 63) // 64 * 64
    one = 2 * cfg.batch * cfg.d_model * kv_cap * 2
    for n in (1, 3):
        grown = lib.pd_workspace_bytes(C.byref(config_struct(cfg, kv_pair_layers=n)))
        assert grown - sizes["cfg5"] == n * one
    # fp32 caches have no low halves
    cfg = pi.get_config("cfg1")
    assert lib.pd_workspace_bytes(C.byref(config_struct(cfg, kv_pair_layers=1))) == sizes["cfg1"]
    # kv_pair_layers = -1: the library chooses from the shape alone (one pair layer from width 4096
    # on, none below), whatever the workload is called
    seven_b = pi.get_config("cfg5").scaled(name="some-7b-shaped-model")
    assert lib.pd_workspace_bytes(C.byref(config_struct(seven_b, kv_pair_layers=-1))) == sizes["cfg5"] + one
    for name in ("cfg2", "cfg3", "cfg4"):
        assert lib.pd_workspace_bytes(C.byref(config_struct(pi.get_config(name), kv_pair_layers=-1))) == sizes[name]


@pytest.mark.parametrize("bad", [dict(n_head=3), dict(head_dim=7, n_head=1, d_model=7), dict(dtype=2),
                                 dict(ffn_kind=5), dict(max_batch=0), dict(bos_id=-1), dict(norm_eps=0.0),
                                 dict(eos_id=10 ** 6), dict(max_sub=70000, max_sub_tokens=1), dict(kv_pair_layers=-2), dict(kv_pair_layers=99)])
def test_invalid_configurations_are_rejected(lib, bad):
    cfg = pi.get_config("cfg1")
    assert lib.pd_workspace_bytes(C.byref(config_struct(cfg, **bad))) == 0
    assert len(lib.pd_last_error()) > 0


def test_create_rejects_bad_arguments_without_touching_the_gpu(lib):
    from paper_2506_23431_amd.binding import PdWeights
    cfg = config_struct(pi.get_config("cfg1"))
    out = C.c_void_p()
    w = PdWeights()
    assert lib.pd_create(C.byref(cfg), None, None, 0, None, C.byref(out)) == -1          # PD_EINVAL
    assert lib.pd_create(C.byref(cfg), C.byref(w), 256, 16, None, C.byref(out)) == -3     # PD_ENOMEM
    assert b"workspace too small" in lib.pd_last_error()
    need = lib.pd_workspace_bytes(C.byref(cfg))
    assert lib.pd_create(C.byref(cfg), C.byref(w), 257, need, None, C.byref(out)) == -1   # unaligned
    assert lib.pd_create(C.byref(cfg), C.byref(w), 256, need, None, C.byref(out)) == -1   # NULL weights
    assert b"weight pointer is NULL" in lib.pd_last_error()
    assert lib.pd_destroy(None) == 0
    assert lib.pd_set_option(None, 1, 0) == -1
    assert lib.pd_decode_steps(None, 1, None) == -1


def encdec_struct(cfg, **over):
    from paper_2506_23431_amd.binding import PdEncDecConfig
    f = dict(n_enc_layer=cfg.n_enc_layer, n_dec_layer=cfg.n_dec_layer, d_model=cfg.d_model, n_head=cfg.n_head,
             head_dim=cfg.head_dim, d_ff=cfg.d_ff, vocab=cfg.vocab, rel_buckets=cfg.rel_buckets,
             rel_max_distance=cfg.rel_max_distance, norm_eps=cfg.norm_eps, bos_id=cfg.bos_id, eos_id=cfg.eos_id,
             max_batch=cfg.batch, max_ctx=cfg.ctx_len, max_sub=cfg.n_sub, max_sub_tokens=cfg.sub_tokens)
    f.update(over)
    return PdEncDecConfig(**f)


def test_encoder_decoder_configurations(lib):
    """Workspace sizes of the backbone-shaped encoder-decoder workloads (they hold the re-packed weights of
    both stacks and two caches per decoder layer), and what the form does not take."""
    from paper_2506_23431_amd.binding import PdEncDecWeights
    for name, cfg in pi.ENCDEC_CONFIGS.items():
        n = lib.pd_encdec_workspace_bytes(C.byref(encdec_struct(cfg)))
        d, ff, V = cfg.d_model, cfg.d_ff, cfg.vocab
        packed = 2 * (cfg.n_enc_layer * (4 * d * d + 2 * d * ff) + cfg.n_dec_layer * (8 * d * d + 2 * d * ff) + V * d)
        assert packed < n < packed + (256 << 20), (name, n, packed)
    cfg = pi.ENCDEC_CONFIGS["encdec-small"]
    for bad in (dict(head_dim=48, n_head=16, d_model=768), dict(rel_max_distance=129), dict(rel_buckets=30),
                dict(rel_max_distance=16), dict(max_ctx=4097), dict(n_head=32, head_dim=16), dict(n_enc_layer=0),
                dict(d_ff=2000), dict(bos_id=cfg.vocab), dict(norm_eps=0.0)):
        assert lib.pd_encdec_workspace_bytes(C.byref(encdec_struct(cfg, **bad))) == 0, bad
        assert len(lib.pd_last_error()) > 0
    out = C.c_void_p()
    c, w = encdec_struct(cfg), PdEncDecWeights()
    need = lib.pd_encdec_workspace_bytes(C.byref(c))
    assert lib.pd_encdec_create(C.byref(c), None, None, 0, None, C.byref(out)) == -1
    assert lib.pd_encdec_create(C.byref(c), C.byref(w), 256, 16, None, C.byref(out)) == -3
    assert lib.pd_encdec_create(C.byref(c), C.byref(w), 256, need, None, C.byref(out)) == -1
    assert b"weight pointer is NULL" in lib.pd_last_error()


def test_encdec_device_weights_are_the_rounded_ones():
    """The two views pd_inputs hands out of one set of encoder-decoder weights (bit patterns for the
    library, rounded values for the oracle) describe the same numbers, with the projections stacked in the
    order the header states."""
    cfg = pi.EncDecConfig(name="t", seed=3, n_enc_layer=1, n_dec_layer=1, d_model=32, n_head=1, head_dim=32, d_ff=32,
                          vocab=11)
    w = pi.make_encdec_weights(cfg)
    rounded, device = pi.encdec_to_bf16(w)
    dl, rl = device["dec_layers"][0], rounded["dec_layers"][0]
    assert np.array_equal(pi.bits_to_f32(dl["wqkv"]), np.concatenate([rl["wq"], rl["wk"], rl["wv"]]))
    assert np.array_equal(pi.bits_to_f32(dl["ckv"]), np.concatenate([rl["ck"], rl["cv"]]))
    assert np.array_equal(pi.bits_to_f32(device["tok_emb"]), rounded["tok_emb"])
    assert np.array_equal(pi.bits_to_f32(device["enc_layers"][0]["w1"]), rounded["enc_layers"][0]["w1"])
    assert np.abs(rounded["lm_head"] - w["lm_head"]).max() <= np.abs(w["lm_head"]).max() * 2.0 ** -8
    assert rl["norm3_g"] is w["dec_layers"][0]["norm3_g"] and device["dec_rel_bias"].dtype == np.float32


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    from paper_2506_23431_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(binding.PdError, match="no fallback"):
        binding.load()


def test_option_keys_match_the_header():
    """The binding's option constants are the header's."""
    from paper_2506_23431_amd import binding
    text = open(os.path.join(ROOT, "include", "pd.h")).read()
    keys = dict(re.findall(r"#define\s+(PD_OPT_[A-Z_]+)\s+(\d+)", text))
    assert len(keys) >= 5
    for name, value in keys.items():
        assert getattr(binding, name) == int(value), name
    assert len(set(keys.values())) == len(keys), "option keys must be distinct"


def test_ragged_targets_are_reproducible_and_hold_their_plan():
    """Host logic of the ragged sweep: seeded draws, every length at least delta_t, and a plan
    (S, M, T) that holds the longest target plus one exploratory subsequence."""
    from paper_2506_23431_amd import sweep
    for profile, (mean_n, mean_words) in sweep.RAGGED.items():
        a = sweep.draw_ragged(profile, 64, 3, seed=11)
        assert a == sweep.draw_ragged(profile, 64, 3, seed=11)
        assert a != sweep.draw_ragged(profile, 64, 3, seed=12)
        assert all(len(l) >= 1 and min(l) >= 3 for l in a)
        n = np.mean([len(l) for l in a])
        t = np.mean([x for l in a for x in l])
        assert abs(n - mean_n) < 1.0 and abs(t - mean_words * sweep.TOKENS_PER_WORD) < 3.0
        S, M, T = sweep.ragged_plan(a, 3)
        assert S == max(len(l) for l in a) + 1 and M == max(max(l) for l in a) + 1
        assert T == (S - 1) * 3 + M
    assert all(len(l) <= 4 for l in sweep.draw_ragged("pubmed", 16, 2, seed=1, s_max=4))
