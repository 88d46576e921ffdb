#!/usr/bin/env python3
"""Writes the stored full-run oracle results of the named workloads (CPU only).

  python tests/golden/make_full_run.py cfg4                 # every request of the workload
  python tests/golden/make_full_run.py cfg5 --requests 0    # one request (hours of CPU work each)

For every chosen request the CPU oracle (oracle/, fp64) runs Algorithm 1 free-running over the
whole workload: the causal pass over the context, then every decode iteration until all
subsequences have their M tokens.  Nothing else is called: the inputs come from the seeded
generators of pd_inputs/, no value comes from the HIP library.  Per logit row (one per fed token:
iteration t, subsequence i) the file tests/golden/full_run_<workload>_req<b>.npz keeps

  step, sub       iteration t and subsequence i (1-based) of the row
  token           the token the oracle appended from this row (its argmax, lowest index on ties,
                  Eq. 4), or -1 for a row that only feeds a finished subsequence's last token
  top_idx/top_val the 8 largest logits and their vocabulary indices, best first
  margin          top_val[0] - top_val[1]
  sample          the logits at the fixed columns `cols` (256 columns drawn once per workload
                  from a counter-based generator keyed by the workload's seed), as fp32

The GPU test teacher-forces the library over the whole run with `token`, compares its logits
at `cols` and `top_idx` with the stored values, and requires its own argmax to equal `token`
wherever `margin` exceeds 0.05.
"""

import argparse
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import pd_inputs as pi                      # noqa: E402
from oracle import controller, pipelined    # noqa: E402
from oracle.model import OracleModel        # noqa: E402

N_COLS, N_TOP = 256, 8


def sample_columns(cfg):
    g = np.random.Generator(np.random.Philox(key=[(cfg.seed << 32) | 0x60DE, 7]))
    return np.sort(g.choice(cfg.vocab, size=min(N_COLS, cfg.vocab), replace=False)).astype(np.int32)


def path_for(name, b):
    return os.path.join(HERE, f"full_run_{name}_req{b}.npz")


def run_request(cfg, weights, ctx, b, log):
    # fp64 copies of every layer are kept when they fit comfortably (8 bytes per parameter)
    n_param = cfg.n_layer * (4 * cfg.d_model ** 2 + (3 if cfg.ffn_kind == 1 else 2) * cfg.d_model * cfg.d_ff)
    model = OracleModel(cfg, weights, cache_layers=n_param * 8 < 16e9)
    cols = sample_columns(cfg)
    t0 = time.time()
    last = [t0]

    def tick(msg, every=30.0):
        if time.time() - last[0] > every:
            log(f"[{cfg.name} req {b}] {msg} ({time.time() - t0:.0f} s)")
            last[0] = time.time()

    kv = model.prefill(ctx[b], progress=lambda l: tick(f"context pass, layer {l + 1}/{cfg.n_layer}"))
    log(f"[{cfg.name} req {b}] context pass done ({time.time() - t0:.0f} s)")
    dec = pipelined.PerQueryDecoder(model, ctx[b], keep=True, context_kv=kv)
    rows = {k: [] for k in ("step", "sub", "top_idx", "top_val", "sample")}

    def stepper(G, t):
        out = dec(G, t)
        rec = dec.trace[-1]
        for r, i in enumerate(rec["rows"]):
            lg = rec["logits"][r]
            top = np.argsort(-lg, kind="stable")[:N_TOP]       # equal values: lowest index first
            rows["step"].append(t)
            rows["sub"].append(i)
            rows["top_idx"].append(top.astype(np.int32))
            rows["top_val"].append(lg[top].astype(np.float64))
            rows["sample"].append(lg[cols].astype(np.float32))
        rec.pop("logits", None)                                 # the full rows are not kept
        rec.pop("vis", None)
        tick(f"iteration {t}/{cfg.time_steps}")
        return out

    result, steps, emitted = controller.pipelined_decode(
        stepper, cfg.delta_t, cfg.time_steps, cfg.n_sub, cfg.bos_id, cfg.eos_id, cfg.sub_tokens)
    token = np.array([emitted[t - 1].get(i, -1) for t, i in zip(rows["step"], rows["sub"])], dtype=np.int32)
    top_idx = np.stack(rows["top_idx"])
    top_val = np.stack(rows["top_val"])
    produced = token >= 0
    assert np.array_equal(top_idx[produced, 0], token[produced]), "appended token is not the argmax"
    assert sum(len(r) for r in result) == int(produced.sum())
    np.savez_compressed(
        path_for(cfg.name, b), workload=cfg.name, request=b, steps=steps, cols=cols,
        step=np.array(rows["step"], dtype=np.int32), sub=np.array(rows["sub"], dtype=np.int32),
        token=token, top_idx=top_idx, top_val=top_val, margin=top_val[:, 0] - top_val[:, 1],
        sample=np.stack(rows["sample"]))
    log(f"[{cfg.name} req {b}] {steps} iterations, {len(token)} rows, {int(produced.sum())} tokens, "
        f"{int((top_val[:, 0] - top_val[:, 1] > 0.05)[produced].sum())} with a margin above 0.05; "
        f"wrote {path_for(cfg.name, b)} ({time.time() - t0:.0f} s)")


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("workload")
    ap.add_argument("--requests", default=None, help="comma-separated request indices (default: all)")
    args = ap.parse_args(argv)
    cfg = pi.get_config(args.workload)
    reqs = list(range(cfg.batch)) if args.requests is None else [int(x) for x in args.requests.split(",")]

    def log(msg):
        print(msg, flush=True)

    weights = pi.make_weights(cfg)
    ctx = pi.make_context(cfg)
    log(f"[{cfg.name}] weights drawn; requests {reqs}")
    for b in reqs:
        run_request(cfg, weights, ctx, b, log)


if __name__ == "__main__":
    main()
