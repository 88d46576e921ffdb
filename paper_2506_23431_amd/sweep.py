#!/usr/bin/env python3
"""Sequential decoding versus pipelined decoding on the same kernels, and sweeps over the number of
subsequences S and the delay dt.

  python -m paper_2506_23431_amd.sweep [--workload cfg4] [--s-list 1,4,8,16,32] [--dt-list 1,2,4,8,16]

The paper's headline result is the speed-up of the pipelined decoder over a sequential decoder
that generates the same number of tokens one at a time (Section 5.3, Fig. 4, Tables 2-5).  Its
datasets and fine-tuned weights are not used here; the synthetic analogue keeps what the speed-up
depends on: the total number of generated tokens N = S*M of the workload is fixed, and

  * S = 1, M = N is ordinary sequential greedy decoding (one row per step, N steps),
  * S > 1 splits the same N tokens into S subsequences of N/S tokens started dt steps apart
    ((S-1)*dt + N/S steps).

Every configuration runs on the same library, weights and context; each line reports steps,
milliseconds per step, generated tokens per second and the speed-up over S = 1.  The step ratio
N / ((S-1)*dt + N/S) is the speed-up a decoder whose step cost did not depend on the number of rows
would show (the paper's observation that a step with several tokens costs no more than a step
with one).
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def run_config(dec, ctx, S, dt, M, repeats=2):
    """Times the decode steps of one (S, dt, M) schedule on contexts already known to `dec`.
    Returns (steps, seconds)."""
    import torch
    T = (S - 1) * dt + M
    dec.prefill_context(ctx, S, dt, M, T)
    best = None
    for _ in range(repeats):
        dec.reset_decode()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        dec.decode_steps(T)
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        best = el if best is None else min(best, el)
    return T, best


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="cfg4")
    ap.add_argument("--s-list", default="1,2,4,8,16,32")
    ap.add_argument("--dt-list", default="1,2,4,8,16")
    ap.add_argument("--tokens", type=int, default=0, help="total generated tokens N (default: S*M of the workload)")
    ap.add_argument("--layers", type=int, default=0, help="use only this many layers (quick runs)")
    ap.add_argument("--kv-pair-layers", type=int, default=0,
                    help="leading layers whose cache keeps keys and values as pairs of halves")
    args = ap.parse_args(argv)

    import torch
    import pd_inputs as pi
    from pd_inputs import max_positions
    from paper_2506_23431_amd import PipelinedDecoder

    base = pi.get_config(args.workload)
    if args.layers:
        base = base.scaled(n_layer=args.layers)
    N = args.tokens or base.n_sub * base.sub_tokens
    s_list = [int(x) for x in args.s_list.split(",")]
    dt_list = [int(x) for x in args.dt_list.split(",")]
    plans = []
    for S in s_list:
        if N % S:
            continue
        M = N // S
        for dt in ([1] if S == 1 else dt_list):
            A = min(S, M // dt + 1)
            if base.dtype == 1 and base.batch * A > 128:
                continue                # more rows than one matrix-core step supports
            plans.append(base.scaled(n_sub=S, delta_t=dt, sub_tokens=M))
    # one set of weights whose position table covers the longest run of the sweep
    mp = max(max_positions(c) for c in plans)
    weights = pi.make_weights(base.scaled(n_sub=1, delta_t=1, sub_tokens=mp - base.ctx_len - 1))
    ctx = pi.make_context(base)
    rows = []
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for cfg in plans:
            S, dt, M = cfg.n_sub, cfg.delta_t, cfg.sub_tokens
            dec = PipelinedDecoder(cfg, weights, max_batch=cfg.batch, max_ctx=cfg.ctx_len, max_sub=S,
                                   max_sub_tokens=M, max_pos=mp, kv_pair_layers=args.kv_pair_layers)
            T, sec = run_config(dec, ctx, S, dt, M)
            dec.close()
            rows.append({"S": S, "dt": dt, "M": M, "steps": T, "rows_per_request": min(S, M // dt + 1),
                         "ms_per_step": sec / T * 1e3, "tokens_per_s": base.batch * N / sec,
                         "step_ratio": N / T})
            print(f"S={S:3d} dt={dt:3d} M={M:5d}: {T:5d} steps, {sec / T * 1e3:7.3f} ms/step, "
                  f"{base.batch * N / sec:9.1f} tokens/s", flush=True)
    seq_rate = next((r["tokens_per_s"] for r in rows if r["S"] == 1), None)
    for r in rows:
        r["speedup_vs_sequential"] = r["tokens_per_s"] / seq_rate if seq_rate else None
    print(json.dumps({"workload": base.name, "n_layer": base.n_layer, "tokens": N, "batch": base.batch,
                      "context": base.ctx_len, "results": rows}))
    return rows


if __name__ == "__main__":
    main()
