#!/usr/bin/env python3
"""Benchmark of the pipelined decode step on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4]

A "step" is one time-step of Algorithm 1: every open subsequence of every request
feeds its newest token through all layers (norm, QKV, KV append, masked multi-query
attention, output projection, FFN) and the fused vocabulary projection + argmax,
and the schedule advances.  The workload is synthetic (seeded weights N(0, 0.02),
uniform context ids), already resident in HBM when the timed region starts; the
context pass (prefill) is outside the metric and reported separately.

Prints ONE JSON line: generated tokens/s over exactly K steps, plus
  roofline      achieved HBM GB/s of the attention kernel (algorithmic bytes per launch /
                average launch duration from HIP events attached to its dispatches) vs 8 TB/s,
                beside what a kernel that only reads the same bytes reaches
  cpu_baseline  the CPU oracle timed on the host cores on a bounded sample
"""

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def producing(cfg, t):
    """Subsequences that select a token in iteration t (EOS disabled): (i-1)dt < t <= (i-1)dt + M."""
    return sum(1 for i in range(cfg.n_sub) if i * cfg.delta_t < t <= i * cfg.delta_t + cfg.sub_tokens)


def fed(cfg, t):
    """Rows per request in iteration t: producing rows plus rows that feed a finished
    subsequence's last token once."""
    return sum(1 for i in range(cfg.n_sub) if i * cfg.delta_t < t <= i * cfg.delta_t + cfg.sub_tokens + 1)


def attention_bytes(cfg, steps):
    """Algorithmic HBM bytes of one attention launch, averaged over iterations 1..steps:
    every visible key and value once (bf16), shared by the rows of a request, plus Q in and O out."""
    H, hd, B = cfg.n_head, cfg.head_dim, cfg.batch
    total, n_gen = 0.0, 0
    for t in range(1, steps + 1):
        rows = fed(cfg, t)
        n_gen += rows
        kv = B * H * (cfg.ctx_len + n_gen) * hd * 2 * 2
        qo = B * rows * cfg.d_model * 2 * 2 * 2      # q and o, each as a bf16 pair
        total += kv + qo
    return total / steps


def cpu_baseline(cfg, weights, ctx, budget_s=20.0):
    """The oracle as it stands, on the host cores: decode iterations from t = 1 of request 0 until
    the time budget is used.  The context keys/values are seeded random numbers instead of the causal
    pass over the context (which is outside the metric)."""
    import numpy as np
    from oracle.model import OracleModel
    from oracle import pipelined
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    model = OracleModel(cfg, weights)
    for l in range(cfg.n_layer):          # convert the weights before the clock starts
        model.layer(l)
    model._lm()
    rng = np.random.default_rng(cfg.seed)
    shape = (cfg.n_head, cfg.ctx_len, cfg.head_dim)
    kv = ([rng.standard_normal(shape) * 0.3 for _ in range(cfg.n_layer)],
          [rng.standard_normal(shape) * 0.3 for _ in range(cfg.n_layer)])
    dec = pipelined.PerQueryDecoder(model, ctx[0], keep=False, context_kv=kv)
    G, tokens, t = [], 0, 0
    t0 = time.time()
    while time.time() - t0 < budget_s and t < cfg.time_steps:
        t += 1
        if (t - 1) % cfg.delta_t == 0 and len(G) < cfg.n_sub:
            G.append([cfg.bos_id])
        new = dec(G, t)
        for i, g in enumerate(G):
            if len(g) - 1 < cfg.sub_tokens:
                g.append(new[i])
                tokens += 1
    dt = time.time() - t0
    return {"value": tokens / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {t} decode iterations of request 0 of {cfg.name} ({tokens} tokens, "
                      f"{dt:.1f} s), fp64 numpy; context K/V are seeded random values, the context "
                      f"pass is not timed"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="decode iterations to time (default: the full run)")
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="cfg4")
    ap.add_argument("--graph", type=int, default=0, help="replay each step from a captured HIP graph")
    ap.add_argument("--attn-splits", type=int, default=0)
    ap.add_argument("--kv-pair-layers", type=int, default=None,
                    help="leading layers whose cache keeps keys and values as pairs of halves (cfg5 needs 1 "
                         "to stay inside the logit tolerance and gets it by default; cfg1-cfg4 do not)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sync-every", type=int, default=0,
                    help="synchronise after every N iterations of the timed pass (0: never; a counter-collecting "
                         "profiler cannot queue tens of thousands of launches)")
    ap.add_argument("--no-event-passes", action="store_true",
                    help="skip the passes that time the attention kernel with HIP events and the plain-read "
                         "measurement (for runs under a counter-collecting profiler)")
    ap.add_argument("--calibrate-copy-mb", type=int, default=0,
                    help="also run plain device-to-device copies of this many MiB (a kernel of known "
                         "traffic, to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.kv_pair_layers is None:
        args.kv_pair_layers = 1 if args.workload.startswith("cfg5") else 0
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}): no collectives, no "
              "sharding; requests, context keys and heads are the axes it would shard along", file=sys.stderr)
        sys.exit(2)

    import torch
    import pd_inputs as pi
    from pd_inputs import max_positions
    from paper_2506_23431_amd import PipelinedDecoder, binding

    cfg = pi.get_config(args.workload)
    K = args.steps if args.steps is not None else cfg.time_steps
    K = max(1, min(K, cfg.time_steps))
    W = max(0, min(args.warmup, cfg.time_steps))
    weights = pi.make_weights(cfg)
    ctx = pi.make_context(cfg)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        dec = PipelinedDecoder(cfg, weights, max_batch=cfg.batch, max_ctx=cfg.ctx_len, max_sub=cfg.n_sub,
                               max_sub_tokens=cfg.sub_tokens, max_pos=max_positions(cfg),
                               kv_pair_layers=args.kv_pair_layers)
        dec.set_option(binding.PD_OPT_USE_GRAPH, args.graph)
        dec.set_option(binding.PD_OPT_ATTN_SPLITS, args.attn_splits)
        if args.calibrate_copy_mb > 0:
            src = torch.ones(args.calibrate_copy_mb << 20, dtype=torch.uint8, device="cuda")
            dst = torch.empty_like(src)
            for _ in range(3):
                dst.copy_(src)
            del src, dst
        torch.cuda.synchronize()
        t0 = time.time()
        dec.prefill_context(ctx, cfg.n_sub, cfg.delta_t, cfg.sub_tokens, cfg.time_steps)
        torch.cuda.synchronize()
        prefill_s = time.time() - t0
        # warm-up: W untimed iterations, then back to t = 0
        dec.decode_steps(W)
        dec.reset_decode()
        torch.cuda.synchronize()
        # timed region: exactly K iterations
        t0 = time.perf_counter()
        if args.sync_every > 0:
            for k0 in range(0, K, args.sync_every):
                dec.decode_steps(min(args.sync_every, K - k0))
                torch.cuda.synchronize()
        else:
            dec.decode_steps(K)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        attn_us, attn_launches, pair_us, read_gbs = 0.0, 0, 0.0, 0.0
        if not args.no_event_passes:
            # second pass over the same K iterations with HIP events around every launch of the attention
            # kernel (the one that streams the keys and values); third pass: around the kernel and the
            # small kernel that merges its partial results
            dec.set_option(binding.PD_OPT_USE_GRAPH, 0)
            dec.set_option(binding.PD_OPT_PROFILE, 1)
            dec.reset_decode()
            dec.decode_steps(K)
            torch.cuda.synchronize()
            attn_us, attn_launches = dec.profile_read()
            dec.set_option(binding.PD_OPT_PROFILE, 2)
            dec.reset_decode()
            dec.decode_steps(K)
            torch.cuda.synchronize()
            pair_us, _ = dec.profile_read()
            dec.set_option(binding.PD_OPT_PROFILE, 0)
            # what a kernel that only reads reaches on this device, at the size of one attention launch
            buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
            buf.fill_(1)
            torch.cuda.synchronize()
            chunk = int(attention_bytes(cfg, K)) // 4096 * 4096
            read_gbs = binding.measure_read_bandwidth(buf.data_ptr(), buf.numel(), chunk, 200,
                                                      torch.cuda.current_stream().cuda_stream)
            del buf

        dec.close()

    tokens = cfg.batch * sum(producing(cfg, t) for t in range(1, K + 1))
    # a pair layer reads every key and value twice (high and low halves)
    abytes = attention_bytes(cfg, K) * (1.0 + args.kv_pair_layers / cfg.n_layer)
    achieved = abytes / (attn_us * 1e-6) / 1e9 if attn_us > 0 else 0.0
    # HBM bytes per launch from the rocprofv3 counter runs summarised under profiles/ (null if none)
    traffic = None
    pmc = os.path.join(ROOT, "profiles", f"attention_{cfg.name}_hbm_traffic.md")
    if os.path.exists(pmc):
        m = re.search(r"bytes_per_launch\s*=\s*(\d+)", open(pmc).read())
        traffic = float(m.group(1)) if m else None
    out = {
        "metric": "pipelined_decode_generated_tokens_per_s", "value": tokens / elapsed, "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": elapsed / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.n_layer} layers, d_model {cfg.d_model}, "
                               f"{cfg.n_head}x{cfg.head_dim} heads, FFN {cfg.d_ff}, vocab {cfg.vocab}, "
                               f"batch {cfg.batch}, context {cfg.ctx_len}, S={cfg.n_sub}, dt={cfg.delta_t}, "
                               f"M={cfg.sub_tokens}",
                   "tokens_generated": tokens, "time_steps_full_run": cfg.time_steps,
                   "prefill_s": prefill_s, "hip_graph": bool(args.graph),
                   "kv_pair_layers": args.kv_pair_layers},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "kernel": "k_attn_mfma (masked multi-query attention over the KV cache, one launch "
                               "per layer per step)",
                     "algorithmic_bytes_per_launch": abytes, "avg_launch_us": attn_us,
                     "launches": attn_launches,
                     "timing": "HIP start and stop events attached to every dispatch of the kernel on the "
                               "launch stream, in a second pass over the same K iterations",
                     "with_merge_kernel_us": pair_us,
                     "plain_read_same_bytes": {"GB/s": read_gbs, "frac_of_peak": read_gbs / HBM_PEAK_GBS,
                                               "note": "a kernel that only reads this many bytes, launched "
                                                       "back to back on the same device"}},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, weights, ctx)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
