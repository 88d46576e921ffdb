#!/usr/bin/env python3
"""Benchmark of the pipelined decode step on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4]

A "step" is one time-step of Algorithm 1: every open subsequence of every request
feeds its newest token through all layers (norm, QKV, KV append, masked multi-query
attention, output projection, FFN) and the fused vocabulary projection + argmax,
and the schedule advances.  The workload is synthetic (seeded weights N(0, 0.02),
uniform context ids), already resident in HBM when the timed region starts; the
context pass (prefill) is outside the metric and reported separately.

Prints ONE JSON line: generated tokens/s over exactly K steps (median of several repeats).  With
K below the length of the run, the K steps are a window centred in the run, reached by an untimed
fast-forward from t = 1; the line then also carries `full_run`, the whole run from t = 1 (B*S*M
tokens over its T steps).  Further objects:
  roofline      achieved HBM GB/s of the attention kernel (algorithmic bytes per launch over the
                window / average launch duration from HIP events attached to its dispatches) vs
                8 TB/s, the same with the kernel that merges its partials, the whole step against
                its algorithmic bytes, and what a kernel that only reads the same bytes reaches
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


def attention_bytes(cfg, t0, t1):
    """Algorithmic HBM bytes of one attention launch, averaged over iterations t0..t1 (1-based,
    inclusive): every visible key and value once (16 bit), shared by the rows of a request, plus Q in
    and O out."""
    H, hd, B = cfg.n_head, cfg.head_dim, cfg.batch
    total, n_gen = 0.0, 0
    for t in range(1, t1 + 1):
        rows = fed(cfg, t)
        n_gen += rows
        if t < t0:
            continue
        kv = B * H * (cfg.ctx_len + n_gen) * hd * 2 * 2
        qo = B * rows * cfg.d_model * 2 * 2 * 2      # q and o, each as a 16-bit pair
        total += kv + qo
    return total / (t1 - t0 + 1)


def step_bytes(cfg, t0, t1, pair_layers):
    """Algorithmic HBM bytes of one whole time-step, averaged over iterations t0..t1: every weight
    once (shared by all rows and requests), every request's visible keys and values once per layer."""
    d, ff, V, nl = cfg.d_model, cfg.d_ff, cfg.vocab, cfg.n_layer
    c = 3 if cfg.ffn_kind == 1 else 2
    weights = 2.0 * (nl * (4 * d * d + c * d * ff) + V * d)
    attn = attention_bytes(cfg, t0, t1) * (nl + pair_layers)
    return weights + attn


def window(cfg, K):
    """Iterations t0..t1 that a run of K < T steps times: K consecutive iterations centred in the run,
    where the schedule is in its steady state (every slot of the pipeline holds a subsequence) and the
    generated-side cache is about as long as on average over the run."""
    T = cfg.time_steps
    if K >= T:
        return 1, T
    t0 = (T - K) // 2 + 1
    return t0, t0 + K - 1


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
    ap.add_argument("--steps", type=int, default=None,
                    help="decode iterations to time (default: the full run; fewer: a window centred in the run, "
                         "reached by an untimed fast-forward)")
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--repeats", type=int, default=5, help="timed repeats of the window (the median is reported)")
    ap.add_argument("--workload", default="cfg4")
    ap.add_argument("--graph", type=int, default=0, help="replay each step from a captured HIP graph")
    ap.add_argument("--attn-splits", type=int, default=0)
    ap.add_argument("--prefill-chunk", type=int, default=0, help="rows of the context pass per launch (0: the library's default)")
    ap.add_argument("--kv-pair-layers", type=int, default=-1,
                    help="leading layers whose cache keeps keys and values as pairs of halves (-1: the library "
                         "chooses from the shape)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sync-every", type=int, default=0,
                    help="synchronise after every N iterations of the timed pass (0: never; for runs under a "
                         "counter-collecting profiler)")
    ap.add_argument("--no-event-passes", action="store_true",
                    help="skip the passes that time the attention kernel with HIP events, the full-run pass and the "
                         "plain-read measurement (for runs under a profiler)")
    ap.add_argument("--calibrate-copy-mb", type=int, default=0,
                    help="also run plain device-to-device copies of this many MiB (a kernel of known "
                         "traffic, to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (got --gpus {args.gpus}): no collectives, no "
              "sharding; requests, context keys and heads are the axes it would shard along", file=sys.stderr)
        sys.exit(2)

    import statistics
    import torch
    import pd_inputs as pi
    from pd_inputs import max_positions
    from paper_2506_23431_amd import PipelinedDecoder, binding

    cfg = pi.get_config(args.workload)
    T = cfg.time_steps
    K = args.steps if args.steps is not None else T
    K = max(1, min(K, T))
    W = max(0, min(args.warmup, T))
    reps = max(1, args.repeats)
    t0w, t1w = window(cfg, K)
    weights = pi.make_weights(cfg)
    ctx = pi.make_context(cfg)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        dec = PipelinedDecoder(cfg, weights, max_batch=cfg.batch, max_ctx=cfg.ctx_len, max_sub=cfg.n_sub,
                               max_sub_tokens=cfg.sub_tokens, max_pos=max_positions(cfg),
                               kv_pair_layers=args.kv_pair_layers)
        pair_layers = dec.get_info(binding.PD_INFO_KV_PAIR_LAYERS)
        dec.set_option(binding.PD_OPT_USE_GRAPH, args.graph)
        dec.set_option(binding.PD_OPT_ATTN_SPLITS, args.attn_splits)
        dec.set_option(binding.PD_OPT_PREFILL_CHUNK, args.prefill_chunk)
        if args.calibrate_copy_mb > 0:
            src = torch.ones(args.calibrate_copy_mb << 20, dtype=torch.uint8, device="cuda")
            dst = torch.empty_like(src)
            for _ in range(3):
                dst.copy_(src)
            del src, dst
        # context pass: three calls, the first one cold (its kernels are loaded on first use); one call in
        # runs without the extra passes (profiler runs)
        prefill_calls = []
        for _ in range(1 if args.no_event_passes else 3):
            torch.cuda.synchronize()
            t0 = time.time()
            dec.prefill_context(ctx, cfg.n_sub, cfg.delta_t, cfg.sub_tokens, T)
            torch.cuda.synchronize()
            prefill_calls.append(time.time() - t0)
        prefill_s = sorted(prefill_calls)[len(prefill_calls) // 2]
        context_pairs = bool(dec.get_info(binding.PD_INFO_CONTEXT_PAIRS))
        # the same pass with single bf16 activations (PD_OPT_CONTEXT_SPLIT_ACT 0: half the multiplies, 5-8 times
        # the logit error; an option, not what the timed decode below runs on), then the default again
        prefill_single = None
        if cfg.dtype == 1 and not args.no_event_passes:
            dec.set_option(binding.PD_OPT_CONTEXT_SPLIT_ACT, 0)
            single_calls = []
            for _ in range(2):
                torch.cuda.synchronize()
                t0 = time.time()
                dec.prefill_context(ctx, cfg.n_sub, cfg.delta_t, cfg.sub_tokens, T)
                torch.cuda.synchronize()
                single_calls.append(time.time() - t0)
            prefill_single = min(single_calls)
            dec.set_option(binding.PD_OPT_CONTEXT_SPLIT_ACT, 1)
            dec.prefill_context(ctx, cfg.n_sub, cfg.delta_t, cfg.sub_tokens, T)
            torch.cuda.synchronize()
        def advance(n):
            """n decode iterations; under --sync-every in groups with a synchronisation after each."""
            if args.sync_every > 0:
                for k0 in range(0, n, args.sync_every):
                    dec.decode_steps(min(args.sync_every, n - k0))
                    torch.cuda.synchronize()
            else:
                dec.decode_steps(n)

        # warm-up: W untimed iterations
        advance(W)
        torch.cuda.synchronize()

        def timed_window():
            """Back to t = 0, untimed fast-forward to the window, then exactly K timed iterations."""
            dec.reset_decode()
            advance(t0w - 1)
            torch.cuda.synchronize()
            t_start = time.perf_counter()
            advance(K)
            torch.cuda.synchronize()
            return time.perf_counter() - t_start

        times = [timed_window() for _ in range(reps)]
        elapsed = statistics.median(times)
        attn_us, attn_launches, pair_us, read_gbs, full, in_place_us = 0.0, 0, 0.0, 0.0, None, 0.0
        if not args.no_event_passes:
            # the whole run, all T iterations from t = 1 (the metric as defined: B*S*M tokens over the T steps)
            full_times = []
            for _ in range(3 if K < T else 0):
                dec.reset_decode()
                torch.cuda.synchronize()
                t_start = time.perf_counter()
                dec.decode_steps(T)
                torch.cuda.synchronize()
                full_times.append(time.perf_counter() - t_start)
            if K >= T:
                full_times = times
            ft = statistics.median(full_times)
            full_tokens = cfg.batch * cfg.n_sub * cfg.sub_tokens
            full = {"steps": T, "tokens": full_tokens, "ms_per_step": ft / T * 1e3,
                    "tokens_per_s": full_tokens / ft, "repeats": len(full_times),
                    "hbm_frac_step": step_bytes(cfg, 1, T, pair_layers) / (ft / T) / 1e9 / HBM_PEAK_GBS}
            # the same window again with HIP events attached to every launch of the attention kernel (the
            # one that streams the keys and values); then with events around that kernel and the small
            # kernel that merges its partial results
            dec.set_option(binding.PD_OPT_USE_GRAPH, 0)
            for mode in (1, 2):
                dec.reset_decode()
                dec.decode_steps(t0w - 1)
                torch.cuda.synchronize()
                dec.set_option(binding.PD_OPT_PROFILE, mode)
                dec.decode_steps(K)
                torch.cuda.synchronize()
                us, n = dec.profile_read()
                dec.set_option(binding.PD_OPT_PROFILE, 0)
                if mode == 1:
                    attn_us, attn_launches = us, n
                else:
                    pair_us = us
            # The kernel's cost where it runs, with no event next to it: the window between two HIP events on
            # the launch stream, alternately as it is and with every launch of the kernel doubled (the extra
            # launch reads another layer's cache, same size, and its output is overwritten by the real one);
            # the difference of the medians per extra launch.
            def window_between_events(mode):
                dec.reset_decode()
                advance(t0w - 1)
                dec.set_option(binding.PD_OPT_PROFILE, mode)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                advance(K)
                e1.record()
                e1.synchronize()
                dec.set_option(binding.PD_OPT_PROFILE, 0)
                return e0.elapsed_time(e1) * 1e-3
            plain, doubled = [], []
            for _ in range(reps):
                plain.append(window_between_events(0))
                doubled.append(window_between_events(3))
            extra_launches = K * (cfg.n_layer - pair_layers)
            in_place_us = (statistics.median(doubled) - statistics.median(plain)) / extra_launches * 1e6 if extra_launches else 0.0
            # what a kernel that only reads reaches on this device, at the size of one attention launch
            buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
            buf.fill_(1)
            torch.cuda.synchronize()
            chunk = int(attention_bytes(cfg, t0w, t1w)) // 4096 * 4096
            read_gbs = binding.measure_read_bandwidth(buf.data_ptr(), buf.numel(), chunk, 200,
                                                      torch.cuda.current_stream().cuda_stream)
            del buf
        dec.close()

    tokens = cfg.batch * sum(producing(cfg, t) for t in range(t0w, t1w + 1))
    # a pair layer reads every key and value twice (high and low halves)
    abytes = attention_bytes(cfg, t0w, t1w) * (1.0 + pair_layers / cfg.n_layer)
    # the kernel's duration: the in-place figure (it agrees with the rocprofv3 kernel trace of the same command;
    # the events attached to a dispatch also time the command processor's handling of their own two packets,
    # 1.2-1.6 us, which no kernel of an ordinary step pays); the attached-event figure is reported beside it
    launch_us = in_place_us if in_place_us > 0 else attn_us
    achieved = abytes / (launch_us * 1e-6) / 1e9 if launch_us > 0 else 0.0
    # HBM bytes per launch from the rocprofv3 counter runs summarised under profiles/: the figure
    # measured for exactly this window when there is one, else the measured ratio of counter bytes to
    # algorithmic bytes (over the full run) times this window's algorithmic bytes; null if neither
    traffic, traffic_src = None, None
    pmc = os.path.join(ROOT, "profiles", f"attention_{cfg.name}_hbm_traffic.md")
    if os.path.exists(pmc):
        text = open(pmc).read()
        m = re.search(rf"bytes_per_launch\[t{t0w}-{t1w}\]\s*=\s*(\d+)", text)
        r = re.search(r"traffic_over_algorithmic\s*=\s*([0-9.]+)", text)
        if m:
            traffic, traffic_src = float(m.group(1)), "rocprofv3 FETCH_SIZE + WRITE_SIZE over this window"
        elif r:
            traffic = float(r.group(1)) * abytes
            traffic_src = "rocprofv3 FETCH_SIZE + WRITE_SIZE ratio to algorithmic bytes over the full run, scaled to this window"
    sbytes = step_bytes(cfg, t0w, t1w, pair_layers)
    out = {
        "metric": "pipelined_decode_generated_tokens_per_s", "value": tokens / elapsed, "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": elapsed / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == 1 else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.n_layer} layers, d_model {cfg.d_model}, "
                               f"{cfg.n_head}x{cfg.head_dim} heads, FFN {cfg.d_ff}, vocab {cfg.vocab}, "
                               f"batch {cfg.batch}, context {cfg.ctx_len}, S={cfg.n_sub}, dt={cfg.delta_t}, "
                               f"M={cfg.sub_tokens}",
                   "window": {"first_iteration": t0w, "last_iteration": t1w,
                              "rows_per_request": [fed(cfg, t0w), fed(cfg, t1w)],
                              "reached_by": "untimed decode iterations from t = 1" if t0w > 1 else "start of the run"},
                   "repeats": reps, "repeat_ms_per_step": [x / K * 1e3 for x in times], "statistic": "median",
                   "tokens_generated": tokens, "time_steps_full_run": T,
                   "prefill_s": prefill_s, "prefill_first_call_s": prefill_calls[0],
                   "context_activations": "bf16 pairs" if context_pairs else "single bf16",
                   "prefill_s_single_bf16_activations": prefill_single, "hip_graph": bool(args.graph),
                   "kv_pair_layers": pair_layers},
        "full_run": full,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_src,
                     "kernel": "k_attn_mfma (masked multi-query attention over the KV cache, one launch "
                               "per layer per step)",
                     "algorithmic_bytes_per_launch": abytes, "avg_launch_us": launch_us,
                     "launches": attn_launches,
                     "timing": "HIP events on the launch stream around the window, as it is and with every launch "
                               "of the kernel doubled (the extra launch reads another layer's cache of the same "
                               "size; its output is overwritten); difference of the medians per extra launch"
                               if in_place_us > 0 else "HIP start and stop events attached to every dispatch",
                     "attached_events": {"avg_us": attn_us,
                                         "frac": abytes / (attn_us * 1e-6) / 1e9 / HBM_PEAK_GBS if attn_us > 0 else 0.0,
                                         "note": "HIP start and stop events attached to every dispatch of the kernel, "
                                                 "in a further pass over the same window; includes the command "
                                                 "processor's handling of the two event packets"},
                     "with_merge_kernel": {"avg_us": pair_us,
                                           "frac": abytes / (pair_us * 1e-6) / 1e9 / HBM_PEAK_GBS if pair_us > 0 else 0.0,
                                           "note": "attention kernel plus the kernel that merges its split "
                                                   "partials, events around the pair; same algorithmic bytes"},
                     "step": {"algorithmic_bytes": sbytes, "ms": elapsed / K * 1e3,
                              "achieved": sbytes / (elapsed / K) / 1e9,
                              "frac": sbytes / (elapsed / K) / 1e9 / HBM_PEAK_GBS,
                              "note": "all kernels of one time-step: every weight once, every request's keys "
                                      "and values once per layer"},
                     "plain_read_same_bytes": {"GB/s": read_gbs, "frac_of_peak": read_gbs / HBM_PEAK_GBS,
                                               "note": "a kernel that only reads this many bytes, launched "
                                                       "back to back on the same device"}},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, weights, ctx)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
