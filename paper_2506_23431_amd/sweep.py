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

  python -m paper_2506_23431_amd.sweep --ragged pubmed [--workload cfg4] [--dt-list 2,4,8]

runs targets of uneven shape instead: per request a number of subsequences and their lengths are
drawn (seeded) around the averages of a sentence-level dataset of Table 1, every subsequence ends with
<eos> when its length is reached, and the subsequences opened after the last real one come back
empty (Algorithm 1 keeps opening one every dt steps while any is unfinished).  The end-of-sequence
decisions are forced from the host, one decode step per call; everything else (row bookkeeping,
early termination, ragged rows) runs on the device as in any other run.  The sequential baseline
generates the same tokens plus one separator per boundary as a single subsequence.

  python -m paper_2506_23431_amd.sweep --encdec encdec-base [--shape pubmed|wikihowqa|cnndm] [--dt-list 1,2,3]

runs the encoder-decoder form (the form the paper measures, Section 5.1: inference batch size 1, the
encoder included in the time of an example) on a backbone-shaped model with random weights: targets of
S subsequences of M tokens, S and M the rounded averages of a dataset of Table 1, sequentially (one
subsequence of S*M tokens) and pipelined; reports examples per second and the speed-up.
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


# Table 1, sentence-level rows: average subsequences per target, average words per subsequence
RAGGED = {"wikihowqa": (7.8, 9.6), "cnndm": (3.8, 14.4), "pubmed": (6.9, 30.0)}
TOKENS_PER_WORD = 1.3       # assumption of this build (sub-word vocabulary); the paper counts words


def draw_ragged(profile, batch, delta_t, seed=0, s_max=None):
    """Per request: a list of subsequence lengths in tokens (Poisson around the profile's averages).
    Every length is at least delta_t, so that a subsequence is still running when the next one
    opens (otherwise Algorithm 1 would stop with all opened subsequences finished)."""
    import numpy as np
    mean_n, mean_words = RAGGED[profile]
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(batch):
        n = max(1, int(rng.poisson(mean_n)))
        if s_max is not None:
            n = min(n, s_max)
        out.append([max(delta_t, int(rng.poisson(mean_words * TOKENS_PER_WORD))) for _ in range(n)])
    return out


def ragged_plan(lens, delta_t):
    """(S, M, T) that hold a ragged target: one exploratory subsequence after the last real one
    of the longest request, M = longest subsequence + its <eos>."""
    S = max(len(l) for l in lens) + 1
    M = max(max(l) for l in lens) + 1
    return S, M, (S - 1) * delta_t + M


def run_ragged(dec, ctx, lens, S, dt, M, T, eos_id):
    """Steps the library until every request is done, forcing <eos> where a subsequence has
    reached its drawn length (subsequences beyond the drawn ones: at once).  Returns
    (steps, seconds, produced) with produced[b][i] = tokens of subsequence i without <eos>."""
    import numpy as np
    import torch
    B = len(lens)
    target = np.zeros((B, S), dtype=np.int64)
    for b, l in enumerate(lens):
        target[b, :len(l)] = l
    dec.prefill_context(ctx, S, dt, M, T)
    produced = np.zeros((B, S), dtype=np.int64)
    ended = np.zeros((B, S), dtype=bool)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    steps = 0
    for t in range(1, T + 1):
        force = np.where((produced >= target) & ~ended, eos_id, -1).astype(np.int32)
        toks, _, done = dec.decode_step(force=force)
        steps = t
        got = toks >= 0
        is_eos = got & (toks == eos_id)
        produced += got & ~is_eos
        ended |= is_eos
        if done:
            break
    torch.cuda.synchronize()
    return steps, time.perf_counter() - t0, produced


def main_ragged(args):
    import numpy as np
    import torch
    import pd_inputs as pi
    from paper_2506_23431_amd import PipelinedDecoder

    base = pi.get_config(args.workload)
    if args.layers:
        base = base.scaled(n_layer=args.layers)
    eos = 1 if base.bos_id != 1 else 2
    dt_list = [int(x) for x in args.dt_list.split(",")]
    # args.targets seeded targets per request slot, the same ones for every delay (lengths clamped
    # to the largest delay); the sequential baseline generates each target's tokens plus one
    # separator per boundary as a single subsequence
    targets = [draw_ragged(args.ragged, base.batch, max(dt_list), seed=base.seed + 1000 * k)
               for k in range(args.targets)]
    runs = [("sequential", 1)] + [("pipelined", dt) for dt in dt_list]

    def plan(mode, dt, lens):
        if mode == "sequential":
            lens = [[sum(l) + len(l) - 1] for l in lens]
            return lens, 1, max(l[0] for l in lens) + 1, max(l[0] for l in lens) + 1
        S, M, T = ragged_plan(lens, dt)
        return lens, S, M, T

    plans = {(m, dt): [plan(m, dt, lens) for lens in targets] for m, dt in runs}
    S_cap = max(p[1] for ps in plans.values() for p in ps)
    M_cap = max(p[2] for ps in plans.values() for p in ps)
    mp = base.ctx_len + max((p[1] - 1) * (dt + 1) + p[2] + 1 for (m, dt), ps in plans.items() for p in ps)
    weights = pi.make_weights(base.scaled(n_sub=1, delta_t=1, sub_tokens=mp - base.ctx_len - 1))
    ctx = pi.make_context(base)
    rows = []
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        dec = PipelinedDecoder(base.scaled(eos_id=eos), weights, max_batch=base.batch, max_ctx=base.ctx_len,
                               max_sub=S_cap, max_sub_tokens=M_cap, max_pos=mp,
                               kv_pair_layers=args.kv_pair_layers)
        for mode, dt in runs:
            steps_all, sec_all, tokens_all, as_drawn = 0, 0.0, 0, True
            for (lens, S, M, T), target in zip(plans[(mode, dt)], targets):
                best = None
                for _ in range(2):
                    steps, sec, produced = run_ragged(dec, ctx, lens, S, dt, M, T, eos)
                    best = sec if best is None else min(best, sec)
                # (the random-weight model may emit <eos> by itself before a forced one: reported)
                want = np.zeros_like(produced)
                for b, l in enumerate(lens):
                    want[b, :len(l)] = l
                as_drawn &= bool(np.array_equal(produced, want))
                steps_all += steps
                sec_all += best
                tokens_all += int(sum(sum(l) for l in target))
            rows.append({"mode": mode, "dt": dt, "targets": len(targets), "steps": steps_all,
                         "ms_per_step": sec_all / steps_all * 1e3, "target_tokens": tokens_all,
                         "tokens_per_s": tokens_all / sec_all, "lengths_as_drawn": as_drawn})
            print(f"{mode:10s} dt={dt:2d}: {len(targets)} targets, {steps_all:5d} steps, "
                  f"{sec_all / steps_all * 1e3:7.3f} ms/step, {tokens_all / sec_all:9.1f} target tokens/s",
                  flush=True)
        dec.close()
    for r in rows:
        r["speedup_vs_sequential"] = r["tokens_per_s"] / rows[0]["tokens_per_s"]
    n_sub = [len(l) for t in targets for l in t]
    n_tok = [x for t in targets for l in t for x in l]
    print(json.dumps({"workload": base.name, "n_layer": base.n_layer, "ragged": args.ragged,
                      "batch": base.batch, "context": base.ctx_len,
                      "mean_subsequences": float(np.mean(n_sub)), "mean_tokens_per_subsequence": float(np.mean(n_tok)),
                      "results": rows}))
    return rows


def main_encdec(args):
    import numpy as np
    import torch
    import pd_inputs as pi
    from paper_2506_23431_amd.binding import EncDecPipelinedDecoder

    base = pi.ENCDEC_CONFIGS[args.encdec]
    if args.layers:
        base = base.scaled(n_enc_layer=args.layers, n_dec_layer=args.layers)
    mean_n, mean_words = RAGGED[args.shape]
    S, M = max(1, round(mean_n)), max(1, round(mean_words * TOKENS_PER_WORD))
    N = S * M
    plans = [(1, 1, N)] + [(S, dt, M) for dt in [int(x) for x in args.dt_list.split(",")]]
    _, weights = pi.encdec_to_bf16(pi.make_encdec_weights(base, threads=8))
    ctx = pi.make_context(base)
    rows = []
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        dec = EncDecPipelinedDecoder(base, weights, max_batch=base.batch, max_ctx=base.ctx_len, max_sub=S,
                                     max_sub_tokens=N)
        if args.attn_splits:
            from paper_2506_23431_amd import binding
            dec.set_option(binding.PD_OPT_ATTN_SPLITS, args.attn_splits)
        for s_, dt, m_ in plans:
            T = (s_ - 1) * dt + m_
            enc_s, dec_s = [], []
            for _ in range(args.repeats + 1):           # the first pass warms up and is dropped
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                dec.prefill_context(ctx, s_, dt, m_, T)
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                dec.decode_steps(T)
                torch.cuda.synchronize()
                t2 = time.perf_counter()
                enc_s.append(t1 - t0)
                dec_s.append(t2 - t1)
            e, d_ = float(np.median(enc_s[1:])), float(np.median(dec_s[1:]))
            rows.append({"S": s_, "dt": dt, "M": m_, "steps": T, "encode_ms": e * 1e3, "ms_per_step": d_ / T * 1e3,
                         "examples_per_s": base.batch / (e + d_), "tokens_per_s": base.batch * N / (e + d_)})
            print(f"S={s_:3d} dt={dt:2d} M={m_:4d}: {T:4d} steps, encode {e * 1e3:6.2f} ms, {d_ / T * 1e3:6.3f} ms/step, "
                  f"{base.batch / (e + d_):7.2f} examples/s", flush=True)
        dec.close()
    for r in rows:
        r["speedup_vs_sequential"] = r["examples_per_s"] / rows[0]["examples_per_s"]
    print(json.dumps({"workload": base.name, "layers": [base.n_enc_layer, base.n_dec_layer], "d_model": base.d_model,
                      "input_tokens": base.ctx_len, "batch": base.batch, "shape": args.shape,
                      "target_tokens": N, "results": rows}))
    return rows


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="cfg4")
    ap.add_argument("--s-list", default="1,2,4,8,16,32")
    ap.add_argument("--dt-list", default="1,2,4,8,16")
    ap.add_argument("--tokens", type=int, default=0, help="total generated tokens N (default: S*M of the workload)")
    ap.add_argument("--layers", type=int, default=0, help="use only this many layers (quick runs)")
    ap.add_argument("--kv-pair-layers", type=int, default=None,
                    help="leading layers whose cache keeps keys and values as pairs of halves (default: -1, the library chooses from the shape)")
    ap.add_argument("--ragged", default="", choices=[""] + sorted(RAGGED),
                    help="uneven targets drawn around this dataset's averages (Table 1), <eos>-terminated")
    ap.add_argument("--targets", type=int, default=8, help="ragged mode: seeded targets per request slot")
    ap.add_argument("--encdec", default="", help="encoder-decoder form on this shape (encdec-small, encdec-base, encdec-large)")
    ap.add_argument("--shape", default="pubmed", choices=sorted(RAGGED), help="encoder-decoder mode: target shape (Table 1 averages)")
    ap.add_argument("--repeats", type=int, default=5, help="encoder-decoder mode: timed passes per schedule (median)")
    ap.add_argument("--attn-splits", type=int, default=0, help="encoder-decoder mode: work-groups per (request, head) in the attention kernel (0: automatic)")
    args = ap.parse_args(argv)
    if args.encdec:
        if args.dt_list == "1,2,4,8,16":
            args.dt_list = "1,2,3"
        return main_encdec(args)
    if args.kv_pair_layers is None:
        args.kv_pair_layers = -1
    if args.ragged:
        return main_ragged(args)

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
