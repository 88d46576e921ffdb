"""Shared driver of the GPU parity tests: runs the CPU oracle and the HIP library on the
same seeded workload, teacher-forced, and compares every logit row."""

import numpy as np

import pd_inputs as pi
from pd_inputs import max_positions
from oracle.model import OracleModel
from oracle import pipelined

TOL = {0: 1e-4, 1: 2e-2}      # max-abs logit tolerance: fp32 / bf16 (spec bar)
MARGIN = 0.05                 # greedy tokens must agree where the oracle's top-2 margin exceeds this


def oracle_run(cfg, weights, ctx, force=None, steps=None, context_kv=None, log=None, cache_layers=True):
    """Oracle traces per request. force: int array [steps][B][S] or None.
    log: optional callable; gets a progress line at least every ~20 s of oracle work.
    cache_layers=False converts every layer's weights to fp64 each time they are used instead of
    keeping all of them (a 7B-parameter model would hold 52 GB of fp64 copies)."""
    import time
    from oracle import controller
    model = OracleModel(cfg, weights, cache_layers=cache_layers)
    outs = []
    last = [time.time()]

    def tick(msg):
        if log is not None and time.time() - last[0] > 20:
            log(msg)
            last[0] = time.time()

    for b in range(cfg.batch):
        f = None if force is None else force[:, b, :]
        kv = None if context_kv is None else context_kv[b]
        if kv is None:
            kv = model.prefill(ctx[b], progress=lambda l, b=b: tick(
                f"[oracle] {cfg.name}: request {b} context pass, layer {l + 1}/{cfg.n_layer}"))
            tick(f"[oracle] {cfg.name}: request {b} context pass done")
        dec = pipelined.PerQueryDecoder(model, ctx[b], force=f, context_kv=kv)

        def stepper(G, t, dec=dec, b=b):
            out = dec(G, t)
            tick(f"[oracle] {cfg.name}: request {b} iteration {t}")
            return out

        result, n_steps, emitted = controller.pipelined_decode(
            stepper, cfg.delta_t, cfg.time_steps if steps is None else steps, cfg.n_sub, cfg.bos_id,
            cfg.eos_id, cfg.sub_tokens)
        outs.append({"result": result, "steps": n_steps, "emitted": emitted, "trace": dec.trace})
    return outs


def make_decoder(cfg, weights, **kw):
    """The library on this workload, with the library's own choice of pair layers (from the shape)."""
    from paper_2506_23431_amd import PipelinedDecoder
    args = dict(max_batch=cfg.batch, max_ctx=cfg.ctx_len, max_sub=cfg.n_sub,
                max_sub_tokens=cfg.sub_tokens, max_pos=max_positions(cfg))
    args.update(kw)
    return PipelinedDecoder(cfg, weights, **args)


def compare_teacher_forced(cfg, weights, ctx, dec, outs, force=None, steps=None, tol=None, log=print):
    """Steps the library with the oracle's tokens and checks logits and greedy tokens.

    Rows whose oracle top-2 margin exceeds MARGIN are NOT forced: the library must pick the
    same token by itself (bit-exact).  All other produced rows are forced to the oracle's token
    so that both sides keep the same history.  Returns summary statistics."""
    tol = TOL[cfg.dtype] if tol is None else tol
    B, S = cfg.batch, cfg.n_sub
    n_steps = max(o["steps"] for o in outs)
    if steps is not None:
        n_steps = min(n_steps, steps)
    dec.prefill_context(ctx, S, cfg.delta_t, cfg.sub_tokens, cfg.time_steps if steps is None else steps)
    worst, n_rows, n_exact = 0.0, 0, 0
    import os
    verbose = os.environ.get("PD_PARITY_VERBOSE") == "1"
    for t in range(1, n_steps + 1):
        f = np.full((B, S), -1, dtype=np.int32)
        expect = np.full((B, S), -1, dtype=np.int32)
        free = np.zeros((B, S), dtype=bool)
        for b, o in enumerate(outs):
            if t > o["steps"]:
                continue
            rec = o["trace"][t - 1]
            for i, tok in o["emitted"][t - 1].items():
                lg = rec["logits"][rec["rows"].index(i)]
                top2 = np.partition(lg, -2)[-2:]
                expect[b, i - 1] = tok
                forced_here = force is not None and force[t - 1, b, i - 1] >= 0
                if (top2[1] - top2[0]) > MARGIN and not forced_here:
                    free[b, i - 1] = True          # library decides; must equal the oracle
                else:
                    f[b, i - 1] = tok
        toks, logits, done = dec.decode_step(force=f, want_logits=True)
        logits = logits.cpu().numpy().astype(np.float64)
        for b, o in enumerate(outs):
            if t > o["steps"]:
                continue
            rec = o["trace"][t - 1]
            for r, i in enumerate(rec["rows"]):
                err = np.abs(logits[b, i - 1] - rec["logits"][r]).max()
                assert np.isfinite(err), f"step {t} request {b} subsequence {i}: non-finite logits"
                worst = max(worst, err)
                n_rows += 1
                if verbose:
                    log(f"  step {t} req {b} sub {i}: err {err:.3e}")
                assert err <= tol, (f"step {t} request {b} subsequence {i}: max|logit diff| = "
                                    f"{err:.3e} > {tol}")
        assert np.array_equal(toks[expect >= 0], expect[expect >= 0]), \
            f"step {t}: tokens {toks.tolist()} != oracle {expect.tolist()} (free rows {free.tolist()})"
        assert np.all(toks[expect < 0] == -1), f"step {t}: token produced where the oracle has none"
        n_exact += int(free.sum())
        all_done = all(t >= o["steps"] for o in outs)
        if steps is None:
            assert done == all_done, f"step {t}: all_done = {done}, oracle says {all_done}"
    log(f"[parity] {cfg.name}: {n_steps} steps, {n_rows} logit rows, max|diff| = {worst:.3e} "
        f"(tol {tol}), {n_exact} greedy tokens chosen by the library and bit-exact")
    return {"worst": worst, "rows": n_rows, "exact": n_exact}
