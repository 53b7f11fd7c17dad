#!/usr/bin/env python3
"""Throughput of the SFB hot path on one MI355X.

A "step" is one full bulk-synchronous SFB iteration (scores, factor u, factor v, the
concatenation standing in for the broadcast, reconstruction, W update) over one synthetic
minibatch of P*B samples whose features, labels and W already sit in HBM.

Prints ONE JSON line.  Its headline fields (value, ms_per_step, dtype, config, roofline,
cpu_baseline) are those of the largest configuration, mlr_large (W of 860 MB, bf16 features);
`configs` carries the same record for every configuration of the benchmark set, `floors` the
yardsticks measured in the same process (plain copy, bare W traffic in the kernels' access shapes,
register-resident matrix-core loops).

Procedure per configuration: W warm-up steps, then 5 repeats of exactly K timed steps, each
bracketed by torch.cuda.synchronize() and started from W0; `value` is N*K over the MEDIAN repeat
(min and all five are reported too).  A separate instrumented pass times every kernel from HIP
events attached to its own dispatch on the library's stream; `roofline` is the dominant
contraction's algorithmic flops (or bytes) over that duration, against the MI355X peak that
bounds it.  `cpu_baseline` is the fp64 numpy oracle timed on this host's cores on a bounded
number of the same steps: a reported baseline, not a target.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3     # MI355X dense fp32 matrix-core peak
PEAK_BF16_MFMA_TFLOPS = 2500.0    # dense bf16
PEAK_HBM_GBS = 8000.0
FAMILIES = {0: "scores", 1: "factor u", 2: "reconstruct-apply", 3: "csr densify", 5: "update + next scores (one pass)"}
ALL_CONFIGS = ["mlr_large", "mlr_medium", "dml", "l2svm", "mlr_tiny"]      # headline first
REPEATS = 5


def cpu_baseline(wl, budget_s):
    """The oracle as it stands, on the host cores, for a bounded number of steps."""
    import numpy as np
    import oracle
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    W = wl.W0.astype(np.float64)
    _, _, W, _ = oracle.step(wl.model, W, wl.batch(0), wl.P, wl.B, wl.eta)      # warm-up
    n, t0 = 0, time.perf_counter()
    while True:
        _, _, W, _ = oracle.step(wl.model, W, wl.batch(n + 1), wl.P, wl.B, wl.eta)
        n += 1
        el = time.perf_counter() - t0
        if el >= budget_s or n >= 200:
            break
    return {"value": wl.N * n / el, "unit": "samples/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{n} consecutive fp64 numpy oracle steps of {wl.name} (after 1 warm-up step), "
                      f"{el:.2f} s wall, {len(os.sched_getaffinity(0))} cores in the affinity mask",
            "steps_per_s": n / el}


def stage_pool(wl, sfb, torch, dev):
    """The workload's batches as device tensors (resident in HBM before anything is timed)."""
    import numpy as np
    vdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    pool = []
    for b in wl.batches:
        y = torch.from_numpy(np.ascontiguousarray(b["y"], dtype=np.int32)).to(dev)
        if wl.model == "mlr":
            pool.append((sfb.SfbBatch(a=torch.from_numpy(b["A"]).to(vdt).to(dev)), y))
        elif wl.model == "dml":
            pool.append((sfb.SfbBatch(a=torch.from_numpy(b["X"]).to(dev), a2=torch.from_numpy(b["Y"]).to(dev)), y))
        else:
            pool.append((sfb.SfbBatch(rowptr=torch.from_numpy(b["rowptr"]).to(dev),
                                      col=torch.from_numpy(b["col"]).to(dev),
                                      val=torch.from_numpy(b["val"]).to(dev)), y))
    return pool, vdt


SETTLE_S = 0.3


def settle(run, restore, torch, chunk):
    """Untimed: keeps the step loop running for SETTLE_S seconds (W restored every `chunk` steps) and returns the
    number of steps run.  The device needs tens of milliseconds of sustained load before its dispatch path reaches
    its steady rate: straight after the W warm-up steps asked for (0.5 ms of work at mlr_medium) a 20-step repeat reads
    9 % above the same repeat taken after this loop (2 % at mlr_large), and any run of a few thousand steps is in the
    steady state.  The timed regions are untouched: exactly `steps` steps between two synchronisations."""
    done = 0
    t_end = time.perf_counter() + SETTLE_S
    while time.perf_counter() < t_end:
        restore()
        run(chunk)
        torch.cuda.synchronize()
        done += chunk
    return done


def timed_repeats(run, restore, torch, steps, repeats=REPEATS):
    """`repeats` times: restore W, synchronise, time exactly `steps` steps, synchronise."""
    out = []
    for _ in range(repeats):
        restore()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(steps)
        torch.cuda.synchronize()
        out.append(time.perf_counter() - t0)
    return out


def roofline_of(wl, per_kernel, split_k, traffic_table, pipelined):
    """Roofline record of the dominant contraction.  fp32 workloads: both contractions are bound by
    the fp32 matrix cores (2*N*J*D flops per launch).  bf16 workload: bound by streaming W through
    HBM; algorithmic bytes per launch are W once (scores) / twice (reconstruction) plus the factor
    operands; the fused update-and-score pass reads and writes W once and carries both contractions."""
    flops = 2.0 * wl.N * wl.J * wl.D
    cands = [f for f in per_kernel if f in (0, 2)]
    if wl.model == "l2svm" and 0 in cands:
        cands.remove(0)                                     # CSR scores: a gather kernel, no dense roofline
    dom = max(cands, key=lambda f: per_kernel[f][1])
    if pipelined and 5 in per_kernel:
        dom = 5                                             # every step but the chain's two ends is this one kernel
    us = per_kernel[dom][1]
    traffic = traffic_table.get(f"{wl.name}:{'fused' if pipelined else dom}")
    if wl.dtype == "bf16":
        wbytes = 4.0 * wl.J * wl.D
        if pipelined:
            # W read + written once; packed factors (alpha u)^T, v^T and next features read once; partial scores written
            alg = 2.0 * wbytes + 2.0 * wl.N * (wl.J + wl.D) + 2.0 * wl.N * wl.D + split_k * 4.0 * wl.N * wl.J
        elif dom == 0:
            alg = wbytes + 2.0 * wl.N * wl.D * 2 + split_k * 4.0 * wl.N * wl.J
        else:
            alg = 2.0 * wbytes + 2.0 * wl.N * (wl.J + wl.D)
        achieved = alg / (us * 1e-6) / 1e9
        r = {"bound": "hbm", "kernel": per_kernel[dom][0], "achieved": achieved, "peak": PEAK_HBM_GBS,
             "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS, "traffic": traffic,
             "algorithmic_bytes": alg, "us_per_launch": us,
             "frac_of_bf16_mfma_peak": (2.0 if pipelined else 1.0) * flops / (us * 1e-6) / 1e12 / PEAK_BF16_MFMA_TFLOPS}
    else:
        achieved = flops / (us * 1e-6) / 1e12
        r = {"bound": "mfma", "kernel": per_kernel[dom][0], "achieved": achieved,
             "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_FP32_MFMA_TFLOPS,
             "traffic": traffic, "algorithmic_flops": flops, "us_per_launch": us}
    r["kernels_us"] = {v[0]: round(v[1], 2) for v in per_kernel.values()}
    return r


def bench_config(name, args, sfb, torch, workloads, traffic_table, cpu_seconds, extras=False):
    """One configuration: returns its record (the fields of the JSON line)."""
    dev = "cuda:0"
    over = {}
    if extras and args.shape:
        # e.g. --config dml --shape J=600,D=780: the configuration's model and recipe at another size
        over = {k: int(v) for k, v in (kv.split("=") for kv in args.shape.split(","))}
        if set(over) - {"J", "D", "P", "B"}:
            raise SystemExit("bench.py: --shape takes J, D, P and B only")
    wl = workloads.make(name, **over)
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, dtype=wl.dtype, device=dev)
    if args.plan:
        vals = [int(x) for x in args.plan.split(",")] + [-1]
        ctx.set_plan(*vals[:5])
    pool, vdt = stage_pool(wl, sfb, torch, dev)
    W0 = torch.from_numpy(wl.W0).to(dev)
    W = W0.clone()
    U = torch.empty((wl.N, wl.J), dtype=torch.float32, device=dev)
    V = torch.empty((wl.N, wl.D), dtype=vdt, device=dev)
    pipelined = bool(args.pipelined) and hasattr(ctx, "pipeline_ok") and ctx.pipeline_ok()

    def run_eager(k):
        for t in range(k):
            b, y = pool[t % len(pool)]
            ctx.step(W, b, y, U, V, wl.eta)

    def run_pipelined(k):
        # same K updates of W and K factor computations, regrouped: factors of batch 0 first, then
        # K-1 calls that apply the pending factors and form the next batch's, then the last update
        b, y = pool[0]
        ctx.compute_factors(W, b, y, U, V)
        for t in range(1, k):
            b, y = pool[t % len(pool)]
            ctx.update_and_next_factors(W, U, V, b, y, wl.eta)
        ctx.reconstruct_apply(W, U, V, wl.eta)

    run = run_pipelined if pipelined else run_eager
    launch = "eager, update fused with the next batch's scores" if pipelined else "eager"
    steps, warmup = args.steps, args.warmup
    run(warmup)
    if args.graph:
        # one graph = one pass over the batch pool; replays keep the pool cycling as in the eager loop
        torch.cuda.synchronize()
        cap = torch.cuda.Stream(device=dev)
        with torch.cuda.stream(cap):
            gctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, dtype=wl.dtype, device=dev)
            if args.plan:
                gctx.set_plan(*vals[:5])
            for b, y in pool:
                gctx.step(W, b, y, U, V, wl.eta)      # warm-up on the capture stream
            cap.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=cap):
            for b, y in pool:
                gctx.step(W, b, y, U, V, wl.eta)

        def run_graph(k):
            assert k % len(pool) == 0, "--graph needs steps and warmup to be multiples of the batch pool size"
            for _ in range(k // len(pool)):
                graph.replay()

        run, launch = run_graph, "hip graph replay"
        warmup = max(len(pool), warmup // len(pool) * len(pool))
        steps = max(len(pool), steps // len(pool) * len(pool))
        run(warmup)

    settled = settle(run, lambda: W.copy_(W0), torch, max(warmup, len(pool)))
    times = timed_repeats(run, lambda: W.copy_(W0), torch, steps)
    assert bool(torch.isfinite(W).all()), "W is not finite after the timed steps"
    med, best = statistics.median(times), min(times)

    # instrumented pass: same launches (eager), HIP events attached to each dispatch on the library's stream
    # (a context's first launches with events attached read high -- 720 us where every later pass reads 620 us for the
    # one-pass kernel -- so a first pass fills the event pool and primes the profiled dispatch path and is thrown away)
    ctx.enable_timing(True)
    (run_pipelined if pipelined else run_eager)(min(steps, 200))
    ctx.reset_timing()
    W.copy_(W0)
    (run_pipelined if pipelined else run_eager)(min(steps, 200))
    per_kernel = {}
    for fam, fname in FAMILIES.items():
        ms, n = ctx.kernel_time_ms(fam)
        if n:
            per_kernel[fam] = (fname, ms / n * 1e3, n)       # microseconds per launch
    ctx.enable_timing(False)
    ctx.reset_timing()

    plan = ctx.plan_info()
    rec = {
        "metric": "sfb_samples_per_sec", "value": wl.N * steps / med, "unit": "samples/s",
        "steps_per_sec": steps / med,
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": med / steps * 1e3,
        "ms_per_step_min": best / steps * 1e3, "repeats_ms_per_step": [round(t / steps * 1e3, 6) for t in times],
        "timing": f"median of {REPEATS} repeats of {steps} steps, W restored to W0 before each; before them, untimed, "
                  f"{warmup} warm-up steps and {settled} more over {SETTLE_S} s (the device's dispatch path needs "
                  f"tens of ms of load to reach its steady rate)",
        "warmup_settle_steps": settled,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if wl.dtype == "f32" else "bf16 features, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.model} J={wl.J} D={wl.D} P={wl.P} B={wl.B} eta={wl.eta}",
                   "plan": plan, "launch": launch},
        "roofline": roofline_of(wl, per_kernel, plan["fwd_split_k"], {} if over else traffic_table, pipelined),
    }
    if extras:
        rec.update(extras_of(args, wl, ctx, sfb, torch, pool, W, W0, U, V, steps, warmup))
    if cpu_seconds > 0:
        rec["cpu_baseline"] = cpu_baseline(wl, cpu_seconds)
    ctx.close()
    return rec, (wl, W0)


def extras_of(args, wl, ctx, sfb, torch, pool, W, W0, U, V, steps, warmup):
    """Informational additions of the single-configuration mode."""
    dev = "cuda:0"
    out = {}
    if wl.dtype == "f32" and not args.plan and not args.graph:
        # the same steps with both contractions taken as split-bf16 products on the bf16 matrix cores
        # (opt-in plan bits 2 and 3; fp32-level error, same parity tests).  Not the headline.
        alt = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, dtype=wl.dtype, device=dev)
        alt.set_plan(fwd_dma=13)

        def run_alt(k):
            for t in range(k):
                b, y = pool[t % len(pool)]
                alt.step(W, b, y, U, V, wl.eta)
        run_alt(warmup)
        times = timed_repeats(run_alt, lambda: W.copy_(W0), torch, steps)
        assert bool(torch.isfinite(W).all()), "W is not finite after the split-bf16 steps"
        med = statistics.median(times)
        out["alt_plan"] = {"name": "split-bf16 contractions (sfb_set_plan fwd_dma=13)", "value": wl.N * steps / med,
                           "unit": "samples/s", "ms_per_step": med / steps * 1e3,
                           "note": "fp32 operands split exactly into three bf16 terms, six term products per product"}
        alt.close()
    if args.prox:
        # proximal SGD (Section 2.1), the step followed by the proximal operator of h
        kind, param = args.prox.split(":")
        param = float(param)

        def timed(fn):
            def go(k):
                for t in range(k):
                    fn(*pool[t % len(pool)])
            W.copy_(W0)
            go(warmup)
            return statistics.median(timed_repeats(go, lambda: W.copy_(W0), torch, steps)) / steps * 1e3

        def two_calls(b, y):
            ctx.step(W, b, y, U, V, wl.eta)
            ctx.prox(W, kind, wl.eta, param)

        out["proximal_step"] = {
            "h": f"{kind} (parameter {param})",
            "ms_per_step_one_call": timed(lambda b, y: ctx.step_prox(W, b, y, U, V, wl.eta, kind, param)),
            "ms_per_step_two_calls": timed(two_calls),
            "note": "sfb_step_prox folds the entrywise operators into the reconstruction's store; the column "
                    "projection runs as its own kernels either way"}
    if args.objective_every > 0:
        # objective vs samples on the synthetic data (Section 6's third panel), from the loss the factor kernel emits
        W.copy_(W0)
        loss = torch.empty((wl.N,), dtype=torch.float32, device=dev)
        curve = []
        for t in range(steps):
            b, y = pool[t % len(pool)]
            ctx.step(W, b, y, U, V, wl.eta, loss=loss)
            if t % args.objective_every == 0 or t == steps - 1:
                curve.append([wl.N * t, float(loss.double().mean().item())])
        out["objective_curve"] = {"unit": "mean per-sample loss of the step's batch, before its update",
                                  "samples_vs_loss": curve}
    return out


def measure_floors(sfb, torch, big_wl=None, big_W0=None):
    """Yardsticks from the library's measurement aids, each timed from the events of its own dispatch."""
    dev = "cuda:0"
    floors = {}
    ctx = sfb.Sfb("mlr", 1000, 4096, 8, 64, device=dev)

    def timed(ctx, launch, n=5):
        ctx.enable_timing(True)
        launch()                                        # warm-up, with events attached: the first such launches read high
        launch()
        ctx.reset_timing()
        for _ in range(n):
            launch()
        ms, cnt = ctx.kernel_time_ms(3)
        ctx.enable_timing(False)
        ctx.reset_timing()
        return ms / cnt * 1e3                           # microseconds per launch

    # plain streaming copy, 256 MiB each way: also the known-size kernel the HBM counters are scaled by
    big = torch.empty(2, 64 * 1024 * 1024, dtype=torch.float32, device=dev)
    big[0].fill_(1.0)
    us = timed(ctx, lambda: ctx.stream_copy(big[1], big[0]), 10)
    copy_bytes = 2.0 * big[0].numel() * 4
    floors["stream_copy"] = {"GB/s": copy_bytes / (us * 1e-6) / 1e9, "us_per_launch": us, "bytes_per_launch": copy_bytes,
                             "note": "plain float4 copy kernel, 256 MiB read + 256 MiB written per launch"}
    del big
    # register-resident matrix-core loops: what the cores sustain at the clock the part holds under that load
    iters = ctx.PROBE_MFMA_ITERS
    for kind, flop in (("mfma_f32", 4096.0), ("mfma_bf16", 32768.0)):
        for wps in (1, 2):
            us = timed(ctx, lambda: ctx.probe(kind, param=wps), 3)
            total = flop * 16 * iters * 256 * 4 * wps
            floors[f"{kind}_loop_{wps}_wavefronts_per_simd"] = {"TFLOP/s": total / (us * 1e-6) / 1e12, "us_per_launch": us}
    # an empty kernel: the dispatch cost under every launch-bound kernel (factor u at the small configurations);
    # back to back on the stream (wall clock over 200 launches) and from its own dispatch events
    us = timed(ctx, lambda: ctx.probe("empty"), 50)
    ctx.probe("empty")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(200):
        ctx.probe("empty")
    torch.cuda.synchronize()
    floors["empty_kernel"] = {"us_per_launch": us, "us_per_launch_back_to_back": (time.perf_counter() - t0) / 200 * 1e6,
                              "note": "256 workgroups that do nothing"}
    ctx.close()
    if big_wl is not None:
        # bare W traffic of the 860 MB matrix in the access shapes of the bf16 kernels
        wl = big_wl
        c2 = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, dtype=wl.dtype, device=dev)
        W = big_W0.clone()
        wbytes = 4.0 * wl.J * wl.D
        for dup in (1, 2):
            us = timed(c2, lambda: c2.probe("w_stream", W, dup), 5)
            floors[f"w_stream_read_{dup}x"] = {
                "us_per_launch": us, "GB/s_of_W": wbytes / (us * 1e-6) / 1e9,
                "note": f"W read in the bf16 score pass's access shape, every block by {dup} workgroup(s)"}
        us = timed(c2, lambda: c2.probe("w_rmw", W), 5)
        floors["w_read_modify_write"] = {
            "us_per_launch": us, "GB/s": 2.0 * wbytes / (us * 1e-6) / 1e9,
            "note": "W += 0 in the bf16 reconstruction's tile and lane mapping (256 x 128 tiles, accumulator layout)"}
        assert torch.equal(W, big_W0), "the read-modify-write probe must leave W as it was"
        if c2.pipeline_info()["fused"]:
            us = timed(c2, lambda: c2.probe("fused_traffic", W), 5)
            floors["one_pass_kernel_traffic_only"] = {
                "us_per_launch": us,
                "note": "the one-pass update + score kernel's own copies and stores (same grid, tiles, addresses and "
                        "instructions), no matrix work, no barriers: what the memory path alone takes for that traffic"}
            assert torch.equal(W, big_W0), "the traffic probe must leave W as it was"
        c2.close()
    return floors


def bench_sdca(args):
    """--config sdca_*: SFB driven by SDCA (Section 2.1) on a fixed synthetic data set.  A "step" is
    one iteration over P*B distinct picked samples: scores, dual update + factors, reconstruction.
    Same JSON keys as the main bench; informational (the headline configs are the SGD ones)."""
    import torch

    import paper_1511_08486_amd as sfb
    import workloads

    dev = "cuda:0"
    wl = workloads.make_sdca(args.config)
    ctx = sfb.Sfb("mlr", wl.J, wl.D, wl.P, wl.B, dtype=wl.dtype, device=dev)
    A = torch.from_numpy(wl.A).to(dev)
    yd = torch.from_numpy(wl.y).to(dev)
    pool = []
    for t in range(min(len(wl.picks), 4)):                   # gathered batches resident in HBM
        idx = torch.from_numpy(wl.pick(t)).to(dev)
        pool.append((sfb.SfbBatch(a=A[idx.long()].contiguous()), yd[idx.long()].contiguous(), idx))
    W = torch.zeros((wl.J, wl.D), dtype=torch.float32, device=dev)
    dual = torch.zeros((wl.n_data, wl.J), dtype=torch.float32, device=dev)
    U = torch.empty((wl.N, wl.J), dtype=torch.float32, device=dev)
    V = torch.empty((wl.N, wl.D), dtype=torch.float32, device=dev)
    s = 0.05

    def run(k):
        for t in range(k):
            b, y, idx = pool[t % len(pool)]
            ctx.sdca_step(W, b, y, dual, idx, wl.lam, s, U, V)

    run(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert bool(torch.isfinite(W).all())
    ctx.enable_timing(True)
    run(min(args.steps, 500))                           # fills the event pool: the first launches with events read high
    ctx.reset_timing()
    run(min(args.steps, 500))
    per = {}
    for fam, name in FAMILIES.items():
        ms, n = ctx.kernel_time_ms(fam)
        if n:
            per[name] = round(ms / n * 1e3, 2)
    ctx.enable_timing(False)
    flops = 2.0 * wl.N * wl.J * wl.D
    us = per["reconstruct-apply"]
    achieved = flops / (us * 1e-6) / 1e12
    out = {"metric": "sfb_samples_per_sec", "value": wl.N * args.steps / elapsed, "unit": "samples/s",
           "steps_per_sec": args.steps / elapsed, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"{wl.name}: SDCA on l2-regularised MLR, J={wl.J} D={wl.D} n_data={wl.n_data} "
                                  f"P={wl.P} B={wl.B} lam={wl.lam} s={s}", "plan": ctx.plan_info(), "launch": "eager"},
           "roofline": {"bound": "mfma", "kernel": "reconstruct-apply", "achieved": achieved,
                        "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_FP32_MFMA_TFLOPS,
                        "traffic": None, "algorithmic_flops": flops, "us_per_launch": us, "kernels_us": per}}
    if args.cpu_seconds > 0:
        from oracle.sdca_oracle import SdcaMlrOracle
        o = SdcaMlrOracle(wl.A, wl.y, wl.J, wl.lam)
        o.step_matrix(wl.pick(0), s)
        n, t1 = 0, time.perf_counter()
        while True:
            o.step_matrix(wl.pick(n + 1), s)
            n += 1
            el = time.perf_counter() - t1
            if el >= args.cpu_seconds or n >= 200:
                break
        out["cpu_baseline"] = {"value": wl.N * n / el, "unit": "samples/s", "cores": len(os.sched_getaffinity(0)),
                               "kind": "oracle", "sample": f"{n} fp64 numpy SDCA oracle iterations of {wl.name}, {el:.2f} s"}
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="all",
                    help="'all' (default): every configuration of the benchmark set, the largest one (mlr_large) as "
                         "the headline; or one configuration's name (also sdca_tiny / sdca_medium)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="oracle timing budget of the headline configuration (0 = skip; the others get a quarter)")
    ap.add_argument("--no-floors", action="store_true", help="skip the yardstick probes")
    ap.add_argument("--pipelined", type=int, default=1,
                    help="1 (default): where the library offers it for the shape, run the update fused with the next "
                         "batch's scores (one pass over W per step); 0: always the plain sfb_step sequence")
    ap.add_argument("--graph", action="store_true",
                    help="single configuration only: record the pool's steps in a HIP graph and time replays")
    ap.add_argument("--plan", default="", help="single configuration only: fwd_bm,fwd_bn,split_k,recon_variant[,fwd_dma]")
    ap.add_argument("--shape", default="",
                    help="single configuration only: J=..,D=..,P=..,B=.. (any subset) in place of the configuration's "
                         "own sizes, e.g. --config dml --shape J=600,D=780 (not a benchmark line: for ragged shapes)")
    ap.add_argument("--objective-every", type=int, default=0,
                    help="single configuration only: replay the steps from W0 (untimed) and report the mean per-sample "
                         "loss of the batch of every K-th step against samples processed")
    ap.add_argument("--prox", default="",
                    help="single configuration only: KIND:PARAM (l2sq, l1 or column_ball), also time proximal-SGD "
                         "iterations (the step followed by prox_{eta h}), fused and as two calls")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import __graft_entry__
    __graft_entry__.ensure_built()        # compiles only when no library has been built yet
    import paper_1511_08486_amd as sfb
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    if args.config.startswith("sdca"):
        return bench_sdca(args)
    traffic_table = {}
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        traffic_table = json.load(open(tpath))

    single = args.config != "all"
    if not single and (args.graph or args.plan or args.prox or args.objective_every or args.shape):
        print("bench.py: --graph, --plan, --prox, --shape and --objective-every need --config NAME", file=sys.stderr)
        sys.exit(2)
    names = [args.config] if single else ALL_CONFIGS
    records, big = [], (None, None)
    for i, name in enumerate(names):
        rec, (wl, W0) = bench_config(name, args, sfb, torch, workloads, traffic_table,
                                     args.cpu_seconds if i == 0 else args.cpu_seconds / 4, extras=single)
        records.append(rec)
        if name == "mlr_large":
            big = (wl, W0)
        else:
            del wl, W0
        print(f"bench.py: {name}: {rec['ms_per_step']:.4f} ms/step (median of {REPEATS}), "
              f"roofline {rec['roofline']['frac']:.3f} of {rec['roofline']['bound']}", file=sys.stderr, flush=True)
    out = dict(records[0])
    if not args.no_floors:
        out["floors"] = measure_floors(sfb, torch, *big)
        out["stream_copy"] = out["floors"]["stream_copy"]
    if not single:
        out["configs"] = records
    print(json.dumps(out))


if __name__ == "__main__":
    main()
