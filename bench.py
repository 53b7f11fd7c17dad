#!/usr/bin/env python3
"""Throughput of the SFB hot path on one MI355X.

A "step" is one full bulk-synchronous SFB iteration (scores, factor u, factor v, the
concatenation standing in for the broadcast, reconstruction, W update) over one synthetic
minibatch of P*B samples whose features, labels and W already sit in HBM.

Prints ONE JSON line: whole-job samples/s (= P*B * steps/s), plus
  roofline      the dominant kernel's achieved rate against the MI355X peak that bounds it,
                from HIP events recorded around every launch of a second, instrumented pass
  cpu_baseline  the fp64 numpy oracle timed on this host's cores on the same workload
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3     # MI355X dense fp32 matrix-core peak
PEAK_HBM_GBS = 8000.0
FAMILIES = {0: "scores", 1: "factor u", 2: "reconstruct-apply", 3: "csr densify"}


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


def bench_sdca(args):
    """--config sdca_*: SFB driven by SDCA (Section 2.1) on a fixed synthetic data set.  A "step" is
    one iteration over P*B distinct picked samples: scores, dual update + factors, reconstruction.
    Same JSON keys as the main bench; informational (the headline configs are the SGD ones)."""
    import numpy as np
    import torch

    import __graft_entry__
    __graft_entry__.ensure_built()
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
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", default="mlr_medium")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="oracle timing budget (0 = skip)")
    ap.add_argument("--graph", action="store_true",
                    help="record the pool's steps in a HIP graph and time replays (helps launch-bound tiny configs)")
    ap.add_argument("--plan", default="", help="fwd_bm,fwd_bn,split_k,recon_variant[,fwd_dma] override")
    ap.add_argument("--objective-every", type=int, default=0,
                    help="after the timed run, replay the steps from W0 (untimed) and report the mean per-sample "
                         "loss of the batch of every K-th step against samples processed")
    ap.add_argument("--prox", default="",
                    help="KIND:PARAM (l2sq, l1 or column_ball): after the timed run, also time proximal-SGD "
                         "iterations (the step followed by prox_{eta h}), fused and as two calls; informational")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
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
    dev = "cuda:0"
    wl = workloads.make(args.config)
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, dtype=wl.dtype, device=dev)
    if args.plan:
        vals = [int(x) for x in args.plan.split(",")] + [-1]
        ctx.set_plan(*vals[:5])

    # inputs resident in HBM before anything is timed
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
    W0 = torch.from_numpy(wl.W0).to(dev)
    W = W0.clone()
    U = torch.empty((wl.N, wl.J), dtype=torch.float32, device=dev)
    V = torch.empty((wl.N, wl.D), dtype=vdt, device=dev)

    def run_eager(k):
        for t in range(k):
            b, y = pool[t % len(pool)]
            ctx.step(W, b, y, U, V, wl.eta)

    run = run_eager
    run(args.warmup)
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

        run = run_graph
        args.warmup = max(len(pool), args.warmup // len(pool) * len(pool))
        args.steps = max(len(pool), args.steps // len(pool) * len(pool))
        run(args.warmup)
    torch.cuda.synchronize()
    W.copy_(W0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert bool(torch.isfinite(W).all()), "W is not finite after the timed steps"

    # instrumented pass: same launches (eager), HIP events around each one on the library's stream
    W.copy_(W0)
    ctx.enable_timing(True)
    ctx.reset_timing()
    k2 = min(args.steps, 500)
    run_eager(k2)
    per_kernel = {}
    for fam, name in FAMILIES.items():
        ms, n = ctx.kernel_time_ms(fam)
        if n:
            per_kernel[fam] = (name, ms / n * 1e3, n)       # microseconds per launch
    ctx.enable_timing(False)
    ctx.reset_timing()

    # yardstick: a plain streaming copy, large enough (256 MiB each way) that launch and
    # host overheads vanish; it is also the known-size kernel the HBM counters are scaled by
    big = torch.empty(2, 64 * 1024 * 1024, dtype=torch.float32, device=dev)
    big[0].fill_(1.0)
    ctx.stream_copy(big[1], big[0])
    ctx.enable_timing(True)
    ctx.reset_timing()
    n_other = ctx.kernel_time_ms(3)[1]
    for _ in range(10):
        ctx.stream_copy(big[1], big[0])
    ms, n = ctx.kernel_time_ms(3)
    copy_bytes = 2.0 * big[0].numel() * 4
    copy_gbs = copy_bytes / (ms / n * 1e-3) / 1e9 if n and not n_other else None
    ctx.enable_timing(False)
    ctx.reset_timing()
    del big

    # Roofline of the dominant contraction.  fp32 workloads: both contractions are bound by the
    # fp32 matrix cores (2*N*J*D flops per launch).  bf16 workload: both are bound by streaming W
    # through HBM; the algorithmic bytes per launch are W once (scores) / twice (reconstruct)
    # plus the factor operands.
    S = ctx.plan_info()["fwd_split_k"]
    flops = 2.0 * wl.N * wl.J * wl.D
    cands = [f for f in per_kernel if f in (0, 2)]
    if wl.model == "l2svm" and 0 in cands:
        cands.remove(0)                                     # CSR scores: a gather kernel, no dense roofline
    dom = max(cands, key=lambda f: per_kernel[f][1])
    us = per_kernel[dom][1]
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(f"{args.config}:{dom}")
    if wl.dtype == "bf16":
        wbytes = 4.0 * wl.J * wl.D
        if dom == 0:
            alg = wbytes + 2.0 * wl.N * wl.D * 2 + S * 4.0 * wl.N * wl.J
        else:
            alg = 2.0 * wbytes + 2.0 * wl.N * (wl.J + wl.D)
        achieved = alg / (us * 1e-6) / 1e9
        roofline = {"bound": "hbm", "kernel": per_kernel[dom][0], "achieved": achieved, "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS, "traffic": traffic,
                    "algorithmic_bytes": alg, "us_per_launch": us}
    else:
        achieved = flops / (us * 1e-6) / 1e12
        roofline = {"bound": "mfma", "kernel": per_kernel[dom][0], "achieved": achieved,
                    "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_FP32_MFMA_TFLOPS,
                    "traffic": traffic, "algorithmic_flops": flops, "us_per_launch": us}
    roofline["kernels_us"] = {v[0]: round(v[1], 2) for v in per_kernel.values()}

    out = {
        "metric": "sfb_samples_per_sec", "value": wl.N * args.steps / elapsed, "unit": "samples/s",
        "steps_per_sec": args.steps / elapsed,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if wl.dtype == "f32" else "bf16 features, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.model} J={wl.J} D={wl.D} P={wl.P} B={wl.B} eta={wl.eta}",
                   "plan": ctx.plan_info(), "launch": "hip graph replay" if args.graph else "eager"},
        "roofline": roofline,
        "stream_copy": {"GB/s": copy_gbs, "bytes_per_launch": copy_bytes,
                        "note": "plain float4 copy kernel, 256 MiB read + 256 MiB written per launch"},
    }
    if wl.dtype == "f32" and not args.plan and not args.graph:
        # informational second line: the same steps with both contractions taken as split-bf16 products on the
        # bf16 matrix cores (opt-in plan bits 2 and 3; fp32-level error, same parity tests).  Not the headline.
        alt = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, dtype=wl.dtype, device=dev)
        alt.set_plan(fwd_dma=13)
        W.copy_(W0)
        for t in range(args.warmup):
            b, y = pool[t % len(pool)]
            alt.step(W, b, y, U, V, wl.eta)
        torch.cuda.synchronize()
        W.copy_(W0)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for t in range(args.steps):
            b, y = pool[t % len(pool)]
            alt.step(W, b, y, U, V, wl.eta)
        torch.cuda.synchronize()
        el = time.perf_counter() - t1
        assert bool(torch.isfinite(W).all()), "W is not finite after the split-bf16 steps"
        out["alt_plan"] = {"name": "split-bf16 contractions (sfb_set_plan fwd_dma=13)", "value": wl.N * args.steps / el,
                           "unit": "samples/s", "ms_per_step": el / args.steps * 1e3,
                           "note": "fp32 operands split exactly into three bf16 terms, six term products per product"}
        alt.close()
    if args.prox:
        # informational: proximal SGD (Section 2.1), the step followed by the proximal operator of h
        kind, param = args.prox.split(":")
        param = float(param)

        def timed(fn):
            W.copy_(W0)
            for t in range(args.warmup):
                fn(*pool[t % len(pool)])
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for t in range(args.steps):
                fn(*pool[t % len(pool)])
            torch.cuda.synchronize()
            return (time.perf_counter() - t1) / args.steps * 1e3

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
        for t in range(args.steps):
            b, y = pool[t % len(pool)]
            ctx.step(W, b, y, U, V, wl.eta, loss=loss)
            if t % args.objective_every == 0 or t == args.steps - 1:
                curve.append([wl.N * t, float(loss.double().mean().item())])
        out["objective_curve"] = {"unit": "mean per-sample loss of the step's batch, before its update",
                                  "samples_vs_loss": curve}
    if args.cpu_seconds > 0:
        out["cpu_baseline"] = cpu_baseline(wl, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
