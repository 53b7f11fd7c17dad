"""Helpers for the GPU parity tests: upload a workload, run the HIP path through the
C ABI binding, run the oracle on the same arrays, compare element by element."""
import numpy as np
import torch

import oracle
import workloads


def close(got, want, tol, floor=1e-2, terms=None):
    """|got - want| <= tol * max(|want|, floor * max|want|), element by element.
    With `terms` (same shape: for a sum, the sum of the magnitudes of its terms) the allowance is
    tol * max(|want|, floor * max|want|, terms): an entry whose terms cancel is held to the size of
    what was added up, the componentwise bound of a rounded inner product.
    Returns (ok, worst ratio of error to allowance)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if want.size == 0:
        return True, 0.0
    scale = np.abs(want).max()
    allow = np.maximum(np.abs(want), floor * scale)
    if terms is not None:
        allow = np.maximum(allow, np.asarray(terms, dtype=np.float64))
    allow = np.maximum(tol * allow, 1e-30)
    err = np.abs(got - want)
    if not np.all(np.isfinite(got)):
        return False, float("inf")
    worst = float((err / allow).max())
    return worst <= 1.0, worst


def assert_close(got, want, tol, what, terms=None):
    ok, worst = close(got, want, tol, terms=terms)
    assert ok, f"{what}: error is {worst:.3g} x the allowance (tol {tol})"
    return worst


def to_device(wl, batch, dev="cuda:0"):
    """torch device tensors for one batch (storage type per workload) + label tensor."""
    import paper_1511_08486_amd as sfb
    y = torch.from_numpy(np.ascontiguousarray(batch["y"], dtype=np.int32)).to(dev)
    if wl.model == "mlr":
        a = torch.from_numpy(batch["A"])
        if wl.dtype == "bf16":
            a = a.to(torch.bfloat16)          # exact: the values are bf16-representable
        return sfb.SfbBatch(a=a.to(dev)), y
    if wl.model == "dml":
        return sfb.SfbBatch(a=torch.from_numpy(batch["X"]).to(dev), a2=torch.from_numpy(batch["Y"]).to(dev)), y
    return sfb.SfbBatch(rowptr=torch.from_numpy(batch["rowptr"]).to(dev),
                        col=torch.from_numpy(batch["col"]).to(dev),
                        val=torch.from_numpy(batch["val"]).to(dev)), y


def alloc_factors(wl, dev="cuda:0", pad_u=0, pad_v=0, fill=float("nan")):
    vdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    U = torch.full((wl.N, wl.J + pad_u), fill, dtype=torch.float32, device=dev)[:, :wl.J]
    V = torch.full((wl.N, wl.D + pad_v), fill, dtype=vdt, device=dev)[:, :wl.D]
    loss = torch.full((wl.N,), fill, dtype=torch.float32, device=dev)
    return U, V, loss


def fresh_update(ctx, U, V, eta, like, scale=None, active=None):
    """-eta * scale * U^T V as the library's reconstruction forms it, applied to a zero matrix shaped
    and strided like `like`: the update itself, not hidden behind the much larger entries of W."""
    Z = torch.zeros_like(like._base if like._base is not None else like)
    if like._base is not None:
        Z = Z[:, :like.shape[1]]
    ctx.reconstruct_apply(Z, U, V, eta, scale=scale, active=active)
    ctx.sync()
    return Z


def make_clear_of_kink(name, seed, chain_steps, guard=1e-4, **over):
    """workloads.make(name, seed=s, **over) for the first s >= seed whose metric-learning chain keeps
    every dissimilar pair further than `guard` from the hinge kink |z|^2 = 1 during `chain_steps` oracle steps
    (inside that band an fp32 path may legitimately take the other branch, so such inputs decide
    nothing).  Decided by the oracle alone, on the CPU; other models are returned as they are."""
    for s in range(seed, seed + 64):
        wl = workloads.make(name, seed=s, **over)
        if wl.model != "dml":
            return wl
        W = wl.W0.astype(np.float64)
        clear = True
        for t in range(chain_steps):
            b = wl.batch(t)
            _, Vo, W_new, _ = oracle.step(wl.model, W, b, wl.P, wl.B, wl.eta)
            if oracle.dml_margin_distance(oracle.scores(W, Vo), b["y"]) <= guard:
                clear = False
                break
            W = W_new
        if clear:
            return wl
    raise AssertionError("no seed keeps the chain clear of the hinge kink")


def run_chain(wl, steps, tol, check_every=1, dml_guard=1e-4, pad=0, plan=None, progress=None):
    """Runs `steps` SFB steps on the GPU and in the oracle from the same W0 and batches and
    compares U, V, W, the per-sample loss and the update -eta*dW itself after every checked step.
    (W alone would not pin the reconstruction: one step's update is far below tol * |W| for most
    entries, so the same factors are also applied to a zero matrix and compared with the oracle's
    W_new - W.)  `progress` (optional) is called with a line of text after every step: long chains
    report through it so that a watcher of the run's output sees them advance."""
    import paper_1511_08486_amd as sfb
    dev = "cuda:0"
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, dtype=wl.dtype, device=dev)
    if plan:
        ctx.set_plan(**plan)
    Wg = torch.empty((wl.J, wl.D + pad), dtype=torch.float32, device=dev)[:, :wl.D]
    Wg.copy_(torch.from_numpy(wl.W0))
    U, V, loss = alloc_factors(wl, dev, pad_u=pad, pad_v=pad)
    Wo = wl.W0.astype(np.float64)
    dev_batches = [to_device(wl, b, dev) for b in wl.batches]
    worst = {"U": 0.0, "V": 0.0, "W": 0.0, "loss": 0.0, "dW": 0.0}
    for t in range(steps):
        b = wl.batch(t)
        db, dy = dev_batches[t % len(dev_batches)]
        ctx.step(Wg, db, dy, U, V, wl.eta, loss=loss)
        ctx.sync()
        Uo, Vo, Wo_new, fo = oracle.step(wl.model, Wo, b, wl.P, wl.B, wl.eta)
        if wl.model == "dml":
            margin = oracle.dml_margin_distance(oracle.scores(Wo, Vo), b["y"])
            assert margin > dml_guard, f"step {t}: a dissimilar pair sits {margin:.2e} from the hinge kink"
        checked = t % check_every == 0 or t == steps - 1
        upd_o = (Wo_new - Wo) if checked else None          # -eta * dW of the oracle
        Wo = Wo_new
        if checked:
            worst["U"] = max(worst["U"], assert_close(U.cpu().numpy(), Uo, tol, f"U step {t}"))
            worst["V"] = max(worst["V"], assert_close(V.float().cpu().numpy(), Vo, tol, f"V step {t}"))
            worst["W"] = max(worst["W"], assert_close(Wg.cpu().numpy(), Wo, tol, f"W step {t}"))
            worst["loss"] = max(worst["loss"], assert_close(loss.cpu().numpy(), fo, tol, f"loss step {t}"))
            upd_g = fresh_update(ctx, U, V, wl.eta, Wg)
            # sum of the magnitudes of every entry's terms, eta/B * sum_i |u_i| |v_i|^T, from the oracle's factors
            mag = wl.eta * oracle.delta_w(np.abs(Uo), np.abs(Vo), wl.P, wl.B)
            worst["dW"] = max(worst["dW"], assert_close(upd_g.cpu().numpy(), upd_o, tol, f"-eta*dW step {t}", terms=mag))
            del upd_g, upd_o, mag
        if progress:
            progress(f"{wl.name}: step {t + 1}/{steps}" + (f" checked, worst error/allowance so far {worst}" if checked else ""))
    ctx.close()
    return worst


def run_chain_pipelined(wl, steps, tol, check_every=1, plan=None, progress=None, active=None):
    """The same `steps` iterations as run_chain, regrouped the way sfb_step_pipelined runs them: factors of
    batch 0, then steps - 1 calls that apply the pending factors and form the next batch's, then the last
    update.  After call t the GPU's W must be the oracle's W after t updates and U, V, loss the oracle's
    factors of batch t at that W; the update a call applies is also compared on its own (the same call on
    a zero matrix, with copies of the pending factors).  `active` masks the workers of every update."""
    import paper_1511_08486_amd as sfb
    dev = "cuda:0"
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, dtype=wl.dtype, device=dev)
    if plan:
        ctx.set_plan(**plan)
    Wg = torch.from_numpy(wl.W0).to(dev)
    U, V, loss = alloc_factors(wl, dev)
    Wo = wl.W0.astype(np.float64)
    dev_batches = [to_device(wl, b, dev) for b in wl.batches]
    worst = {"U": 0.0, "V": 0.0, "W": 0.0, "loss": 0.0, "dW": 0.0}

    def check(t, Uo, Vo, fo, what):
        worst["U"] = max(worst["U"], assert_close(U.cpu().numpy(), Uo, tol, f"U {what}"))
        worst["V"] = max(worst["V"], assert_close(V.float().cpu().numpy(), Vo, tol, f"V {what}"))
        worst["W"] = max(worst["W"], assert_close(Wg.cpu().numpy(), Wo, tol, f"W {what}"))
        worst["loss"] = max(worst["loss"], assert_close(loss.cpu().numpy(), fo, tol, f"loss {what}"))

    db, dy = dev_batches[0]
    ctx.compute_factors(Wg, db, dy, U, V, loss)
    ctx.sync()
    Uo, Vo, fo = oracle.factors(wl.model, Wo, wl.batch(0))
    check(0, Uo, Vo, fo, "before the first update")
    for t in range(1, steps + 1):
        checked = t % check_every == 0 or t >= steps - 1
        W_new = oracle.apply_update(Wo, oracle.delta_w(Uo, Vo, wl.P, wl.B, active), wl.eta)
        if t < steps:
            db, dy = dev_batches[t % len(dev_batches)]
            if checked:
                # the update this call applies, on its own: same call, zero matrix, copies of the pending factors
                Wz, U2, V2 = torch.zeros_like(Wg), U.clone(), V.clone()
                ctx.update_and_next_factors(Wz, U2, V2, db, dy, wl.eta, active=active)
                ctx.sync()
                mag = wl.eta * oracle.delta_w(np.abs(Uo), np.abs(Vo), wl.P, wl.B, active)
                worst["dW"] = max(worst["dW"], assert_close(Wz.cpu().numpy(), W_new - Wo, tol, f"-eta*dW of call {t}", terms=mag))
                del Wz, U2, V2, mag
            ctx.update_and_next_factors(Wg, U, V, db, dy, wl.eta, loss=loss, active=active)
            ctx.sync()
            Wo = W_new
            Uo, Vo, fo = oracle.factors(wl.model, Wo, wl.batch(t))
            if checked:
                check(t, Uo, Vo, fo, f"after call {t}")
        else:
            ctx.reconstruct_apply(Wg, U, V, wl.eta, active=active)
            ctx.sync()
            Wo = W_new
            worst["W"] = max(worst["W"], assert_close(Wg.cpu().numpy(), Wo, tol, "W after the last update"))
        if progress:
            progress(f"{wl.name}: pipelined call {t}/{steps}" + (f" checked, worst error/allowance so far {worst}" if checked else ""))
    info = ctx.pipeline_info()
    ctx.close()
    return worst, info
