"""Helpers for the GPU parity tests: upload a workload, run the HIP path through the
C ABI binding, run the oracle on the same arrays, compare element by element."""
import numpy as np
import torch

import oracle
import workloads


def close(got, want, tol, floor=1e-2):
    """|got - want| <= tol * max(|want|, floor * max|want|), element by element.
    Returns (ok, worst ratio of error to allowance)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if want.size == 0:
        return True, 0.0
    scale = np.abs(want).max()
    allow = tol * np.maximum(np.abs(want), floor * scale)
    allow = np.maximum(allow, 1e-30)
    err = np.abs(got - want)
    if not np.all(np.isfinite(got)):
        return False, float("inf")
    worst = float((err / allow).max())
    return worst <= 1.0, worst


def assert_close(got, want, tol, what):
    ok, worst = close(got, want, tol)
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


def run_chain(wl, steps, tol, check_every=1, dml_guard=2e-5, pad=0, plan=None):
    """Runs `steps` SFB steps on the GPU and in the oracle from the same W0 and batches and
    compares U, V, W and the per-sample loss after every step."""
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
    worst = {"U": 0.0, "V": 0.0, "W": 0.0, "loss": 0.0}
    for t in range(steps):
        b = wl.batch(t)
        db, dy = dev_batches[t % len(dev_batches)]
        ctx.step(Wg, db, dy, U, V, wl.eta, loss=loss)
        ctx.sync()
        Uo, Vo, Wo_new, fo = oracle.step(wl.model, Wo, b, wl.P, wl.B, wl.eta)
        if wl.model == "dml":
            margin = oracle.dml_margin_distance(oracle.scores(Wo, Vo), b["y"])
            assert margin > dml_guard, f"step {t}: a dissimilar pair sits {margin:.2e} from the hinge kink"
        Wo = Wo_new
        if t % check_every == 0 or t == steps - 1:
            worst["U"] = max(worst["U"], assert_close(U.cpu().numpy(), Uo, tol, f"U step {t}"))
            worst["V"] = max(worst["V"], assert_close(V.float().cpu().numpy(), Vo, tol, f"V step {t}"))
            worst["W"] = max(worst["W"], assert_close(Wg.cpu().numpy(), Wo, tol, f"W step {t}"))
            worst["loss"] = max(worst["loss"], assert_close(loss.cpu().numpy(), fo, tol, f"loss step {t}"))
    ctx.close()
    return worst
