"""The entry point that allocates nothing (sfb_step_noalloc), through the C ABI: same factors, loss
and W as sfb_step, bit for bit (same kernels, only the scratch memory differs), on two calls in a
row, the second on a smaller problem -- the library's scratch array keeps the first call's
contents, and nothing of them may leak into the second."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import alloc_factors, assert_close, to_device

pytestmark = pytest.mark.gpu


def _both(sfb, name, over, dev="cuda:0"):
    wl = workloads.make(name, seed=31, steps=1, pool=1, **over)
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, dtype=wl.dtype, device=dev)
    assert ctx.workspace_bytes() <= 16 << 20
    db, dy = to_device(wl, wl.batch(0), dev)
    out = []
    for call in (ctx.step, ctx.step_noalloc):
        W = torch.from_numpy(wl.W0).to(dev)
        U, V, loss = alloc_factors(wl, dev)
        call(W, db, dy, U, V, wl.eta, loss=loss)
        ctx.sync()
        out.append((W, U, V, loss))
    ctx.close()
    return wl, out


@pytest.mark.parametrize("first,second", [
    (("mlr_medium", dict()), ("mlr_medium", dict(J=200, D=520, P=3, B=24))),            # 8.2 MB of scratch, then 58 KB
    (("dml", dict(J=300, D=1024, P=4, B=64)), ("l2svm", dict(J=68, D=300, P=2, B=9, density=0.06))),
    (("mlr_large", dict(J=1000, D=2048, P=4, B=64)), ("mlr_large", dict(J=300, D=1024, P=4, B=40))),   # bf16: packed factors too
    # padded factor copies and planes of partial sums (few tiles, many pairs) in the scratch, then a whole shape with planes
    (("mlr_tiny", dict(J=10, D=784, P=12, B=100)), ("mlr_tiny", dict(J=64, D=128, P=16, B=128))),
])
def test_noalloc_step_equals_step_on_two_calls_in_a_row(first, second):
    import paper_1511_08486_amd as sfb
    assert torch.cuda.is_available()
    for name, over in (first, second):
        wl, (want, got) = _both(sfb, name, over)
        for w, g, what in zip(want, got, ("W", "U", "V", "loss")):
            assert torch.equal(w, g), f"{name} {over}: {what} differs between sfb_step and sfb_step_noalloc"
        # and both are the oracle's step (the same bar as every other parity test)
        tol = 2e-2 if wl.dtype == "bf16" else 1e-4
        Uo, Vo, Wo, fo = oracle.step(wl.model, wl.W0, wl.batch(0), wl.P, wl.B, wl.eta)
        assert_close(got[0].cpu().numpy(), Wo, tol, "W")
        assert_close(got[1].cpu().numpy(), Uo, tol, "U")
        assert_close(got[2].float().cpu().numpy(), Vo, tol, "V")
        assert_close(got[3].cpu().numpy(), fo, tol, "loss")


def test_noalloc_step_with_a_dead_worker_and_no_registered_workspace_interference():
    """The registered workspace is neither needed nor touched: it is filled with NaN before the call
    and still all NaN afterwards; a dead worker's mask works as in sfb_step."""
    import paper_1511_08486_amd as sfb
    dev = "cuda:0"
    wl = workloads.make("mlr_medium", seed=32, J=260, D=512, P=4, B=32, steps=1, pool=1)
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, device=dev)
    db, dy = to_device(wl, wl.batch(0), dev)
    ws = ctx._ws.view(torch.float32)
    ws.fill_(float("nan"))
    W = torch.from_numpy(wl.W0).to(dev)
    U, V, loss = alloc_factors(wl, dev)
    active = [1, 1, 0, 1]
    ctx.step_noalloc(W, db, dy, U, V, wl.eta, loss=loss, active=active)
    ctx.sync()
    assert bool(torch.isnan(ws).all())
    _, _, Wo, _ = oracle.step(wl.model, wl.W0, wl.batch(0), wl.P, wl.B, wl.eta, active=active)
    assert_close(W.cpu().numpy(), Wo, 1e-4, "W, dead worker")
    ctx.close()
