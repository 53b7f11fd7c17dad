"""sfb_step_pipelined: the update of iteration t and the factors of iteration t+1 in one call (for
bf16 contexts of the covered shapes: one kernel that passes over W once).  Chains of calls against
the fp64 oracle, element by element, to the bf16-input bar (2e-2); fall-back shapes to their own bar."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import alloc_factors, assert_close, make_clear_of_kink, run_chain_pipelined, to_device

pytestmark = pytest.mark.gpu

TOL32 = 1e-4
TOLBF = 2e-2


@pytest.mark.parametrize("J,D,P,B,active", [
    (300, 1024, 4, 32, None),          # N = 128: 3 bands (the last 44 rows), column slices of 8 tiles
    (130, 512, 8, 32, None),           # N = 256: second band has 2 rows
    (1000, 2048, 16, 32, None),        # N = 512: the benchmark's worker layout
    (128, 32, 4, 32, None),            # one band, one tile
    (260, 1056, 16, 32, [1] * 5 + [0] + [1] * 10),   # a dead worker's pending factors contribute nothing; 33 tiles
    (33000, 256, 4, 32, None),         # 258 bands: more workgroups than compute units, the launch takes two rounds
])
def test_fused_chain_matches_the_oracle(J, D, P, B, active):
    wl = workloads.make("mlr_large", seed=J + D, J=J, D=D, P=P, B=B, steps=4, pool=3)
    worst, info = run_chain_pipelined(wl, 4, TOLBF, active=active)
    assert info["fused"] and info["grid"] >= 1
    print(f"fused chain J={J} D={D} N={P * B}: worst error/allowance {worst}, {info}")


@pytest.mark.timeout(1500)
def test_mlr_large_twenty_pipelined_steps(capsys):
    """The largest configuration through the one-pass kernel, its whole chain of 20 iterations."""
    wl = workloads.make("mlr_large")

    def say(line):
        with capsys.disabled():
            print(line, flush=True)
    worst, info = run_chain_pipelined(wl, wl.steps, TOLBF, check_every=4, progress=say)
    assert info["fused"]
    print("mlr_large pipelined worst error/allowance", worst, info)


@pytest.mark.parametrize("name,over,tol", [
    ("mlr_large", dict(J=300, D=1004, P=3, B=30), TOLBF),       # bf16, but neither N nor D is what the fused kernel takes
    ("mlr_medium", dict(J=200, D=512, P=4, B=32), TOL32),       # fp32 features
    ("dml", dict(J=64, D=256, P=2, B=64, seed=3), TOL32),
    ("l2svm", dict(J=64, D=512, P=2, B=32, density=0.04), TOL32),
])
def test_shapes_the_fused_kernel_does_not_take_run_the_two_passes(name, over, tol):
    seed = over.pop("seed", 12)
    wl = make_clear_of_kink(name, seed, 3, steps=3, pool=3, **over)
    worst, info = run_chain_pipelined(wl, 3, tol)
    assert not info["fused"]


def test_fused_and_two_pass_forms_agree_and_the_switch_turns_the_fused_kernel_off():
    wl = workloads.make("mlr_large", seed=5, J=520, D=1024, P=8, B=32, steps=3, pool=3)
    got = {}
    for name, plan in (("fused", None), ("two passes", dict(fwd_dma=1 | 16))):
        worst, info = run_chain_pipelined(wl, 3, TOLBF, plan=plan)
        assert info["fused"] == (plan is None)
        got[name] = worst
    print(got)


def test_fused_call_is_deterministic_and_misaligned_operands_fall_back():
    import paper_1511_08486_amd as sfb
    dev = "cuda:0"
    wl = workloads.make("mlr_large", seed=6, J=260, D=512, P=4, B=32, steps=2, pool=2)
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, dtype="bf16", device=dev)
    (b0, y0), (b1, y1) = [to_device(wl, b, dev) for b in wl.batches]
    res = []
    for _ in range(2):
        W = torch.from_numpy(wl.W0).to(dev)
        U, V, loss = alloc_factors(wl, dev)
        ctx.compute_factors(W, b0, y0, U, V, loss)
        ctx.update_and_next_factors(W, U, V, b1, y1, wl.eta, loss=loss)
        ctx.sync()
        res.append((W.clone(), U.clone(), V.clone(), loss.clone()))
    for a, b in zip(*res):
        assert torch.equal(a, b)
    # W one element off 16-byte alignment: the call must take the two-pass form and still be right
    buf = torch.zeros((wl.J, wl.D + 8), dtype=torch.float32, device=dev)
    Wm = buf[:, 1:wl.D + 1]
    Wm.copy_(torch.from_numpy(wl.W0))
    U, V, loss = alloc_factors(wl, dev)
    ctx.compute_factors(Wm, b0, y0, U, V, loss)
    ctx.update_and_next_factors(Wm, U, V, b1, y1, wl.eta, loss=loss)
    ctx.sync()
    assert_close(Wm.cpu().numpy(), res[0][0].cpu().numpy(), 1e-5, "W, misaligned, against the fused result")
    assert_close(U.cpu().numpy(), res[0][1].cpu().numpy(), 1e-3, "U, misaligned, against the fused result")
    assert float(buf[:, 0].abs().max()) == 0.0 and float(buf[:, wl.D + 1:].abs().max()) == 0.0
    ctx.close()


def test_probes_leave_w_as_it_was_and_refuse_bad_arguments():
    """The measurement aids run on real buffers: the read-modify-write probe adds zero (W keeps its bits), the
    stream probe only reads; wrong parameters are refused with a status, nothing is launched."""
    import paper_1511_08486_amd as sfb
    dev = "cuda:0"
    ctx = sfb.Sfb("mlr", 520, 1024, 4, 32, dtype="bf16", device=dev)
    W = torch.randn((520, 1024), device=dev)
    keep = W.clone()
    for kind, param in (("w_stream", 1), ("w_stream", 2), ("w_rmw", 1), ("mfma_f32", 1), ("mfma_bf16", 2), ("empty", 1),
                        ("fused_traffic", 0)):
        ctx.probe(kind, W, param)
    ctx.sync()
    assert torch.equal(W, keep)
    for kind, param in (("w_stream", 3), ("mfma_f32", 0), ("mfma_bf16", 5)):
        with pytest.raises(sfb.SfbError):
            ctx.probe(kind, W, param)
    with pytest.raises(sfb.SfbError):
        ctx.probe("w_rmw", None)
    ctx.close()
    # a ragged last band (J = 300: 44 rows of the third band) and a short matrix; a shape the one-pass kernel
    # does not take is refused
    for J, D, P, B in ((300, 1024, 2, 64), (40, 64, 4, 64)):
        ctx = sfb.Sfb("mlr", J, D, P, B, dtype="bf16", device=dev)
        W = torch.randn((J, D), device=dev)
        keep = W.clone()
        ctx.probe("fused_traffic", W)
        ctx.sync()
        assert torch.equal(W, keep)
        ctx.close()
    ctx = sfb.Sfb("mlr", 300, 1000, 2, 64, dtype="bf16", device=dev)
    with pytest.raises(sfb.SfbError):
        ctx.probe("fused_traffic", torch.zeros((300, 1000), device=dev))
    ctx.close()
