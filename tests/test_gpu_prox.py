"""GPU parity of the proximal step (Section 2.1: W <- prox_{eta h}(W) after the update) against
oracle/prox_oracle.py, through the C ABI, alone and chained after SFB steps."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import alloc_factors, assert_close, to_device
from oracle.prox_oracle import prox

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def sfb():
    import paper_1511_08486_amd as m
    return m


def device_w(W0, pad):
    J, D = W0.shape
    W = torch.full((J, D + pad), float("nan"), dtype=torch.float32, device=DEV)[:, :D]
    W.copy_(torch.from_numpy(W0))
    return W


def column_scaled(rng, J, D, radius):
    """W whose column norms straddle the radius: about half inside the ball, half outside."""
    W = rng.standard_normal((J, D))
    W *= radius * rng.uniform(0.3, 1.7, size=D) / np.sqrt((W * W).sum(0))
    return W.astype(np.float32)


SHAPES = [(10, 100, 0), (37, 203, 3), (129, 1030, 0), (1000, 4096, 0), (5, 4100, 1), (2600, 64, 0)]


@pytest.mark.parametrize("J,D,pad", SHAPES)
@pytest.mark.parametrize("kind,eta,param", [("none", 0.3, 0.5), ("l2sq", 0.1, 0.7), ("l1", 0.5, 0.2),
                                            ("column_ball", 0.1, 1.0)])
def test_prox_matches_the_oracle(sfb, J, D, pad, kind, eta, param):
    rng = np.random.default_rng(J * 7919 + D)
    W0 = column_scaled(rng, J, D, 1.0) if kind == "column_ball" else (0.2 * rng.standard_normal((J, D))).astype(np.float32)
    ctx = sfb.Sfb("mlr", J, D, 2, 4, device=DEV)
    W = device_w(W0, pad)
    ctx.prox(W, kind, eta, param)
    ctx.sync()
    want = prox(kind, W0, eta, param)
    got = W.cpu().numpy()
    assert_close(got, want, 1e-4, f"{kind} {J}x{D}")
    if kind == "none":
        assert np.array_equal(got, W0)
    if kind == "l1":
        # the dead zone is decided on the same fp32 inputs: zeros agree except within rounding of the threshold
        edge = np.abs(np.abs(W0.astype(np.float64)) - eta * param) < 1e-6
        assert np.array_equal((got == 0)[~edge], (want == 0)[~edge])
    if kind == "column_ball":
        inside = np.sqrt((W0.astype(np.float64) ** 2).sum(0)) < param * (1 - 1e-5)
        assert inside.any() and (~inside).any()
        assert np.array_equal(got[:, inside], W0[:, inside])          # untouched, bit for bit
        assert np.sqrt((got.astype(np.float64) ** 2).sum(0)).max() <= param * (1 + 1e-5)
        if pad:
            assert torch.isnan(W.as_strided((J, pad), (D + pad, 1), D)).all()   # padding never written
    ctx.close()


def test_column_ball_twice_is_idempotent_and_all_inside_skips_the_second_pass(sfb):
    rng = np.random.default_rng(3)
    W0 = column_scaled(rng, 300, 2048, 0.5)
    ctx = sfb.Sfb("mlr", 300, 2048, 2, 4, device=DEV)
    W = device_w(W0, 0)
    ctx.prox(W, "column_ball", 0.0, 0.5)
    ctx.sync()
    once = W.clone()
    ctx.prox(W, "column_ball", 0.0, 0.5 * (1 + 1e-5))
    ctx.sync()
    assert torch.equal(W, once)
    ctx.close()


@pytest.mark.parametrize("kind,param", [("l2sq", 0.05), ("l1", 1e-3), ("column_ball", 1.5)])
def test_proximal_sgd_chain(sfb, kind, param):
    """Proximal SGD as Section 2.1 states it: the SFB step, then the proximal operator, five times."""
    wl = workloads.make("mlr_tiny", seed=4, J=24, D=136, P=3, B=8)
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, device=DEV)
    W = device_w(wl.W0, 0)
    U, V, loss = alloc_factors(wl, DEV)
    Wo = wl.W0.astype(np.float64)
    for t in range(5):
        db, dy = to_device(wl, wl.batch(t), DEV)
        ctx.step(W, db, dy, U, V, wl.eta)
        ctx.prox(W, kind, wl.eta, param)
        ctx.sync()
        _, _, Wo, _ = oracle.step(wl.model, Wo, wl.batch(t), wl.P, wl.B, wl.eta)
        Wo = prox(kind, Wo, wl.eta, param)
        assert_close(W.cpu().numpy(), Wo, 1e-4, f"W after step {t} + {kind}")
    ctx.close()


def test_full_size_columns_sampled(sfb):
    """mlr_large's W (10000 x 21504, 860 MB): the column projection checked on sampled columns,
    which the oracle computes one by one."""
    J, D = 10000, 21504
    g = torch.Generator(device=DEV)
    g.manual_seed(5)
    W = torch.randn((J, D), generator=g, device=DEV, dtype=torch.float32)
    W.mul_(0.01 * (0.5 + torch.arange(D, device=DEV, dtype=torch.float32) % 3))       # norms 0.5, 1.5, 2.5
    cols = np.random.default_rng(6).choice(D, size=48, replace=False)
    before = W[:, cols].cpu().numpy()
    ctx = sfb.Sfb("mlr", J, D, 2, 4, device=DEV)
    ctx.prox(W, "column_ball", 0.1, 1.0)
    ctx.sync()
    assert_close(W[:, cols].cpu().numpy(), prox("column_ball", before, 0.1, 1.0), 1e-4, "sampled columns")
    norms = torch.linalg.vector_norm(W.double(), dim=0)
    assert float(norms.max()) <= 1.0 + 1e-5
    ctx.close()


FUSED_CASES = [
    ("mlr_medium", {}, None),                                            # LDS-DMA fp32 kernels
    ("mlr_tiny", dict(J=37, D=203, P=3, B=5), None),                     # register-staged fp32 kernel, ragged
    ("mlr_medium", dict(J=520, D=1024, P=4, B=48), dict(fwd_dma=13)),    # split-bf16 contractions
    ("mlr_large", dict(J=300, D=1024, P=4, B=40), None),                 # bf16 features: bf16 matrix-core kernels
    ("dml", dict(J=72, D=256, P=2, B=32), None),
    ("l2svm", dict(J=64, D=512, P=2, B=16, density=0.05), None),
]


@pytest.mark.parametrize("name,override,plan", FUSED_CASES)
@pytest.mark.parametrize("kind,param", [("l2sq", 0.05), ("l1", 2e-3), ("column_ball", 1.2), ("none", 0.0)])
def test_step_prox_is_step_then_prox_bit_for_bit_and_matches_the_oracle(sfb, name, override, plan, kind, param):
    wl = workloads.make(name, seed=7, **override)
    tol = 2e-2 if wl.dtype == "bf16" else 1e-4
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, dtype=wl.dtype, device=DEV)
    if plan:
        ctx.set_plan(**plan)
    Wa, Wb = device_w(wl.W0, 0), device_w(wl.W0, 0)
    U, V, loss = alloc_factors(wl, DEV)
    Wo = wl.W0.astype(np.float64)
    for t in range(3):
        db, dy = to_device(wl, wl.batch(t), DEV)
        active = [1, 0] + [1] * (wl.P - 2) if (t == 1 and wl.P >= 2) else None      # one dead worker once
        ctx.step_prox(Wa, db, dy, U, V, wl.eta, kind, param, active=active)
        ctx.step(Wb, db, dy, U, V, wl.eta, active=active)
        ctx.prox(Wb, kind, wl.eta, param)
        ctx.sync()
        assert torch.equal(Wa, Wb), f"step {t}: fused and separate proximal steps differ"
        _, _, Wo, _ = oracle.step(wl.model, Wo, wl.batch(t), wl.P, wl.B, wl.eta, active=active)
        Wo = prox(kind, Wo, wl.eta, param)
        assert_close(Wa.cpu().numpy(), Wo, tol, f"W after step {t} + {kind}")
    # the two-call form of the same iteration
    db, dy = to_device(wl, wl.batch(3), DEV)
    ctx.compute_factors(Wa, db, dy, U, V)
    ctx.reconstruct_apply_prox(Wa, U, V, wl.eta, kind, param)
    ctx.step_prox(Wb, db, dy, U, V, wl.eta, kind, param)
    ctx.sync()
    assert torch.equal(Wa, Wb)
    ctx.close()
