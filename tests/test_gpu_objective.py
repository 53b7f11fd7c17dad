"""GPU checks of the objective (Section 2, problem (P)) along a short SFB run, and of the
statement behind the whole method (Section 3): applying the received sufficient factors is
the same update as a step along the full-matrix minibatch gradient.

The full-matrix gradients below are written out from the loss definitions in matrix form
(softmax / hinge masks, then one dense product), a different route from the oracle's
per-sample factors; both are compared with what the HIP path leaves in W.
"""
import numpy as np
import pytest
import torch
from scipy.special import softmax

import oracle
import workloads
from gpu_util import alloc_factors, assert_close, to_device

pytestmark = pytest.mark.gpu

TOL32 = 1e-4


@pytest.fixture(scope="module")
def sfb():
    import paper_1511_08486_amd as m
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return m


def full_matrix_gradient(wl, W, batch):
    """dF/dW for F(W) = sum_p (1/B) sum_i f_i(W a_i), as one [J, D] matrix, with no factors."""
    W = W.astype(np.float64)
    if wl.model == "mlr":
        A = batch["A"].astype(np.float64)
        S = softmax(A @ W.T, axis=1)
        S[np.arange(wl.N), batch["y"]] -= 1.0
        return S.T @ A / wl.B
    if wl.model == "dml":
        Dm = batch["X"].astype(np.float64) - batch["Y"].astype(np.float64)
        Z = Dm @ W.T
        sq = (Z * Z).sum(axis=1)
        coef = np.where(batch["y"] == 1, 2.0, np.where(sq < 1.0, -2.0, 0.0))
        return (coef[:, None] * Z).T @ Dm / wl.B
    A = oracle.csr_to_dense(batch["rowptr"], batch["col"], batch["val"], wl.D)
    Z = A @ W.T
    T = -np.ones_like(Z)
    T[np.arange(wl.N), batch["y"]] = 1.0
    G = -2.0 * T * np.maximum(0.0, 1.0 - T * Z)
    return G.T @ A / wl.B


@pytest.mark.parametrize("name,override", [
    ("mlr_tiny", {}),
    ("mlr_tiny", dict(J=130, D=260, P=3, B=40)),
    ("dml", dict(J=48, D=200, P=2, B=24)),
    ("l2svm", dict(J=70, D=256, P=2, B=20, density=0.05)),
])
def test_factor_step_is_the_full_matrix_gradient_step(sfb, name, override):
    """W after sfb_step == W0 - eta * (full-matrix minibatch gradient at W0)."""
    dev = "cuda:0"
    wl = workloads.make(name, seed=11, **override)
    b = wl.batch(0)
    if wl.model == "dml":
        # keep every dissimilar pair away from the hinge kink, where the fp32 and fp64 sides may pick different branches
        assert oracle.dml_margin_distance(oracle.scores(wl.W0.astype(np.float64),
                                                        oracle.dense_features(wl.model, b)), b["y"]) > 2e-5
    want = wl.W0.astype(np.float64) - wl.eta * full_matrix_gradient(wl, wl.W0, b)
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, dtype=wl.dtype, device=dev)
    W = torch.from_numpy(wl.W0).to(dev)
    db, dy = to_device(wl, b, dev)
    U, V, _ = alloc_factors(wl, dev)
    ctx.step(W, db, dy, U, V, wl.eta)
    ctx.sync()
    assert_close(W.cpu().numpy(), want, TOL32, f"{name}: W after one step vs the full-matrix gradient step")
    ctx.close()


@pytest.mark.parametrize("name,steps", [("mlr_medium", 60), ("dml", 20), ("l2svm", 20)])
def test_objective_along_a_run(sfb, name, steps):
    """Objective vs samples on synthetic data: the per-sample losses the factor kernel emits add
    up to the oracle's F(W_t) on the batch of step t, and F on a held-fixed batch goes down."""
    dev = "cuda:0"
    wl = workloads.make(name, seed=1 if name == "dml" else 0)   # dml seed: no pair near the hinge kink
    ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, dtype=wl.dtype, device=dev)
    W = torch.from_numpy(wl.W0).to(dev)
    dev_batches = [to_device(wl, b, dev) for b in wl.batches]
    U, V, loss = alloc_factors(wl, dev)

    def objective_on_batch0():
        ctx.compute_factors(W, dev_batches[0][0], dev_batches[0][1], U, V, loss)
        ctx.sync()
        return float(loss.double().sum().item()) / wl.B

    f_start = objective_on_batch0()
    want_start = oracle.objective(wl.model, wl.W0.astype(np.float64), wl.batch(0), wl.P, wl.B)
    assert abs(f_start - want_start) <= TOL32 * abs(want_start), (f_start, want_start)
    curve = []
    Wo = wl.W0.astype(np.float64)
    for t in range(steps):
        db, dy = dev_batches[t % len(dev_batches)]
        ctx.step(W, db, dy, U, V, wl.eta, loss=loss)
        ctx.sync()
        got = float(loss.double().sum().item()) / wl.B            # F(W_t) on batch t, from the HIP path
        want = oracle.objective(wl.model, Wo, wl.batch(t), wl.P, wl.B)
        assert abs(got - want) <= 5 * TOL32 * abs(want), f"step {t}: objective {got} vs oracle {want}"
        curve.append(got)
        _, _, Wo, _ = oracle.step(wl.model, Wo, wl.batch(t), wl.P, wl.B, wl.eta)
    f_end = objective_on_batch0()
    print(f"{name}: F(batch 0) {f_start:.6g} -> {f_end:.6g} after {steps} steps ({wl.N * steps} samples)")
    assert f_end < f_start, "the objective on a fixed batch did not decrease"
    if wl.model == "mlr":
        # convex loss, small step: the same batch revisited (the pool cycles) is lower every time round
        pool = len(dev_batches)
        for t in range(pool, steps):
            assert curve[t] < curve[t - pool], f"objective on batch {t % pool} rose between step {t - pool} and {t}"
    ctx.close()
