"""Pins for the SDCA oracle (oracle/sdca_oracle.py), none of which re-types its formulas:
a schedule worked by hand (tests/golden/sdca_hand_example.json), the conjugate function
against its definition as a supremum, the primal-dual link rebuilt from the dual vectors,
weak duality and monotone descent of problem (D), the exact one-coordinate minimiser found
numerically, convergence to the minimiser that two independent libraries find for the primal
problem, and planted mistakes that these must catch."""
import json
import os

import numpy as np
import pytest
import scipy.optimize
import torch

import workloads
from oracle.sdca_oracle import SdcaMlrOracle, mlr_conjugate, safe_fraction

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sdca_hand_example.json")


def small_problem(seed=0, J=3, D=5, n_data=24, P=2, B=3, lam=0.05, steps=400):
    return workloads.make_sdca("sdca_tiny", seed=seed, J=J, D=D, n_data=n_data, P=P, B=B, lam=lam, steps=steps)


def safe_s(wl, n_picked=None):
    return safe_fraction(wl.lam, wl.n_data, wl.N if n_picked is None else n_picked,
                         float((wl.A.astype(np.float64) ** 2).sum(1).max()))


def run(cls, wl, steps, s):
    o = cls(wl.A, wl.y, wl.J, wl.lam)
    for t in range(steps):
        o.step(wl.pick(t), s)
    return o


def torch_primal(wl, W):
    """The primal objective through torch's own cross-entropy (an independent implementation)."""
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    A = torch.tensor(wl.A, dtype=torch.float64)
    y = torch.tensor(wl.y, dtype=torch.int64)
    val = torch.nn.functional.cross_entropy(A @ Wt.T, y, reduction="mean") + 0.5 * wl.lam * (Wt * Wt).sum()
    (grad,) = torch.autograd.grad(val, Wt)
    return float(val.detach()), grad.numpy()


# ---------------------------------------------------------------------------------------------
def hand_example(cls=SdcaMlrOracle):
    g = json.load(open(GOLDEN))
    o = cls(np.array(g["A"]), np.array(g["y"]), g["J"], g["lam"])
    out = []
    for picked in g["picks"]:
        delta, loss = o.step(picked, g["s"])
        out.append((delta.copy(), loss.copy(), o.W.copy(), o.U.copy()))
    return g, out


def hand_example_matches(cls):
    g, out = hand_example(cls)
    ok = True
    for t, (delta, loss, W, U) in enumerate(out):
        ok &= np.allclose(delta, g["delta_u"][t], rtol=0, atol=1e-14)
        ok &= np.allclose(loss, g["loss"][t], rtol=0, atol=1e-14)
        ok &= np.allclose(W, g["W_after"][t], rtol=0, atol=1e-14)
        ok &= np.allclose(U, g["U_after"][t], rtol=0, atol=1e-14)
    return bool(ok)


def test_hand_worked_iterations():
    assert hand_example_matches(SdcaMlrOracle)


# ---------------------------------------------------------------------------------------------
def test_conjugate_is_the_supremum_of_its_definition():
    """f*(v) = sup_z v.z - f(z), evaluated by a numerical maximisation over z."""
    rng = np.random.default_rng(1)
    for _ in range(6):
        J = int(rng.integers(2, 6))
        label = int(rng.integers(J))
        p = rng.dirichlet(np.ones(J))
        v = p.copy()
        v[label] -= 1.0                                   # p = v + e_y strictly inside the simplex
        res = scipy.optimize.minimize(lambda z: SdcaMlrOracle.loss(z, label) - v @ z, np.zeros(J), method="BFGS",
                                      options={"gtol": 1e-10})
        assert abs(-res.fun - mlr_conjugate(v, label)) < 1e-8
    # outside the simplex the supremum is unbounded
    assert mlr_conjugate(np.array([0.3, 0.3]), 0) == np.inf
    # vertex: 0 log 0 = 0
    assert mlr_conjugate(np.zeros(4), 2) == 0.0


def link_holds(o):
    """W = grad h*(Z) with Z = (1/N) sum u_i a_i^T, rebuilt from the dual vectors alone."""
    Z = o.U.T @ o.A / o.N
    return np.allclose(o.lam * o.W, Z, rtol=1e-12, atol=1e-15) and np.allclose(o.Z, Z, rtol=1e-12, atol=1e-15)


def test_primal_dual_link_survives_every_iteration():
    wl = small_problem(seed=2)
    o = SdcaMlrOracle(wl.A, wl.y, wl.J, wl.lam)
    for t in range(25):
        o.step(wl.pick(t), 0.3)
        assert link_holds(o)
        # dual feasibility: e_y - u_i stays in the simplex
        p = -o.U.copy()
        p[np.arange(o.N), o.y] += 1.0
        assert p.min() > -1e-15 and np.allclose(p.sum(1), 1.0, atol=1e-13)


def descends(cls, wl, steps, s):
    """Weak duality at every iterate and monotone descent of (D); returns the last gap."""
    o = cls(wl.A, wl.y, wl.J, wl.lam)
    prev = o.dual()
    rng = np.random.default_rng(0)
    for t in range(steps):
        o.step(wl.pick(t), s)
        d = o.dual()
        if d > prev + 1e-13:
            return None
        prev = d
        if t % 10 == 0:
            # any primal point bounds any dual point
            if o.primal(rng.standard_normal(o.W.shape)) + d < -1e-12 or o.gap() < -1e-12:
                return None
    return o.gap()


def test_weak_duality_and_monotone_descent_with_the_safe_fraction():
    wl = small_problem(seed=3)
    gap = descends(SdcaMlrOracle, wl, 400, safe_s(wl))
    assert gap is not None and 0 <= gap < 1e-3
    # a full sweep of exact-fraction steps on disjoint single samples also descends
    wl1 = small_problem(seed=4, P=1, B=1)
    assert descends(SdcaMlrOracle, wl1, 200, safe_s(wl1)) is not None


def test_step_lies_between_no_move_and_the_exact_coordinate_minimiser():
    """Section 2.1 asks for the u_i minimising (D) with the others fixed.  That minimiser, found
    numerically over the simplex, must do at least as well as the fractional step, which must
    do at least as well as not moving."""
    wl = small_problem(seed=5, P=1, B=1)
    o = run(SdcaMlrOracle, wl, 30, safe_s(wl))
    i = int(wl.pick(30)[0])
    before = o.dual()

    def dual_with(theta):                   # e_y - u_i = softmax(theta): any interior point of the simplex
        keep = o.U[i].copy()
        e = np.exp(theta - theta.max())
        o.U[i] = -e / e.sum()
        o.U[i, o.y[i]] += 1.0
        val = o.dual()
        o.U[i] = keep
        return val
    res = scipy.optimize.minimize(dual_with, np.zeros(o.J), method="BFGS", options={"gtol": 1e-10})
    assert res.fun < before
    o.step([i], safe_s(wl))
    after = o.dual()
    assert res.fun <= after + 1e-10 <= before + 1e-10
    assert after < before                   # and it does move


@pytest.mark.parametrize("seed", [6, 7])
def test_converges_to_the_primal_minimiser(seed):
    """At the fixed point -u_i = grad f_i(W a_i) and W = grad h*(Z): the gradient of the primal
    vanishes.  Checked with torch's autograd and against scikit-learn's solver."""
    from sklearn.linear_model import LogisticRegression
    wl = small_problem(seed=seed, steps=1500)
    o = run(SdcaMlrOracle, wl, 1500, safe_s(wl))
    val, grad = torch_primal(wl, o.W)
    assert abs(val - o.primal()) < 1e-12
    assert np.abs(grad).max() < 1e-7
    assert -1e-14 <= o.gap() < 1e-10            # zero up to rounding
    # sum_i loss + ||W||^2 / (2 C) has the same minimiser with C = 1 / (lam N)
    clf = LogisticRegression(C=1.0 / (wl.lam * wl.n_data), fit_intercept=False, tol=1e-12, max_iter=10000)
    clf.fit(wl.A.astype(np.float64), wl.y)
    assert clf.coef_.shape == o.W.shape
    np.testing.assert_allclose(o.W, clf.coef_, rtol=0, atol=2e-5)


def test_one_iteration_is_a_minibatch_not_a_sequence():
    """All factors of an iteration come from the W of its start: the order of the picked samples
    does not matter, and two half-iterations in sequence give something else."""
    wl = small_problem(seed=8)
    a = run(SdcaMlrOracle, wl, 3, 0.4)
    b = run(SdcaMlrOracle, wl, 3, 0.4)
    pk = wl.pick(3)
    a.step(pk, 0.4)
    b.step(pk[::-1], 0.4)
    np.testing.assert_allclose(a.W, b.W, rtol=1e-13, atol=1e-16)
    np.testing.assert_allclose(a.U, b.U, rtol=1e-13, atol=1e-16)
    c = run(SdcaMlrOracle, wl, 3, 0.4)
    c.step(pk[:3], 0.4)
    c.step(pk[3:], 0.4)
    assert np.abs(c.W - a.W).max() > 1e-6
    with pytest.raises(ValueError):
        a.step([1, 1], 0.4)


def test_matrix_form_is_the_per_sample_form():
    wl = workloads.make_sdca("sdca_tiny", seed=10, J=7, D=13, n_data=60, P=3, B=5, lam=0.02, steps=6)
    a = SdcaMlrOracle(wl.A, wl.y, wl.J, wl.lam)
    b = SdcaMlrOracle(wl.A, wl.y, wl.J, wl.lam)
    for t in range(6):
        da, fa = a.step(wl.pick(t), 0.35)
        db, fb = b.step_matrix(wl.pick(t), 0.35)
        np.testing.assert_allclose(db, da, rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(fb, fa, rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(b.W, a.W, rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(b.U, a.U, rtol=1e-12, atol=1e-15)


def test_safe_fraction_is_the_single_sample_prox_sdca_step():
    """One picked sample: lam N gamma / (R^2 + lam N gamma) with gamma = 1 / smoothness."""
    assert abs(safe_fraction(0.1, 50, 1, 2.0) - 5.0 / 7.0) < 1e-15
    assert abs(safe_fraction(0.1, 50, 4, 2.0, smoothness=0.5) - 10.0 / 18.0) < 1e-15


# ---------------------------------------------------------------------------------------------
class _NoMeanInZ(SdcaMlrOracle):
    """Planted mistake: the update of Z as literally printed, without 1/N."""
    def step(self, picked, s):
        n = self.N
        self.N = 1
        try:
            return super().step(picked, s)
        finally:
            self.N = n


class _WrongSignOfDelta(SdcaMlrOracle):
    """Planted mistake: u_i <- u_i + delta u_i while Z is still decreased."""
    def step(self, picked, s):
        before = self.U.copy()
        out = super().step(picked, s)
        self.U = 2 * before - self.U
        return out


class _GradientInsteadOfItsNegative(SdcaMlrOracle):
    """Planted mistake: g = softmax - e_y (the SGD factor) used as the optimal dual vector."""
    @staticmethod
    def optimal_dual(z, label):
        return -SdcaMlrOracle.optimal_dual(z, label)


class _LinkMultipliesByLam(SdcaMlrOracle):
    """Planted mistake: W = lam Z."""
    def grad_h_conj(self, Z):
        return Z * self.lam


class _Sequential(SdcaMlrOracle):
    """Planted mistake: every sample sees the updates of the samples picked before it."""
    def step(self, picked, s):
        outs = [super(_Sequential, self).step([i], s) for i in picked]
        return np.concatenate([o[0] for o in outs]), np.concatenate([o[1] for o in outs])


def pins_passed(cls):
    wl = small_problem(seed=9, lam=0.3)
    passed = {"hand": hand_example_matches(cls)}
    o = run(cls, wl, 40, 0.3)
    passed["link"] = bool(link_holds(o))
    passed["descent"] = descends(cls, wl, 60, safe_s(wl)) is not None
    a, b = run(cls, wl, 2, 0.4), run(cls, wl, 2, 0.4)
    a.step(wl.pick(2), 0.4)
    b.step(wl.pick(2)[::-1], 0.4)
    passed["minibatch"] = bool(np.allclose(a.W, b.W, rtol=1e-12, atol=1e-15))
    return passed


def test_the_pins_accept_the_oracle():
    assert all(pins_passed(SdcaMlrOracle).values())


@pytest.mark.parametrize("cls", [_NoMeanInZ, _WrongSignOfDelta, _GradientInsteadOfItsNegative, _LinkMultipliesByLam,
                                 _Sequential])
def test_planted_mistakes_fail_a_pin(cls):
    passed = pins_passed(cls)
    assert not all(passed.values()), f"{cls.__name__} passes every pin: {passed}"
