"""Pins for the proximal-step oracle (oracle/prox_oracle.py): every closed form against the
definition prox_{eta h}(W) = argmin_X 1/2 ||X - W||^2 + eta h(X), minimised numerically, and
against what characterises a projection; planted mistakes must fail."""
import numpy as np
import pytest
import scipy.optimize

from oracle.prox_oracle import prox

RNG = np.random.default_rng(0)


def h(kind, X, lam):
    if kind == "none":
        return 0.0
    if kind == "l2sq":
        return 0.5 * lam * float((X * X).sum())
    if kind == "l1":
        return lam * float(np.abs(X).sum())
    raise ValueError(kind)


def entrywise_argmin(kind, w, eta, lam):
    """The definition, one entry at a time (these regularisers are separable): a bounded scalar
    minimisation, which does not need h to be smooth."""
    obj = lambda x: 0.5 * (x - w) ** 2 + eta * h(kind, np.array([[x]]), lam)
    r = scipy.optimize.minimize_scalar(obj, bounds=(-abs(w) - 1.0, abs(w) + 1.0), method="bounded",
                                       options={"xatol": 1e-12})
    return r.x


@pytest.mark.parametrize("kind", ["none", "l2sq", "l1"])
def test_entrywise_closed_forms_are_the_argmin_of_the_definition(kind, fn=prox):
    W = RNG.standard_normal((3, 4))
    W[0, 0], W[1, 1] = 0.05, -0.05               # inside the l1 dead zone for eta lam = 0.12
    eta, lam = 0.4, 0.3
    got = fn(kind, W, eta, lam)
    for j in range(W.shape[0]):
        for k in range(W.shape[1]):
            assert abs(got[j, k] - entrywise_argmin(kind, W[j, k], eta, lam)) < 1e-6
    if kind == "l1":
        assert got[0, 0] == 0.0 and got[1, 1] == 0.0


def project_columns_numerically(W, r):
    """argmin ||X - W||^2 subject to ||X_k|| <= r for every column, by a constrained solver."""
    J, D = W.shape
    cons = [{"type": "ineq", "fun": (lambda x, k=k: r * r - np.sum(x.reshape(J, D)[:, k] ** 2))} for k in range(D)]
    res = scipy.optimize.minimize(lambda x: 0.5 * np.sum((x - W.ravel()) ** 2), np.zeros(J * D), method="SLSQP",
                                  constraints=cons, options={"ftol": 1e-12, "maxiter": 500})
    assert res.status in (0, 8)                  # 8: the line search cannot improve any further
    return res.x.reshape(J, D)


def test_column_ball_is_the_euclidean_projection(fn=prox):
    W = RNG.standard_normal((4, 5))
    W[:, 1] *= 0.1                               # a column already inside the ball stays put
    r = 0.9
    got = fn("column_ball", W, 0.7, r)
    np.testing.assert_allclose(got, project_columns_numerically(W, r), rtol=0, atol=1e-5)
    assert np.array_equal(got[:, 1], W[:, 1])
    norms = np.sqrt((got * got).sum(0))
    assert norms.max() <= r + 1e-12
    # a projection: idempotent, independent of eta, and W - P(W) makes an obtuse angle with every
    # feasible direction
    np.testing.assert_allclose(fn("column_ball", got, 0.7, r), got, rtol=0, atol=1e-15)
    np.testing.assert_array_equal(fn("column_ball", W, 123.0, r), got)
    for _ in range(20):
        X = RNG.standard_normal(W.shape)
        X *= np.minimum(1.0, r / np.sqrt((X * X).sum(0)))
        assert float(((W - got) * (X - got)).sum()) <= 1e-12


@pytest.mark.parametrize("kind,param", [("l2sq", 0.3), ("l1", 0.3), ("column_ball", 0.8)])
def test_prox_is_nonexpansive(kind, param):
    A, B = RNG.standard_normal((5, 6)), RNG.standard_normal((5, 6))
    d = np.linalg.norm(prox(kind, A, 0.5, param) - prox(kind, B, 0.5, param))
    assert d <= np.linalg.norm(A - B) + 1e-12


def test_limits():
    W = RNG.standard_normal((3, 3))
    for kind in ("l2sq", "l1"):
        np.testing.assert_array_equal(prox(kind, W, 0.0, 0.7), W)        # eta = 0: identity
        np.testing.assert_array_equal(prox(kind, W, 0.7, 0.0), W)        # lam = 0: identity
    np.testing.assert_array_equal(prox("column_ball", W, 1.0, 1e9), W)
    np.testing.assert_array_equal(prox("none", W, 1.0, 1.0), W)
    with pytest.raises(ValueError):
        prox("trace", W, 1.0, 1.0)


# -- planted mistakes ----------------------------------------------------------------------------
def _l1_without_eta(kind, W, eta, param):
    return prox(kind, W, 1.0, param) if kind == "l1" else prox(kind, W, eta, param)


def _l2sq_without_eta(kind, W, eta, param):
    return prox(kind, W, 1.0, param) if kind == "l2sq" else prox(kind, W, eta, param)


def _rows_instead_of_columns(kind, W, eta, param):
    return prox(kind, W.T, eta, param).T if kind == "column_ball" else prox(kind, W, eta, param)


def _normalise_every_column(kind, W, eta, param):
    if kind != "column_ball":
        return prox(kind, W, eta, param)
    return W * (param / np.sqrt((W * W).sum(0)))


@pytest.mark.parametrize("wrong,check,args", [
    (_l1_without_eta, test_entrywise_closed_forms_are_the_argmin_of_the_definition, ("l1",)),
    (_l2sq_without_eta, test_entrywise_closed_forms_are_the_argmin_of_the_definition, ("l2sq",)),
    (_rows_instead_of_columns, test_column_ball_is_the_euclidean_projection, ()),
    (_normalise_every_column, test_column_ball_is_the_euclidean_projection, ()),
])
def test_planted_mistakes_fail(wrong, check, args):
    with pytest.raises(AssertionError):
        check(*args, fn=wrong)
