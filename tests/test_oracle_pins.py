"""Pins for the fp64 oracle: every check here compares the oracle with something
that is not the oracle -- hand-derived values, autograd of library losses, finite
differences, closed forms, textbook special cases, invariants.  CPU only."""
import json
import os

import numpy as np
import pytest
import scipy.special
import torch

import oracle
import workloads
from oracle import sfb_oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_examples.json")


def small_batch(model, J, D, P, B, seed=0, scale=1.0):
    """A small random problem built directly (not through the workload recipes)."""
    rng = np.random.default_rng(seed)
    n = P * B
    W = rng.standard_normal((J, D)) * scale
    if model == "mlr":
        batch = {"A": rng.standard_normal((n, D)), "y": rng.integers(0, J, n)}
    elif model == "dml":
        batch = {"X": rng.standard_normal((n, D)) * 0.4, "Y": rng.standard_normal((n, D)) * 0.4,
                 "y": rng.integers(0, 2, n)}
    else:
        dense = rng.standard_normal((n, D)) * (rng.random((n, D)) < 0.4)
        rowptr, col, val = [0], [], []
        for r in range(n):
            nz = np.nonzero(dense[r])[0]
            col += list(nz)
            val += list(dense[r, nz])
            rowptr.append(len(col))
        batch = {"rowptr": np.array(rowptr), "col": np.array(col, dtype=np.int64),
                 "val": np.array(val), "D": D, "y": rng.integers(0, J, n), "_dense": dense}
    return W, batch


def dense_of(model, batch):
    if model == "mlr":
        return np.asarray(batch["A"], dtype=np.float64)
    if model == "dml":
        return np.asarray(batch["X"], dtype=np.float64) - np.asarray(batch["Y"], dtype=np.float64)
    return batch["_dense"]


# ---- independent definition of the objective, written with torch library ops ----
def torch_objective(model, Wt, A, y, P, B, active=None):
    """sum over live workers of the mean per-sample loss, via torch (autograd-able)."""
    Z = A @ Wt.T
    yt = torch.as_tensor(np.asarray(y), dtype=torch.long)
    if model == "mlr":
        f = torch.nn.functional.cross_entropy(Z, yt, reduction="none")
    elif model == "dml":
        q = torch.linalg.vector_norm(Z, dim=1) ** 2
        f = torch.where(yt == 1, q, torch.clamp(1.0 - q, min=0.0))
    else:
        # multi_margin-free spelling: one-vs-rest targets in {+1,-1}, squared hinge
        T = -torch.ones_like(Z)
        T[torch.arange(Z.shape[0]), yt] = 1.0
        f = (torch.relu(1.0 - T * Z) ** 2).sum(dim=1)
    w = torch.ones(P, dtype=torch.float64) if active is None else torch.as_tensor(
        np.asarray(active), dtype=torch.float64)
    return (f.reshape(P, B).mean(dim=1) * w).sum(), f, Z


@pytest.mark.parametrize("case", ["mlr_four_workers", "mlr_minibatch_mean", "dml_three_pairs",
                                  "l2svm_one_sample"])
@pytest.mark.parametrize("form", ["step", "step_per_sample"])
def test_hand_derived_examples(case, form):
    g = json.load(open(GOLDEN))[case]
    model, P, B = g["model"], g["P"], g["B"]
    if model == "mlr":
        batch = {"A": np.array(g["A"]), "y": np.array(g["y"])}
    elif model == "dml":
        batch = {"X": np.array(g["X"]), "Y": np.array(g["Y"]), "y": np.array(g["y"])}
    else:
        batch = {"rowptr": np.array(g["rowptr"]), "col": np.array(g["col"]), "val": np.array(g["val"]),
                 "D": g["D"], "y": np.array(g["y"])}
    U, V, Wn, f = getattr(oracle, form)(model, np.array(g["W"]), batch, P, B, g["eta"])
    np.testing.assert_allclose(U, np.array(g["U"]), rtol=0, atol=1e-15)
    if "V" in g:
        np.testing.assert_allclose(V, np.array(g["V"]), rtol=0, atol=0)
    np.testing.assert_allclose(Wn, np.array(g["W_new"]), rtol=0, atol=1e-15)
    np.testing.assert_allclose(f, np.array(g["loss"]), rtol=0, atol=1e-15)
    np.testing.assert_allclose(oracle.delta_w(U, V, P, B), np.array(g["dW"]), rtol=0, atol=1e-15)


@pytest.mark.parametrize("model,J,D,P,B", [("mlr", 7, 13, 3, 5), ("dml", 6, 11, 2, 9), ("l2svm", 9, 12, 4, 3)])
def test_reconstruction_equals_autograd_gradient(model, J, D, P, B):
    """sum_p (1/B) sum_i u v^T is the gradient of F (the SF identity, Section 2.1):
    compared with autograd through torch's own loss routines, never the oracle's formulas."""
    W, batch = small_batch(model, J, D, P, B, seed=3, scale=0.3)
    A = dense_of(model, batch)
    U, V, f = oracle.factors(model, W, batch)
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    F, ft, Z = torch_objective(model, Wt, torch.tensor(A), batch["y"], P, B)
    Z.retain_grad()
    F.backward()
    np.testing.assert_allclose(oracle.delta_w(U, V, P, B), Wt.grad.numpy(), rtol=1e-12, atol=1e-13)
    # u_i = df_i/dz_i: autograd gives dF/dz_i = u_i / B
    np.testing.assert_allclose(U / B, Z.grad.numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(f, ft.detach().numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(V, A, rtol=0, atol=0)
    assert oracle.objective(model, W, batch, P, B) == pytest.approx(float(F.detach()), rel=1e-13)


@pytest.mark.parametrize("model", ["mlr", "dml", "l2svm"])
def test_finite_differences_every_entry(model):
    """Central differences of F on every entry of W (tiny shape) against delta_w."""
    J, D, P, B = 4, 5, 2, 3
    W, batch = small_batch(model, J, D, P, B, seed=5, scale=0.4)
    A = torch.tensor(dense_of(model, batch))

    def F(Wm):
        return float(torch_objective(model, torch.tensor(Wm), A, batch["y"], P, B)[0])

    U, V, _ = oracle.factors(model, W, batch)
    if model == "dml":   # stay away from the hinge kink so that F is differentiable there
        assert oracle.dml_margin_distance(oracle.scores(W, V), batch["y"]) > 1e-3
    g = oracle.delta_w(U, V, P, B)
    eps = 1e-6
    fd = np.zeros_like(W)
    for j in range(J):
        for d in range(D):
            Wp, Wm = W.copy(), W.copy()
            Wp[j, d] += eps
            Wm[j, d] -= eps
            fd[j, d] = (F(Wp) - F(Wm)) / (2 * eps)
    np.testing.assert_allclose(g, fd, rtol=2e-6, atol=2e-8)


def test_mlr_probabilities_match_scipy():
    W, batch = small_batch("mlr", 11, 6, 2, 4, seed=7, scale=2.0)
    Z = oracle.scores(W, batch["A"])
    f, U = oracle.loss_and_u("mlr", Z, batch["y"])
    onehot = np.eye(11)[batch["y"]]
    np.testing.assert_allclose(U + onehot, scipy.special.softmax(Z, axis=1), rtol=1e-13, atol=1e-16)
    np.testing.assert_allclose(f, scipy.special.logsumexp(Z, axis=1) - Z[np.arange(8), batch["y"]],
                               rtol=1e-13, atol=1e-15)
    # invariants: probabilities sum to 1, residual rows sum to 0, probabilities in [0, 1]
    np.testing.assert_allclose((U + onehot).sum(axis=1), 1.0, atol=1e-14)
    np.testing.assert_allclose(U.sum(axis=1), 0.0, atol=1e-14)
    assert np.all(U + onehot >= 0) and np.all(U + onehot <= 1)


def test_mlr_softmax_is_shift_invariant_and_safe_for_large_scores():
    z = np.array([[1000.0, 999.0, -1000.0]])
    f, U = oracle.loss_and_u("mlr", z, [1])
    e = np.exp([0.0, -1.0])
    np.testing.assert_allclose(U[0], [e[0] / e.sum(), e[1] / e.sum() - 1.0, 0.0], atol=1e-15)
    assert f[0] == pytest.approx(np.log(e.sum()) + 1.0, rel=1e-14)


def test_closed_forms_at_zero_w():
    J, D, P, B = 5, 4, 2, 3
    rng = np.random.default_rng(0)
    n = P * B
    y = rng.integers(0, J, n)
    W0 = np.zeros((J, D))
    # MLR: u = 1/J - e_y
    U, _, f = oracle.factors("mlr", W0, {"A": rng.standard_normal((n, D)), "y": y})
    np.testing.assert_allclose(U, 1.0 / J - np.eye(J)[y], atol=1e-16)
    np.testing.assert_allclose(f, np.log(J), atol=1e-15)
    # L2SVM (one-vs-rest): z = 0 -> h = 1 for all classes, u_j = -2 t_j, f = J
    _, bsv = small_batch("l2svm", J, D, P, B, seed=1)
    U, _, f = oracle.factors("l2svm", W0, bsv)
    T = -np.ones((n, J))
    T[np.arange(n), bsv["y"]] = 1
    np.testing.assert_allclose(U, -2 * T, atol=0)
    np.testing.assert_allclose(f, J, atol=0)
    # DML: z = 0 -> u = 0 for both kinds of pair, so the step leaves W unchanged
    _, bd = small_batch("dml", J, D, P, B, seed=2)
    U, V, Wn, f = oracle.step("dml", W0, bd, P, B, 0.7)
    assert not U.any() and not Wn.any()
    np.testing.assert_allclose(f, np.where(bd["y"] == 1, 0.0, 1.0), atol=0)


def test_two_class_mlr_is_binary_logistic_regression():
    """J = 2: softmax over (z0, z1) is the logistic sigmoid of z1 - z0 (textbook identity)."""
    W, batch = small_batch("mlr", 2, 6, 1, 10, seed=11)
    U, V, _ = oracle.factors("mlr", W, batch)
    p1 = scipy.special.expit(batch["A"] @ (W[1] - W[0]))
    np.testing.assert_allclose(U[:, 1], p1 - batch["y"], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(U[:, 0], -(p1 - batch["y"]), rtol=1e-12, atol=1e-15)
    # gradient of the binary cross-entropy with respect to w1 is A^T (p - y) / B
    np.testing.assert_allclose(oracle.delta_w(U, V, 1, 10)[1], batch["A"].T @ (p1 - batch["y"]) / 10,
                               rtol=1e-12, atol=1e-15)


def test_dml_branches():
    z_in, z_out = np.array([[0.3, 0.4]]), np.array([[0.6, 0.8]])   # ||z||^2 = 0.25 and exactly 1
    f, U = oracle.loss_and_u("dml", np.vstack([z_in, z_in, z_out, 2 * z_out]), [1, 0, 0, 0])
    np.testing.assert_allclose(U, [[0.6, 0.8], [-0.6, -0.8], [0, 0], [0, 0]], atol=1e-16)
    np.testing.assert_allclose(f, [0.25, 0.75, 0.0, 0.0], atol=1e-16)
    assert oracle.dml_margin_distance(np.vstack([z_in, z_in]), [1, 0]) == pytest.approx(0.75)


@pytest.mark.parametrize("model", ["mlr", "dml", "l2svm"])
def test_rank_bounds(model):
    """One sample's update has rank 1; a step's update has rank <= P*B (Section 2.1, low-rank extensions)."""
    W, batch = small_batch(model, 9, 10, 1, 1, seed=13, scale=0.2)
    U, V, _ = oracle.factors(model, W, batch)
    dW = oracle.delta_w(U, V, 1, 1)
    if np.abs(dW).max() > 0:
        assert np.linalg.matrix_rank(dW) == 1
    W, batch = small_batch(model, 9, 10, 2, 2, seed=14, scale=0.2)
    U, V, _ = oracle.factors(model, W, batch)
    assert np.linalg.matrix_rank(oracle.delta_w(U, V, 2, 2)) <= 4


@pytest.mark.parametrize("model", ["mlr", "dml", "l2svm"])
def test_per_sample_form_equals_matrix_form(model):
    W, batch = small_batch(model, 6, 8, 3, 4, seed=17, scale=0.3)
    a = oracle.step(model, W, batch, 3, 4, 0.1)
    b = oracle.step_per_sample(model, W, batch, 3, 4, 0.1)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, rtol=1e-13, atol=1e-14)
    mask = [1, 0, 1]
    a = oracle.step(model, W, batch, 3, 4, 0.1, active=mask)
    b = oracle.step_per_sample(model, W, batch, 3, 4, 0.1, active=mask)
    np.testing.assert_allclose(a[2], b[2], rtol=1e-13, atol=1e-14)


def test_worker_order_does_not_matter_and_dead_worker_drops_out():
    """BSP: the outcome is a function of the set of factors, not of arrival order (Section 4.1);
    a failed worker's factors are simply absent (Section 4.4)."""
    P, B = 4, 3
    W, batch = small_batch("mlr", 5, 7, P, B, seed=19)
    _, _, Wn, _ = oracle.step("mlr", W, batch, P, B, 0.2)
    perm = [2, 0, 3, 1]
    rows = np.concatenate([np.arange(p * B, (p + 1) * B) for p in perm])
    pb = {"A": batch["A"][rows], "y": batch["y"][rows]}
    np.testing.assert_allclose(oracle.step("mlr", W, pb, P, B, 0.2)[2], Wn, rtol=1e-13, atol=1e-15)
    # dropping worker 1 equals running the three survivors alone
    keep = np.concatenate([np.arange(p * B, (p + 1) * B) for p in (0, 2, 3)])
    sb = {"A": batch["A"][keep], "y": batch["y"][keep]}
    np.testing.assert_allclose(oracle.step("mlr", W, batch, P, B, 0.2, active=[1, 0, 1, 1])[2],
                               oracle.step("mlr", W, sb, 3, B, 0.2)[2], rtol=1e-13, atol=1e-15)
    # and its gradient is the autograd gradient of the masked objective
    Wt = torch.tensor(W, requires_grad=True)
    torch_objective("mlr", Wt, torch.tensor(batch["A"]), batch["y"], P, B, active=[1, 0, 1, 1])[0].backward()
    U, V, _ = oracle.factors("mlr", W, batch)
    np.testing.assert_allclose(oracle.delta_w(U, V, P, B, active=[1, 0, 1, 1]), Wt.grad.numpy(),
                               rtol=1e-12, atol=1e-14)


def test_sign_and_step_size_follow_gradient_descent():
    """W - eta*dW must decrease F for small eta, and the first-order change is -eta*||dW||^2."""
    for model in oracle.MODELS:
        W, batch = small_batch(model, 6, 7, 2, 4, seed=23, scale=0.3)
        A = torch.tensor(dense_of(model, batch))
        F0 = float(torch_objective(model, torch.tensor(W), A, batch["y"], 2, 4)[0])
        U, V, Wn, _ = oracle.step(model, W, batch, 2, 4, 1e-5)
        F1 = float(torch_objective(model, torch.tensor(Wn), A, batch["y"], 2, 4)[0])
        g2 = float((oracle.delta_w(U, V, 2, 4) ** 2).sum())
        assert F1 < F0
        assert (F0 - F1) == pytest.approx(1e-5 * g2, rel=1e-3)


def test_tiny_config_objective_decreases_over_five_steps():
    wl = workloads.make("mlr_tiny")
    W = wl.W0.astype(np.float64)
    batch = wl.batch(0)
    prev = oracle.objective("mlr", W, batch, wl.P, wl.B)
    for _ in range(wl.steps):
        _, _, W, _ = oracle.step("mlr", W, batch, wl.P, wl.B, wl.eta)
        cur = oracle.objective("mlr", W, batch, wl.P, wl.B)
        assert cur < prev
        prev = cur


def test_message_size_is_linear_in_dimensions():
    """Cost table, Section 5.1: a worker sends K(J+D) values per peer instead of J*D."""
    wl = workloads.make("mlr_tiny")
    U, V, _ = oracle.factors("mlr", wl.W0, wl.batch(0))
    per_worker = (U.size + V.size) // wl.P
    assert per_worker == wl.B * (wl.J + wl.D)
    assert U.shape == (wl.N, wl.J) and V.shape == (wl.N, wl.D)


def test_csr_expansion_matches_scipy():
    import scipy.sparse
    _, b = small_batch("l2svm", 3, 17, 2, 5, seed=29)
    ref = scipy.sparse.csr_matrix((b["val"], b["col"], b["rowptr"]), shape=(10, 17)).toarray()
    np.testing.assert_array_equal(oracle.csr_to_dense(b["rowptr"], b["col"], b["val"], 17), ref)
    np.testing.assert_array_equal(ref, b["_dense"])


def test_csr_column_repeated_inside_a_row_counts_as_the_sum_of_its_values():
    """A stored entry is a term of the sparse vector: two entries on one column add up (what scipy's
    CSR does as well), in any order of the entries."""
    import scipy.sparse
    rowptr = np.array([0, 4, 4, 7], dtype=np.int32)
    col = np.array([5, 1, 5, 0, 2, 2, 2], dtype=np.int32)
    val = np.array([0.5, -1.0, 0.25, 2.0, 1.0, 2.0, 4.0], dtype=np.float32)
    got = oracle.csr_to_dense(rowptr, col, val, 6)
    want = np.zeros((3, 6))
    want[0, 5], want[0, 1], want[0, 0], want[2, 2] = 0.75, -1.0, 2.0, 7.0
    np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(got, scipy.sparse.csr_matrix((val, col, rowptr), shape=(3, 6)).toarray())


# ---- planted mistakes: each plausible slip must trip the autograd pin ----
def _autograd_pin_holds(model="mlr"):
    try:
        test_reconstruction_equals_autograd_gradient(model, 7, 13, 3, 5)
        return True
    except AssertionError:
        return False


def test_planted_mistakes_are_caught(monkeypatch):
    assert _autograd_pin_holds("mlr") and _autograd_pin_holds("dml") and _autograd_pin_holds("l2svm")
    real_one = dict(sfb_oracle._ONE)
    # wrong sign of the residual
    monkeypatch.setitem(sfb_oracle._ONE, "mlr", lambda z, y: (real_one["mlr"](z, y)[0], -real_one["mlr"](z, y)[1]))
    assert not _autograd_pin_holds("mlr")
    monkeypatch.setitem(sfb_oracle._ONE, "mlr", real_one["mlr"])
    # dropped one-hot term (u = the probability vector alone)
    def no_onehot(z, y):
        f, u = real_one["mlr"](z, y)
        u = u.copy(); u[y] += 1.0
        return f, u
    monkeypatch.setitem(sfb_oracle._ONE, "mlr", no_onehot)
    assert not _autograd_pin_holds("mlr")
    monkeypatch.setitem(sfb_oracle._ONE, "mlr", real_one["mlr"])
    # dropped factor 2 in DML, non-strict svm sign
    monkeypatch.setitem(sfb_oracle._ONE, "dml", lambda z, s: (real_one["dml"](z, s)[0], 0.5 * real_one["dml"](z, s)[1]))
    assert not _autograd_pin_holds("dml")
    monkeypatch.setitem(sfb_oracle._ONE, "dml", real_one["dml"])
    monkeypatch.setitem(sfb_oracle._ONE, "l2svm", lambda z, y: (real_one["l2svm"](z, y)[0], np.abs(real_one["l2svm"](z, y)[1])))
    assert not _autograd_pin_holds("l2svm")
    monkeypatch.setitem(sfb_oracle._ONE, "l2svm", real_one["l2svm"])
    # dropped 1/B, and transposed operands in the reconstruction
    real_scores = sfb_oracle.scores
    monkeypatch.setattr(sfb_oracle, "scores", lambda W, A: real_scores(W, A) * 1.0001)
    assert not _autograd_pin_holds("mlr")
    monkeypatch.setattr(sfb_oracle, "scores", real_scores)
    real_dw = oracle.delta_w
    monkeypatch.setattr(oracle, "delta_w", lambda U, V, P, B, active=None: real_dw(U, V, P, B, active) * B)
    assert not _autograd_pin_holds("mlr")
    monkeypatch.setattr(oracle, "delta_w", real_dw)
    assert _autograd_pin_holds("mlr")
