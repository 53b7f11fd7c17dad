"""fp64 CPU oracle for one step of Sufficient Factor Broadcasting (SFB).

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only tests, the smoke check and the
bench's cpu_baseline leg may import this module.  It shares no code with the
HIP library and never imports it.

What it computes (one bulk-synchronous SFB iteration on P simulated workers,
each holding B samples of the minibatch and an identical replica of W):

  1. scores        z_i = W a_i                      (Section 2, problem (P))
  2. factor u      u_i = d f_i(z_i) / d z_i         (Section 2.1, proximal SGD)
  3. factor v      v_i = a_i                        (Section 2.1, proximal SGD)
  4. exchange      every worker ends up holding all P*B pairs, worker-major
                   (Section 3, SFB model of computation)
  5. reconstruct   dW = sum_p (1/B) sum_i u_{p,i} v_{p,i}^T
                   (Section 3: sum over workers; mini-batch paragraph: mean
                   inside one worker's mini-batch of K = B samples)
  6. apply         W <- W - eta * dW, prox = identity because h = 0
                   (Section 2.1)

Everything is float64.  Inputs that were quantised to fp32 / bf16 for the
device are passed in already quantised and only widened here, so input
rounding is not counted as error.

Two forms are kept on purpose:
  * ``step_per_sample`` walks workers and samples one at a time, forming every
    rank-1 update u v^T explicitly -- the definition, for small cases;
  * ``step`` does the same arithmetic with matrix products so that it
    finishes at the benchmark sizes.  tests pin the two to each other and
    both to independent references (autograd, finite differences, closed
    forms, a hand-computed example).

Loss functions f(z; b) per model (z = W a):
  MLR    f = logsumexp(z) - z_y                      multiclass logistic loss
                                                     (Section 2, examples of f_i)
  DML    a = x - y (pair difference), z = W a;
         similar pair:    f = ||z||^2                (quadratic)
         dissimilar pair: f = max(0, 1 - ||z||^2)    (hinge, margin 1)
                                                     (Section 2, DML paragraph)
  L2SVM  one-vs-rest squared hinge, t_j = +1 if j == y else -1:
         f = sum_j max(0, 1 - t_j z_j)^2             (reading of "l2 loss ...
                                                     amongst others", Section 2;
                                                     the paper never runs it)
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "MODELS", "dense_features", "csr_to_dense", "scores",
    "loss_and_u", "factors", "delta_w", "apply_update", "step",
    "step_per_sample", "objective", "dml_margin_distance",
]

MODELS = ("mlr", "dml", "l2svm")

_F = np.float64


# --------------------------------------------------------------------------
# inputs
# --------------------------------------------------------------------------
def csr_to_dense(rowptr, col, val, n_cols):
    """Dense fp64 expansion of a CSR matrix, one stored entry at a time."""
    rowptr = np.asarray(rowptr)
    n_rows = rowptr.shape[0] - 1
    out = np.zeros((n_rows, int(n_cols)), dtype=_F)
    for r in range(n_rows):
        for n in range(int(rowptr[r]), int(rowptr[r + 1])):
            out[r, int(col[n])] += float(val[n])
    return out


def dense_features(model, batch):
    """The vectors a_i of problem (P), as an [N, D] fp64 matrix.

    MLR: the feature vector.  DML: the difference of the pair's two feature
    vectors (Section 2, DML paragraph).  L2SVM: the CSR row, densified.
    """
    if model == "mlr":
        return np.asarray(batch["A"], dtype=_F)
    if model == "dml":
        return np.asarray(batch["X"], dtype=_F) - np.asarray(batch["Y"], dtype=_F)
    if model == "l2svm":
        return csr_to_dense(batch["rowptr"], batch["col"], batch["val"], batch["D"])
    raise ValueError(f"unknown model {model!r}")


# --------------------------------------------------------------------------
# step 1: scores
# --------------------------------------------------------------------------
def scores(W, A):
    """Z[i, :] = W a_i for every row a_i of A (problem (P))."""
    return np.asarray(A, dtype=_F) @ np.asarray(W, dtype=_F).T


# --------------------------------------------------------------------------
# step 2: per-sample loss and u = df/dz
# --------------------------------------------------------------------------
def _mlr_one(z, y):
    m = np.max(z)
    e = np.exp(z - m)
    s = e / np.sum(e)                       # softmax(z)
    f = m + np.log(np.sum(e)) - z[y]        # logsumexp(z) - z_y
    u = s.copy()
    u[y] -= 1.0                             # softmax(z) - e_y
    return f, u


def _dml_one(z, similar):
    q = float(np.dot(z, z))                 # ||z||^2
    if similar:
        return q, 2.0 * z
    if q < 1.0:                             # hinge active (strictly inside)
        return 1.0 - q, -2.0 * z
    return 0.0, np.zeros_like(z)            # at or beyond the margin


def _l2svm_one(z, y):
    t = -np.ones_like(z)
    t[y] = 1.0
    h = np.maximum(0.0, 1.0 - t * z)
    return float(np.sum(h * h)), -2.0 * t * h


_ONE = {"mlr": _mlr_one, "dml": _dml_one, "l2svm": _l2svm_one}


def loss_and_u(model, Z, y):
    """Per-sample loss f_i [N] and factor u_i = df_i/dz_i [N, J] (Section 2.1).

    ``y`` holds class ids (MLR, L2SVM) or 1 = similar / 0 = dissimilar (DML).
    """
    Z = np.asarray(Z, dtype=_F)
    y = np.asarray(y)
    one = _ONE[model]
    U = np.empty_like(Z)
    f = np.empty(Z.shape[0], dtype=_F)
    for i in range(Z.shape[0]):
        f[i], U[i] = one(Z[i], int(y[i]))
    return f, U


def dml_margin_distance(Z, y):
    """min over dissimilar pairs of | ||z_i||^2 - 1 |: distance to the hinge kink.

    An fp32 implementation may take the other branch for a pair that sits
    within rounding error of the kink; parity tests consult this.
    """
    Z = np.asarray(Z, dtype=_F)
    y = np.asarray(y)
    q = np.sum(Z * Z, axis=1)
    d = np.abs(q - 1.0)[y == 0]
    return float(d.min()) if d.size else float("inf")


# --------------------------------------------------------------------------
# steps 2-4: factors of the whole step, in worker-major order
# --------------------------------------------------------------------------
def factors(model, W, batch):
    """(U [N,J], V [N,D], f [N]) for all N = P*B samples of the step.

    Every sample is differentiated at the same W: replicas are identical at
    the start of a bulk-synchronous iteration (Section 4.1, BSP-SFB).  Row
    p*B + i belongs to worker p, so the arrays are already the concatenation
    every worker holds after all broadcasts have arrived (Section 3).
    """
    V = dense_features(model, batch)        # v_i = a_i
    Z = scores(W, V)
    f, U = loss_and_u(model, Z, batch["y"])
    return U, V, f


# --------------------------------------------------------------------------
# step 5: reconstruction
# --------------------------------------------------------------------------
def _live(P, active):
    if active is None:
        return np.ones(P, dtype=bool)
    a = np.asarray(active).astype(bool)
    if a.shape != (P,):
        raise ValueError("active mask must have P entries")
    return a


def delta_w(U, V, P, B, active=None):
    """dW = sum over live workers p of (1/B) * sum_i u_{p,i} v_{p,i}^T.

    Section 3: each worker applies the sum of all workers' updates; the
    mini-batch paragraph averages inside one worker's mini-batch.  A worker
    whose mask entry is 0 (a failed worker, Section 4.4) contributes nothing.
    """
    U = np.asarray(U, dtype=_F)
    V = np.asarray(V, dtype=_F)
    if U.shape[0] != P * B or V.shape[0] != P * B:
        raise ValueError("U and V must have P*B rows")
    live = _live(P, active)
    # every sample's outer product u v^T enters with weight 1/B if its worker is live and 0
    # otherwise: scale the rows of U by that weight, then sum the outer products (U^T V)
    weight = np.repeat(np.where(live, 1.0 / B, 0.0), B)
    return (U * weight[:, None]).T @ V


# --------------------------------------------------------------------------
# step 6: apply
# --------------------------------------------------------------------------
def apply_update(W, dW, eta):
    """W - eta * dW (Section 2.1); the proximal operator of h = 0 is the identity."""
    return np.asarray(W, dtype=_F) - float(eta) * dW


def step(model, W, batch, P, B, eta, active=None):
    """One SFB iteration.  Returns (U, V, W_new, f) in fp64."""
    U, V, f = factors(model, W, batch)
    W_new = apply_update(W, delta_w(U, V, P, B, active), eta)
    return U, V, W_new, f


def step_per_sample(model, W, batch, P, B, eta, active=None):
    """The same iteration, one sample and one rank-1 update at a time.

    Worker p, sample i: z = W a, u = df/dz, v = a; the receiver rebuilds the
    worker's update as the mean of its B outer products and subtracts the
    sum over workers, scaled by eta.  Quadratic-cost loops: small cases only.
    """
    W = np.asarray(W, dtype=_F)
    A = dense_features(model, batch)
    y = np.asarray(batch["y"])
    J, D = W.shape
    live = _live(P, active)
    one = _ONE[model]
    U = np.zeros((P * B, J), dtype=_F)
    V = np.zeros((P * B, D), dtype=_F)
    f = np.zeros(P * B, dtype=_F)
    total = np.zeros((J, D), dtype=_F)
    for p in range(P):
        worker_update = np.zeros((J, D), dtype=_F)
        for i in range(B):
            r = p * B + i
            a = A[r]
            z = np.array([np.dot(W[j], a) for j in range(J)])
            f[r], u = one(z, int(y[r]))
            U[r] = u
            V[r] = a
            worker_update += np.outer(u, a)
        if live[p]:
            total += worker_update / B
    return U, V, W - float(eta) * total, f


def objective(model, W, batch, P, B, active=None):
    """F(W) = sum over live workers of (1/B) sum_i f_i(W a_i).

    Its gradient with respect to W is exactly ``delta_w`` of the factors:
    the sufficient-factor identity of Section 2.1.
    """
    _, _, f = factors(model, W, batch)
    live = _live(P, active)
    return float(sum(f[p * B:(p + 1) * B].sum() / B for p in range(P) if live[p]))
