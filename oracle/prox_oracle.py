"""fp64 CPU oracle for the proximal step of proximal SGD (Section 2.1): after
W <- W - eta * dW the operator prox_{eta h} is applied to W,

    prox_{eta h}(W) = argmin_X  1/2 ||X - W||_F^2 + eta h(X).

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only tests, the smoke check and the bench's
cpu_baseline leg may import this module.  It shares no code with the HIP library and
never imports it.

The regularisers are the ones Section 2 names that have an entrywise or columnwise closed
form (the trace norm, which needs a singular value decomposition, is left out):
  none         h = 0                              prox = identity
  l2sq         h = (lam/2) ||W||_F^2              prox = W / (1 + eta lam)
  l1           h = lam ||W||_1 (entrywise)        prox = sign(w) max(|w| - eta lam, 0)
  column_ball  h = indicator{ ||W_k||_2 <= r for every column k }  (sparse coding, Section 2:
               each column of the dictionary inside the unit ball; the prox of an indicator is
               the Euclidean projection, whatever eta)
                                                  prox: W_k <- W_k * min(1, r / ||W_k||_2)
The definition above (a minimisation) is what the tests pin these closed forms to.
"""
from __future__ import annotations

import numpy as np

__all__ = ["PROX_KINDS", "prox"]

PROX_KINDS = ("none", "l2sq", "l1", "column_ball")
_F = np.float64


def prox(kind, W, eta, param):
    """prox_{eta h}(W) for the regulariser ``kind``; ``param`` is lam (l2sq, l1) or the radius r
    (column_ball; eta is irrelevant there)."""
    W = np.asarray(W, dtype=_F)
    J, D = W.shape
    out = np.empty_like(W)
    if kind == "none":
        out[:] = W
    elif kind == "l2sq":
        out[:] = W / (1.0 + eta * param)
    elif kind == "l1":
        thr = eta * param
        out[:] = np.where(W > thr, W - thr, np.where(W < -thr, W + thr, 0.0))
    elif kind == "column_ball":
        for k in range(D):
            norm = float(np.sqrt(np.sum(W[:, k] * W[:, k])))
            out[:, k] = W[:, k] * (param / norm) if norm > param else W[:, k]
    else:
        raise ValueError(kind)
    return out
