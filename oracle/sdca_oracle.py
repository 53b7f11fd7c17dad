"""fp64 CPU oracle for SFB driven by stochastic dual coordinate ascent (SDCA) on
l2-regularised multiclass logistic regression ("L2-MLR").

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only tests, the smoke check and the bench's
cpu_baseline leg may import this module.  It shares no code with the HIP library and
never imports it.

Problem (Section 2, problem (P)):   P(W) = (1/N) sum_i f_i(W a_i) + h(W),
    f_i(z) = logsumexp(z) - z_{y_i}       (multiclass logistic loss)
    h(W)   = (lam/2) ||W||_F^2            (the strongly convex regulariser SDCA needs)
Dual as printed in Section 2.1, problem (D) -- a MINIMISATION, i.e. the negated Fenchel dual:
    D(U) = (1/N) sum_i f_i*(-u_i) + h*(Z),      Z = (1/N) sum_i u_i a_i^T,     W = grad h*(Z)
with one dual vector u_i in R^J per data sample.  Weak duality reads P(W') + D(U) >= 0 for
any W', U, with equality exactly at the optimum, where -u_i = grad f_i(W a_i).
Conjugates, written out:
    f_i*(v) = sum_j p_j log p_j  with p = v + e_{y_i}, finite iff p lies in the simplex
    h*(Z)   = ||Z||_F^2 / (2 lam),      grad h*(Z) = Z / lam

One iteration with P workers x B samples (Section 2.1, "Stochastic DCA", run under the SFB
model of Section 3: the pair (delta u_i, a_i) is the sufficient factor that is broadcast):
    1. every picked sample i:  z_i = W a_i  with the W of the iteration's start
    2. delta u_i   (see the reading below)
    3. u_i <- u_i - delta u_i
    4. Z   <- Z - (1/N) sum_i delta u_i a_i^T         (reconstruction from the factors)
    5. W   <- grad h*(Z) = Z / lam

Readings (the paper leaves both open):
  * Step 4.  The text prints Z <- Z - delta u_i a_i^T while defining Z := (1/N) U A^T; the
    definition only survives the update with the factor 1/N, which is what is taken here.
  * Step 2.  The text asks for the delta u_i that minimises (D) with all other dual vectors
    held fixed.  The logistic loss has no closed form for it, and PB such minimisers
    computed from the same W do not add up to a descent step.  Taken instead: the step of
    proximal SDCA (Shalev-Shwartz & Zhang, cited by the paper) -- move a fraction s in (0, 1]
    of the way from u_i to the dual vector that is optimal for the current scores,
        g_i = -grad f_i(z_i) = e_{y_i} - softmax(z_i),     delta u_i = s (u_i - g_i),
    with s supplied by the caller; ``safe_fraction`` gives a value for which (D) cannot
    increase.  The samples of one iteration must be distinct.
Two forms are kept on purpose: ``step`` walks the picked samples one at a time, forming every
rank-1 update explicitly (the definition); ``step_matrix`` does the same arithmetic with
matrix products so that it finishes at larger sizes.  A test pins one to the other.
Starting point: U = 0 (feasible: e_y - 0 is a vertex of the simplex), hence Z = 0, W = 0.
"""
from __future__ import annotations

import numpy as np

__all__ = ["SdcaMlrOracle", "safe_fraction", "mlr_conjugate"]

_F = np.float64


def safe_fraction(lam, n_data, n_picked, max_sq_norm, smoothness=1.0):
    """A fraction s for which one iteration over ``n_picked`` samples cannot increase (D).

    f_i has a ``smoothness``-Lipschitz gradient (1 is safe for the logistic loss, whose
    Hessian diag(p) - p p^T has eigenvalues <= 1/2), so f_i* is (1/smoothness)-strongly
    convex; h* is (1/lam)-smooth.  Along u_i - s (u_i - g_i) the decrease of the f* terms is
    at least s (gap_i) + s (1 - s) ||u_i - g_i||^2 / (2 smoothness) per sample, and the
    increase of the quadratic h* term is at most s^2 n_picked ||a||^2 ||u_i - g_i||^2 /
    (2 lam N) per sample, the factor n_picked bounding the cross terms between the picked
    samples.  The two balance at the value returned.
    """
    c = lam * n_data / smoothness
    return c / (c + n_picked * max_sq_norm)


def mlr_conjugate(v, label):
    """f*(v) of the multiclass logistic loss with true class ``label``: sum p log p, p = v + e_y."""
    p = np.array(v, dtype=_F)
    p[label] += 1.0
    if np.any(p < -1e-12) or abs(p.sum() - 1.0) > 1e-9:
        return np.inf
    p = np.clip(p, 0.0, None)
    nz = p > 0
    return float(np.sum(p[nz] * np.log(p[nz])))


class SdcaMlrOracle:
    def __init__(self, A, y, J, lam):
        self.A = np.asarray(A, dtype=_F)            # [N, D] data samples a_i (rows)
        self.y = np.asarray(y).astype(np.int64)     # [N] class ids
        self.N, self.D = self.A.shape
        self.J = int(J)
        self.lam = float(lam)
        self.U = np.zeros((self.N, self.J), dtype=_F)       # dual vectors u_i (rows)
        self.Z = np.zeros((self.J, self.D), dtype=_F)
        self.W = self.grad_h_conj(self.Z)

    # -- the two conjugate pairs ------------------------------------------------------
    def grad_h_conj(self, Z):
        return Z / self.lam

    def h(self, W):
        return 0.5 * self.lam * float(np.sum(W * W))

    def h_conj(self, Z):
        return float(np.sum(Z * Z)) / (2.0 * self.lam)

    @staticmethod
    def loss(z, label):
        m = np.max(z)
        return float(m + np.log(np.sum(np.exp(z - m))) - z[label])

    @staticmethod
    def optimal_dual(z, label):
        """-grad f(z) = e_y - softmax(z): the dual vector that is optimal for the scores z."""
        e = np.exp(z - np.max(z))
        g = -e / np.sum(e)
        g[label] += 1.0
        return g

    # -- objectives ---------------------------------------------------------------------
    def primal(self, W=None):
        W = self.W if W is None else np.asarray(W, dtype=_F)
        total = 0.0
        for i in range(self.N):
            total += self.loss(W @ self.A[i], self.y[i])
        return total / self.N + self.h(W)

    def conjugate_terms(self):
        """f_i*(-u_i) for every data sample."""
        return np.array([mlr_conjugate(-self.U[i], self.y[i]) for i in range(self.N)])

    def dual(self):
        """Problem (D) as printed (to be minimised); Z is rebuilt from the dual vectors."""
        Z = np.zeros_like(self.Z)
        for i in range(self.N):
            Z += np.outer(self.U[i], self.A[i])
        return float(np.mean(self.conjugate_terms())) + self.h_conj(Z / self.N)

    def gap(self):
        return self.primal() + self.dual()

    # -- one iteration ----------------------------------------------------------------------
    def step(self, picked, s):
        """One SFB iteration on the distinct sample indices ``picked`` (worker-major order,
        P*B of them).  Returns (delta_U [len(picked), J], per-sample primal losses at the
        iteration's start)."""
        picked = [int(i) for i in picked]
        if len(set(picked)) != len(picked):
            raise ValueError("the samples of one iteration must be distinct")
        W = self.W                                   # every worker's replica at the start
        delta = np.zeros((len(picked), self.J), dtype=_F)
        losses = np.zeros(len(picked), dtype=_F)
        for n, i in enumerate(picked):
            z = W @ self.A[i]
            losses[n] = self.loss(z, self.y[i])
            delta[n] = s * (self.U[i] - self.optimal_dual(z, self.y[i]))
        for n, i in enumerate(picked):
            self.U[i] = self.U[i] - delta[n]
            self.Z = self.Z - np.outer(delta[n], self.A[i]) / self.N
        self.W = self.grad_h_conj(self.Z)
        return delta, losses

    def step_matrix(self, picked, s):
        """Same iteration as ``step`` with matrix products instead of per-sample loops."""
        picked = np.asarray(picked, dtype=np.int64)
        if np.unique(picked).size != picked.size:
            raise ValueError("the samples of one iteration must be distinct")
        A, y = self.A[picked], self.y[picked]
        Zs = A @ self.W.T                                        # [n, J] scores at the start
        m = Zs.max(axis=1, keepdims=True)
        e = np.exp(Zs - m)
        lse = m[:, 0] + np.log(e.sum(axis=1))
        losses = lse - Zs[np.arange(picked.size), y]
        G = -e / e.sum(axis=1, keepdims=True)
        G[np.arange(picked.size), y] += 1.0                      # optimal dual vectors
        delta = s * (self.U[picked] - G)
        self.U[picked] = self.U[picked] - delta
        self.Z = self.Z - delta.T @ A / self.N
        self.W = self.grad_h_conj(self.Z)
        return delta, losses
