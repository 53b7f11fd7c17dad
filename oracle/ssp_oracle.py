"""fp64 CPU oracle for stale-synchronous SFB (SSP-SFB) with P replicas of W.

TEST INFRASTRUCTURE, NOT PRODUCT CODE (same rules as sfb_oracle: only tests may
import it; it shares no code with the HIP library and never imports it).

What it computes is the local update rule of the paper's convergence section
written out as a sum, not as a running update:

    W_p  =  W^0  +  sum over workers q  sum over t < tau[p][q]  U_q^t            (Section 5)

where U_q^t = -eta_t * (1/B) * sum_i u_i v_i^T is the partial update worker q
generated at its t-th iteration, from factors (u_i, v_i) computed AT ITS OWN
REPLICA as it stood at that moment (Section 3: the factors, not the matrix,
travel), and tau[p][q] counts how many of q's updates replica p has applied;
tau[p][p] = t_p, a worker applies its own update at once.

The two rules a schedule must obey (Section 4.1 SSP-SFB; Section 5):
  staleness        worker p may start its next iteration only while
                   t_p - tau[p][q] <= s for every q, else it pauses;
  no fast-forward  tau[p][q] <= t_p for q != p (Section 5 requires
                   tau_p^q(c) <= c - 1 for p's c-th iteration, counted from 1).
With s = 0 the two rules leave exactly the bulk-synchronous schedule.

Readings (the paper's indices are loose here): iterations are counted from 0,
tau is a COUNT of applied updates (the inner sum of the printed rule runs
"t = 0 .. tau", one term too many for a count); the |S_p| weight of the printed
partial update is a constant that rescales eta and is left to the caller, so that
staleness 0 reproduces the bulk-synchronous step of sfb_oracle exactly.

Partial broadcast (Section 4.3, Halton sequence broadcast): a worker sends its factors to
Q peers only, worker p to (p + floor(P h)) mod P for the first Q terms h of the sequence
1/2, 1/4, 3/4, 1/8, 3/8, ... (the order the paper prints: level by level, odd numerators
ascending -- not the bit-reversed order of the textbook base-2 Halton sequence, whose fifth
term would be 5/8; offsets that are 0 or repeat an earlier one are skipped).  ``receivers[q]``
is the set of workers q sends to.  Reading: the staleness rule then ranges over the workers
that send to p (nothing else can ever arrive), a delivery along a missing edge is illegal,
and the replicas no longer agree once everything has arrived (the paper: per-iteration
consistency is lost).  ``queue`` bounds how many of its own factor sets a sender may hold
that some receiver has not applied yet (the output queue of Section 4.4 made finite); with
full broadcast and queue >= 2 s + 2 it never binds.

Every replica is formed from the stored factors by the sum above each time it is
asked for; nothing is accumulated incrementally.
"""
from __future__ import annotations

import numpy as np

from . import sfb_oracle as _o

__all__ = ["SspOracle", "halton_offsets", "halton_receivers"]

_F = np.float64


def halton_offsets(P, Q):
    """The first Q distinct non-zero offsets floor(P h) mod P, h = 1/2, 1/4, 3/4, 1/8, 3/8, ...
    (fewer if the sequence runs out of new offsets: at most P - 1 exist)."""
    out, level = [], 2
    while len(out) < Q and level <= 2 * P:
        for num in range(1, level, 2):
            off = (P * num // level) % P
            if off != 0 and off not in out:
                out.append(off)
                if len(out) == Q:
                    break
        level *= 2
    return out


def halton_receivers(P, Q):
    """receivers[p] = the workers p broadcasts to under Halton sequence broadcast."""
    offs = halton_offsets(P, Q)
    return [[(p + o) % P for o in offs] for p in range(P)]


class SspOracle:
    def __init__(self, model, W0, P, B, staleness, receivers=None, queue=None):
        assert model in _o.MODELS and staleness >= 0
        self.model, self.P, self.B, self.s = model, int(P), int(B), int(staleness)
        if receivers is None:
            receivers = [[p for p in range(self.P) if p != q] for q in range(self.P)]
        self.receivers = [sorted(set(int(p) for p in r) - {q}) for q, r in enumerate(receivers)]
        self.senders = [[q for q in range(self.P) if p in self.receivers[q]] for p in range(self.P)]
        self.queue = queue
        self.W0 = np.asarray(W0, dtype=_F).copy()
        self.t = [0] * self.P                                   # iterations completed
        self.tau = [[0] * self.P for _ in range(self.P)]        # tau[p][q]
        self.sets = {}                                          # (q, t) -> (eta, U [B,J], V [B,D])

    # -- the update rule ------------------------------------------------------
    def partial_update(self, q, t):
        """U_q^t as a dense J x D matrix."""
        eta, U, V = self.sets[(q, t)]
        return -eta * (U.T @ V) / self.B

    def replica(self, p):
        """W_p by the sum of the local update rule."""
        W = self.W0.copy()
        for q in range(self.P):
            for t in range(self.tau[p][q]):
                W += self.partial_update(q, t)
        return W

    def auxiliary(self, c):
        """The auxiliary sequence of Section 5: every worker's first c updates, no delays."""
        W = self.W0.copy()
        for q in range(self.P):
            for t in range(c):
                W += self.partial_update(q, t)
        return W

    # -- the schedule's rules -------------------------------------------------
    def queue_full(self, p):
        return self.queue is not None and any(self.t[p] - self.tau[r][p] >= self.queue for r in self.receivers[p])

    def may_step(self, p):
        return all(self.t[p] - self.tau[p][q] <= self.s for q in self.senders[p]) and not self.queue_full(p)

    def may_deliver(self, p, q, count=1):
        return (p != q and p in self.receivers[q] and count >= 0 and self.tau[p][q] + count <= self.t[q]
                and self.tau[p][q] + count <= self.t[p])

    # -- events ---------------------------------------------------------------
    def worker_step(self, p, batch_p, eta):
        """Worker p's next iteration on its own B samples.  Returns None if the staleness rule
        makes it pause, else (U, V, f) of that iteration (fp64)."""
        if not self.may_step(p):
            return None
        W = self.replica(p)
        V = _o.dense_features(self.model, batch_p)
        assert V.shape[0] == self.B
        f, U = _o.loss_and_u(self.model, _o.scores(W, V), batch_p["y"])
        self.sets[(p, self.t[p])] = (float(eta), U, V)
        self.t[p] += 1
        self.tau[p][p] = self.t[p]
        return U, V, f

    def deliver(self, p, q, count=1):
        """Replica p applies the next `count` updates of worker q.  False (nothing done) if illegal."""
        if not self.may_deliver(p, q, count):
            return False
        self.tau[p][q] += count
        return True
