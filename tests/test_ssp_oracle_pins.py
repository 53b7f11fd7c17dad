"""Pins for the stale-synchronous oracle (oracle/ssp_oracle.py), none of which re-types its
own formula: a schedule worked by hand (tests/golden/ssp_hand_example.json), the
bulk-synchronous oracle as the staleness-0 special case, the auxiliary sequence of Section 5
as the limit of every replica once all updates have arrived, the bound that sizes the
device ring, and planted mistakes that each of these must catch."""
import json
import os

import numpy as np
import pytest

import oracle
import workloads
from oracle.ssp_oracle import SspOracle, halton_offsets, halton_receivers

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "ssp_hand_example.json")


def replay(o, events, shares, eta):
    """Replays proposals; returns the accepted flags."""
    flags = []
    for ev in events:
        if ev[0] == "step":
            flags.append(o.worker_step(ev[1], shares[ev[1]](o.t[ev[1]]), eta) is not None)
        else:
            flags.append(o.deliver(ev[1], ev[2], ev[3]))
    return flags


def hand_example(cls=SspOracle):
    g = json.load(open(GOLDEN))
    W0 = np.array([[g["W0"]]])
    o = cls(g["model"], W0, g["P"], g["B"], g["staleness"])
    shares = [lambda t, a=a: {"X": np.array([[a]]), "Y": np.array([[0.0]]), "y": np.array([1])}
              for a in g["pair_difference"]]
    rows = []
    for ev in g["events"]:
        flag = replay(o, [tuple(ev)], shares, g["eta"])[0]
        rows.append((flag, o.replica(0)[0, 0], o.replica(1)[0, 0]))
    return g, o, rows


def test_hand_worked_schedule():
    g, o, rows = hand_example()
    assert [r[0] for r in rows] == g["accepted"]
    np.testing.assert_allclose([r[1] for r in rows], g["w0_after"], rtol=0, atol=1e-15)
    np.testing.assert_allclose([r[2] for r in rows], g["w1_after"], rtol=0, atol=1e-15)
    assert abs(o.auxiliary(2)[0, 0] - g["auxiliary_after_two"]) < 1e-15
    assert o.t == [2, 2] and o.tau == [[2, 2], [2, 2]]


class _GradientAtSharedW(SspOracle):
    """Planted mistake: one shared W holding every update produced so far, instead of the own replica."""
    def replica(self, p):
        W = self.W0.copy()
        for (q, t) in self.sets:
            W += self.partial_update(q, t)
        return W


class _StrictStaleness(SspOracle):
    """Planted mistake: pauses one iteration too early."""
    def may_step(self, p):
        return all(self.t[p] - self.tau[p][q] < self.s for q in range(self.P) if q != p)


class _InclusiveSum(SspOracle):
    """Planted mistake: the printed rule's 't = 0 .. tau' taken literally on a count."""
    def replica(self, p):
        W = self.W0.copy()
        for q in range(self.P):
            for t in range(min(self.tau[p][q] + 1, self.t[q])):
                W += self.partial_update(q, t)
        return W


class _FastForward(SspOracle):
    """Planted mistake: a replica may apply more of q's iterations than it has completed itself."""
    def may_deliver(self, p, q, count=1):
        return p != q and count >= 0 and self.tau[p][q] + count <= self.t[q]


@pytest.mark.parametrize("cls", [_GradientAtSharedW, _StrictStaleness, _InclusiveSum, _FastForward])
def test_planted_mistakes_fail_the_hand_example(cls):
    g, o, rows = hand_example(cls)
    same = ([r[0] for r in rows] == g["accepted"]
            and np.allclose([r[1] for r in rows], g["w0_after"], rtol=0, atol=1e-12)
            and np.allclose([r[2] for r in rows], g["w1_after"], rtol=0, atol=1e-12))
    assert not same, f"{cls.__name__} reproduces the hand-worked example: the example does not pin that reading"


@pytest.mark.parametrize("name,override", [("mlr_tiny", {}), ("dml", dict(J=6, D=20, P=3, B=4)),
                                           ("l2svm", dict(J=7, D=40, P=2, B=5, density=0.2))])
def test_staleness_zero_is_the_bulk_synchronous_step(name, override):
    """Section 4.1: with s = 0 SSP-SFB reduces to BSP-SFB.  Every replica after round r equals the
    W of the (separately pinned) bulk-synchronous oracle after r steps, and nobody can run ahead."""
    wl = workloads.make(name, seed=3, **override)
    o = SspOracle(wl.model, wl.W0, wl.P, wl.B, 0)
    W = wl.W0.astype(np.float64)
    for r in range(3):
        b = wl.batch(r)
        for p in range(wl.P):
            assert o.worker_step(p, workloads.worker_share(wl.model, b, p, wl.B), wl.eta) is not None
        assert o.worker_step(0, workloads.worker_share(wl.model, b, 0, wl.B), wl.eta) is None   # must pause
        for p in range(wl.P):
            for q in range(wl.P):
                if p != q:
                    assert o.deliver(p, q, 1)
        _, _, W, _ = oracle.step(wl.model, W, b, wl.P, wl.B, wl.eta)
        for p in range(wl.P):
            np.testing.assert_allclose(o.replica(p), W, rtol=1e-12, atol=1e-14)


def drive_to(o, wl, C):
    """Any legal completion: everybody reaches C iterations and receives everything."""
    for _ in range(100 * C * wl.P * wl.P):
        moved = False
        for p in range(wl.P):
            for q in range(wl.P):
                if p != q and o.may_deliver(p, q, 1):
                    o.deliver(p, q, 1)
                    moved = True
            if o.t[p] < C and o.may_step(p):
                o.worker_step(p, workloads.worker_share(wl.model, wl.batch(o.t[p]), p, wl.B), wl.eta)
                moved = True
        if not moved:
            break
    return all(t == C for t in o.t) and all(x == C for row in o.tau for x in row)


@pytest.mark.parametrize("s,seed", [(1, 0), (2, 1), (3, 2)])
def test_random_schedules_keep_the_bounds_and_end_on_the_auxiliary_sequence(s, seed):
    wl = workloads.make("mlr_tiny", seed=seed, J=5, D=12, P=4, B=3)
    o = SspOracle(wl.model, wl.W0, wl.P, wl.B, s)
    accepted = 0
    for ev in workloads.ssp_proposals(wl.P, 400, seed=seed):
        if ev[0] == "step":
            if o.t[ev[1]] >= 12:
                continue
            ok = o.worker_step(ev[1], workloads.worker_share(wl.model, wl.batch(o.t[ev[1]]), ev[1], wl.B), wl.eta) is not None
        else:
            ok = o.deliver(ev[1], ev[2], ev[3])
        accepted += ok
        for p in range(wl.P):
            for q in range(wl.P):
                assert o.t[p] - o.tau[p][q] <= s + 1          # p ran at most one past the rule's check
                assert o.tau[p][q] <= o.t[p] or p == q
                assert o.t[q] - o.tau[p][q] <= 2 * s + 2      # what sizes the device ring: 2s + 2 sets per sender
    assert accepted > 100
    assert max(o.t) - min(o.t) <= s + 1
    C = max(o.t)
    assert drive_to(o, wl, C)
    aux = o.auxiliary(C)
    for p in range(wl.P):
        np.testing.assert_allclose(o.replica(p), aux, rtol=1e-12, atol=1e-15)


def test_replicas_disagree_under_staleness_and_not_without():
    """With s > 0 and undelivered updates the replicas really differ (so the parity tests
    compare something), and the disagreement is exactly the undelivered partial updates."""
    wl = workloads.make("mlr_tiny", seed=5, J=4, D=9, P=2, B=3)
    o = SspOracle(wl.model, wl.W0, wl.P, wl.B, 2)
    o.worker_step(0, workloads.worker_share(wl.model, wl.batch(0), 0, wl.B), wl.eta)
    o.worker_step(0, workloads.worker_share(wl.model, wl.batch(1), 0, wl.B), wl.eta)
    o.worker_step(1, workloads.worker_share(wl.model, wl.batch(0), 1, wl.B), wl.eta)
    gap = o.replica(0) - o.replica(1)
    want = o.partial_update(0, 0) + o.partial_update(0, 1) - o.partial_update(1, 0)
    np.testing.assert_allclose(gap, want, rtol=1e-12, atol=1e-16)
    assert np.abs(gap).max() > 1e-6


# -- partial broadcast (Section 4.3) ----------------------------------------------------------
HSB = os.path.join(os.path.dirname(__file__), "golden", "hsb_hand_example.json")


def test_halton_peers_are_the_papers_example():
    g = json.load(open(HSB))
    ex = g["paper_example"]
    assert halton_offsets(ex["P"], ex["Q"]) == ex["offsets"]
    rec = halton_receivers(ex["P"], ex["Q"])
    for p in range(ex["P"]):
        assert sorted(rec[p]) == sorted([(p + 3) % 6, (p + 1) % 6])
    for label, peers in ex["one_based"].items():            # the paper's labels: machine 6 is index 0
        assert sorted(rec[int(label) % 6]) == sorted(q % 6 for q in peers)
    assert halton_offsets(16, 5) == g["printed_sequence_times_16"]


@pytest.mark.parametrize("P,Q", [(6, 2), (12, 4), (16, 5), (7, 3), (5, 9)])
def test_halton_topology_is_a_circulant_with_q_distinct_peers(P, Q):
    rec = halton_receivers(P, Q)
    want = min(Q, P - 1)
    offs = halton_offsets(P, Q)
    assert len(offs) == len(set(offs)) == want and all(0 < o < P for o in offs)
    for p in range(P):
        assert len(set(rec[p])) == want and p not in rec[p]
        assert sum(p in rec[q] for q in range(P)) == want           # as many senders as receivers
    if Q >= P - 1:
        assert all(sorted(rec[p]) == [q for q in range(P) if q != p] for p in range(P))


def hsb_hand_example(cls=SspOracle, receivers=None):
    g = json.load(open(HSB))
    rec = halton_receivers(g["P"], g["Q"]) if receivers is None else receivers
    o = cls(g["model"], np.array([[g["W0"]]]), g["P"], g["B"], g["staleness"], receivers=rec)
    shares = [lambda t, a=a: {"X": np.array([[a]]), "Y": np.array([[0.0]]), "y": np.array([1])}
              for a in g["pair_difference"]]
    rows = []
    for ev in g["events"]:
        flag = replay(o, [tuple(ev)], shares, g["eta"])[0]
        rows.append((flag, [o.replica(p)[0, 0] for p in range(g["P"])]))
    return g, rows


def hsb_matches(cls=SspOracle, receivers=None):
    g, rows = hsb_hand_example(cls, receivers)
    return ([r[0] for r in rows] == g["accepted"]
            and np.allclose([r[1] for r in rows], g["w_after"], rtol=0, atol=1e-12))


def test_hand_worked_partial_broadcast_schedule():
    assert hsb_matches()


class _StalenessOverEveryWorker(SspOracle):
    """Planted mistake: the pause rule also waits for workers that never send to p."""
    def may_step(self, p):
        return all(self.t[p] - self.tau[p][q] <= self.s for q in range(self.P) if q != p)


class _DeliversAlongMissingEdges(SspOracle):
    """Planted mistake: the topology is ignored when something is delivered."""
    def may_deliver(self, p, q, count=1):
        return p != q and count >= 0 and self.tau[p][q] + count <= self.t[q] and self.tau[p][q] + count <= self.t[p]


def test_planted_mistakes_fail_the_partial_broadcast_example():
    assert not hsb_matches(_StalenessOverEveryWorker)
    assert not hsb_matches(_DeliversAlongMissingEdges)
    assert not hsb_matches(receivers=[[2], [0], [1]])            # the ring the other way round
    # the textbook (bit-reversed) base-2 Halton order would put 5/8 before 3/8
    assert halton_offsets(16, 5)[4] == 6 != 10


def test_full_halton_broadcast_is_the_plain_ssp_oracle():
    wl = workloads.make("mlr_tiny", seed=4, J=4, D=9, P=4, B=2)
    a = SspOracle(wl.model, wl.W0, wl.P, wl.B, 1)
    b = SspOracle(wl.model, wl.W0, wl.P, wl.B, 1, receivers=halton_receivers(wl.P, wl.P - 1))
    for ev in workloads.ssp_proposals(wl.P, 200, seed=4):
        outs = []
        for o in (a, b):
            if ev[0] == "step":
                outs.append(o.t[ev[1]] < 8 and o.worker_step(
                    ev[1], workloads.worker_share(wl.model, wl.batch(o.t[ev[1]]), ev[1], wl.B), wl.eta) is not None)
            else:
                outs.append(o.deliver(ev[1], ev[2], ev[3]))
        assert outs[0] == outs[1]
    for p in range(wl.P):
        np.testing.assert_array_equal(a.replica(p), b.replica(p))


def test_send_queue_bounds_how_far_a_sender_runs_ahead_of_a_receiver():
    """Ring 0 -> 1 -> 2 -> 0, staleness 1: worker 0 is paced by its sender 2 only, so worker 1 can
    fall behind in applying worker 0's sets; the queue stops worker 0 when it holds `queue` of them."""
    wl = workloads.make("mlr_tiny", seed=6, J=3, D=5, P=3, B=2)
    o = SspOracle(wl.model, wl.W0, wl.P, wl.B, 1, receivers=halton_receivers(3, 1), queue=3)
    share = lambda p: workloads.worker_share(wl.model, wl.batch(o.t[p]), p, wl.B)
    steps0 = 0
    for _ in range(10):
        for p in (1, 2):                                     # 1 and 2 keep going as far as they may ...
            if o.may_step(p):
                o.worker_step(p, share(p), wl.eta)
        while o.may_deliver(0, 2, 1):                        # ... and worker 0 receives everything from 2
            o.deliver(0, 2, 1)
        while o.may_deliver(2, 1, 1):
            o.deliver(2, 1, 1)
        if o.worker_step(0, share(0), wl.eta) is not None:   # but worker 1 never applies worker 0's sets
            steps0 += 1
    # the staleness chain alone (1 waits for 0's sets, 2 for 1's, 0 for 2's) would allow a fourth
    assert steps0 == 3 and o.queue_full(0) and o.t[0] - o.tau[1][0] == 3
    assert all(o.t[0] - o.tau[0][q] <= o.s for q in o.senders[0])
    assert o.deliver(1, 0, 1) and not o.queue_full(0) and o.may_step(0)
