"""sfb_step only enqueues kernels on its stream (no allocation, no memset, no sync), so a caller
can record it into a HIP graph.  Replays are checked against the eager chain, several times,
with eager work and synchronisations between them."""
import numpy as np
import pytest
import torch

import workloads
from gpu_util import alloc_factors, to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,over", [("mlr_tiny", {}), ("mlr_medium", dict(J=200, D=512, P=4, B=32)),
                                       ("dml", dict(J=96, D=256, P=2, B=64)),
                                       ("l2svm", dict(J=64, D=512, P=2, B=32)),
                                       # padded factor copies, slices of the pairs over workgroups, the adding-up kernel
                                       ("mlr_tiny", dict(J=10, D=784, P=12, B=100))])
def test_step_recorded_in_a_graph_replays_like_eager_steps(name, over):
    import paper_1511_08486_amd as sfb
    dev = "cuda:0"
    wl = workloads.make(name, seed=3, pool=1, **over)
    side = torch.cuda.Stream(device=dev)           # default priority
    with torch.cuda.stream(side):
        ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, dtype=wl.dtype, device=dev)   # bound to `side`
        db, dy = to_device(wl, wl.batch(0), dev)
        W = torch.from_numpy(wl.W0).to(dev)
        U, V, loss = alloc_factors(wl, dev)
        # eager chain of 5 steps on the same batch: the reference
        ref = []
        for _ in range(5):
            ctx.step(W, db, dy, U, V, wl.eta, loss=loss)
            ctx.sync()
            ref.append((W.clone(), U.clone(), loss.clone()))
        W.copy_(torch.from_numpy(wl.W0))
        side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ctx.step(W, db, dy, U, V, wl.eta, loss=loss)
    # the capture itself ran nothing: W is still W0
    torch.cuda.synchronize()
    assert torch.equal(W.cpu(), torch.from_numpy(wl.W0))
    scratch = torch.zeros(1 << 16, device=dev)
    for t in range(5):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(W, ref[t][0]), f"replay {t}: W differs from the eager chain"
        assert torch.equal(U, ref[t][1]) and torch.equal(loss, ref[t][2])
        scratch.add_(1.0)                          # unrelated eager work between replays
        torch.cuda.synchronize()
    ctx.close()


@pytest.mark.parametrize("what", ["step_prox_l1", "step_prox_column_ball", "sdca_step"])
def test_proximal_and_sdca_iterations_replay_like_eager_ones(what):
    """The proximal iteration (fused entrywise operator; column projection with its three kernels
    and workspace) and the SDCA iteration (dual vectors updated in place) are plain launches too."""
    import paper_1511_08486_amd as sfb
    dev = "cuda:0"
    side = torch.cuda.Stream(device=dev)
    with torch.cuda.stream(side):
        if what == "sdca_step":
            wl = workloads.make_sdca("sdca_tiny", seed=2, J=40, D=256, n_data=96, P=2, B=16)
            ctx = sfb.Sfb("mlr", wl.J, wl.D, wl.P, wl.B, device=dev)
            A, yd = torch.from_numpy(wl.A).to(dev), torch.from_numpy(wl.y).to(dev)
            idx = torch.from_numpy(wl.pick(0)).to(dev)
            batch, yb = sfb.SfbBatch(a=A[idx.long()].contiguous()), yd[idx.long()].contiguous()
            W = torch.zeros((wl.J, wl.D), device=dev)
            dual = torch.zeros((wl.n_data, wl.J), device=dev)
            state = [W, dual]
            U = torch.empty((wl.N, wl.J), device=dev)
            V = torch.empty((wl.N, wl.D), device=dev)
            run = lambda: ctx.sdca_step(W, batch, yb, dual, idx, wl.lam, 0.3, U, V)
        else:
            wl = workloads.make("mlr_medium", seed=3, pool=1, J=200, D=512, P=4, B=32)
            ctx = sfb.Sfb(wl.model, wl.J, wl.D, wl.P, wl.B, device=dev)
            batch, yb = to_device(wl, wl.batch(0), dev)
            W = torch.from_numpy(wl.W0).to(dev)
            state = [W]
            U, V, _ = alloc_factors(wl, dev)
            kind, param = ("l1", 1e-3) if what == "step_prox_l1" else ("column_ball", 1.3)
            run = lambda: ctx.step_prox(W, batch, yb, U, V, wl.eta, kind, param)
        start = [s.clone() for s in state]
        ref = []
        for _ in range(4):
            run()
            ctx.sync()
            ref.append([s.clone() for s in state] + [U.clone()])
        for s, s0 in zip(state, start):
            s.copy_(s0)
        side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run()
    torch.cuda.synchronize()
    assert all(torch.equal(s, s0) for s, s0 in zip(state, start))      # the capture ran nothing
    scratch = torch.zeros(1 << 16, device=dev)
    for t in range(4):
        graph.replay()
        torch.cuda.synchronize()
        for s, want in zip(state + [U], ref[t]):
            assert torch.equal(s, want), f"{what}: replay {t} differs from the eager chain"
        scratch.add_(1.0)
        torch.cuda.synchronize()
    ctx.close()
