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
                                       ("l2svm", dict(J=64, D=512, P=2, B=32))])
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
