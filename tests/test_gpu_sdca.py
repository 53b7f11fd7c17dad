"""GPU parity of SFB driven by SDCA (Section 2.1, "Stochastic DCA") against oracle/sdca_oracle.py:
the broadcast factors (delta u_i, a_i), the dual vectors, the conjugate terms, the per-sample
losses and W after every iteration, through the C ABI."""
import numpy as np
import pytest
import torch

import workloads
from gpu_util import assert_close
from oracle.sdca_oracle import SdcaMlrOracle, safe_fraction

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def sfb():
    import paper_1511_08486_amd as m
    return m


def safe_s(wl):
    return safe_fraction(wl.lam, wl.n_data, wl.N, float((wl.A.astype(np.float64) ** 2).sum(1).max()))


class Device:
    """The data set and the SDCA state in device memory; the batch of a step is gathered by
    torch indexing (plumbing: the library sees a plain [N][D] batch and the index list)."""
    def __init__(self, sfb, wl, pad=0, with_conj=True):
        self.sfb, self.wl = sfb, wl
        self.ctx = sfb.Sfb("mlr", wl.J, wl.D, wl.P, wl.B, dtype=wl.dtype, device=DEV)
        vdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
        self.A = torch.from_numpy(wl.A).to(vdt).to(DEV)
        self.y = torch.from_numpy(wl.y).to(DEV)
        self.W = torch.zeros((wl.J, wl.D + pad), dtype=torch.float32, device=DEV)[:, :wl.D]
        self.dual = torch.zeros((wl.n_data, wl.J + pad), dtype=torch.float32, device=DEV)[:, :wl.J]
        self.conj = torch.zeros(wl.n_data, dtype=torch.float32, device=DEV) if with_conj else None
        nan = float("nan")
        self.U = torch.full((wl.N, wl.J + pad), nan, dtype=torch.float32, device=DEV)[:, :wl.J]
        self.V = torch.full((wl.N, wl.D + pad), nan, dtype=vdt, device=DEV)[:, :wl.D]
        self.loss = torch.full((wl.N,), nan, dtype=torch.float32, device=DEV)

    def step(self, picked, s, split=False):
        idx = torch.from_numpy(np.ascontiguousarray(picked, dtype=np.int32)).to(DEV)
        batch = self.sfb.SfbBatch(a=self.A[idx.long()].contiguous())
        yb = self.y[idx.long()].contiguous()
        if split:
            self.ctx.sdca_compute_factors(self.W, batch, yb, self.dual, idx, self.wl.lam, s, self.U, self.V,
                                          loss=self.loss, conj=self.conj)
            self.ctx.reconstruct_apply(self.W, self.U, self.V, 1.0, scale=1.0 / (self.wl.lam * self.wl.n_data))
        else:
            self.ctx.sdca_step(self.W, batch, yb, self.dual, idx, self.wl.lam, s, self.U, self.V, loss=self.loss,
                               conj=self.conj)
        self.ctx.sync()


def run_parity(sfb, wl, steps, tol, s=None, pad=0, matrix=False, split_at=()):
    s = safe_s(wl) if s is None else s
    d = Device(sfb, wl, pad=pad)
    o = SdcaMlrOracle(wl.A, wl.y, wl.J, wl.lam)
    worst = {}
    for t in range(steps):
        pk = wl.pick(t)
        d.step(pk, s, split=t in split_at)
        delta, losses = (o.step_matrix if matrix else o.step)(pk, s)
        got = {"dU": d.U.cpu().numpy(), "V": d.V.float().cpu().numpy(), "loss": d.loss.cpu().numpy(),
               "W": d.W.cpu().numpy(), "dual": d.dual.cpu().numpy(), "conj": d.conj.cpu().numpy()}
        conj = o.conjugate_terms() if not matrix or t == steps - 1 else None
        want = {"dU": delta, "V": wl.A[pk].astype(np.float64), "loss": losses, "W": o.W, "dual": o.U}
        if conj is not None:
            want["conj"] = conj
        for k, w in want.items():
            worst[k] = max(worst.get(k, 0.0), assert_close(got[k], w, tol, f"{k} step {t}"))
    d.ctx.close()
    return worst


def test_tiny_chain(sfb):
    wl = workloads.make_sdca("sdca_tiny")
    worst = run_parity(sfb, wl, wl.steps, 1e-4, split_at=(2, 5))
    print("sdca_tiny worst error / allowance:", worst)


def test_ragged_shapes_and_padded_rows(sfb):
    """Nothing a multiple of a tile; rows of W, U, V and of the dual matrix padded by 3 floats
    (so no 16-byte aligned rows anywhere)."""
    wl = workloads.make_sdca("sdca_tiny", seed=1, J=37, D=203, n_data=300, P=3, B=7, lam=3e-3, steps=6)
    run_parity(sfb, wl, 6, 1e-4, pad=3)


@pytest.mark.parametrize("s", [1.0, 1e-3])
def test_extreme_fractions(sfb, s):
    """s = 1 jumps to the optimal dual vector (the old one drops out); a tiny s barely moves."""
    wl = workloads.make_sdca("sdca_tiny", seed=2, J=12, D=64, n_data=128, P=2, B=16, lam=0.5, steps=4)
    run_parity(sfb, wl, 4, 1e-4, s=s)


def test_wide_rows(sfb):
    """J beyond one 128-bit item per thread (register-resident rows of 1500) and beyond the
    register-resident kernels altogether (12400)."""
    wl = workloads.make_sdca("sdca_tiny", seed=3, J=1500, D=96, n_data=96, P=2, B=12, lam=1e-2, steps=3)
    run_parity(sfb, wl, 3, 1e-4, matrix=True)
    wl = workloads.make_sdca("sdca_tiny", seed=4, J=12400, D=64, n_data=48, P=2, B=8, lam=1e-2, steps=2)
    run_parity(sfb, wl, 2, 1e-4, matrix=True)


def test_medium_shape(sfb):
    """The mlr_medium tile shapes (J=1000, D=4096, 8 x 64 picked samples) on a data set of 2048."""
    wl = workloads.make_sdca("sdca_medium", n_data=2048, steps=3)
    worst = run_parity(sfb, wl, 3, 1e-4, matrix=True)
    print("sdca_medium worst error / allowance:", worst)


def test_bf16_features(sfb):
    """bf16 features and V on the bf16 matrix cores; dual vectors, U and W stay fp32."""
    wl = workloads.make_sdca("sdca_tiny", seed=5, J=512, D=1024, n_data=1024, P=16, B=32, lam=1e-3, steps=3,
                             dtype="bf16")
    run_parity(sfb, wl, 3, 2e-2, matrix=True)


def test_unpicked_samples_are_untouched_and_conj_is_optional(sfb):
    wl = workloads.make_sdca("sdca_tiny", seed=6)
    d = Device(sfb, wl, with_conj=False)
    d.dual.fill_(0.125)
    before = d.dual.clone()
    pk = wl.pick(0)
    d.step(pk, 0.5)
    rest = np.setdiff1d(np.arange(wl.n_data), pk)
    assert torch.equal(d.dual[rest], before[rest])
    assert not torch.equal(d.dual[pk], before[pk])
    d.ctx.close()


def test_converges_to_the_primal_minimiser_on_the_device(sfb):
    """A long run on a small problem: the duality gap rebuilt from what the device holds (W, the
    dual vectors, the conjugate terms) closes, and W is the oracle's W."""
    wl = workloads.make_sdca("sdca_tiny", seed=7, J=3, D=5, n_data=24, P=2, B=3, lam=0.05, steps=1500)
    s = safe_s(wl)
    d = Device(sfb, wl)
    o = SdcaMlrOracle(wl.A, wl.y, wl.J, wl.lam)
    for t in range(1500):
        d.step(wl.pick(t), s)
        o.step_matrix(wl.pick(t), s)
    W = d.W.cpu().numpy().astype(np.float64)
    assert_close(W, o.W, 1e-4, "W after 1500 iterations")
    A, y = torch.tensor(wl.A, dtype=torch.float64), torch.tensor(wl.y, dtype=torch.int64)
    primal = float(torch.nn.functional.cross_entropy(A @ torch.tensor(W).T, y)) + 0.5 * wl.lam * float((W * W).sum())
    Z = d.dual.cpu().numpy().astype(np.float64).T @ wl.A.astype(np.float64) / wl.n_data
    dual = float(d.conj.cpu().numpy().astype(np.float64).mean()) + float((Z * Z).sum()) / (2 * wl.lam)
    assert abs(primal + dual) < 1e-5, (primal, dual)
    assert o.gap() < 1e-9
    # the primal-dual tie on the device: lam W = (1/n) sum u_i a_i^T
    assert_close(wl.lam * W, Z, 1e-4, "lam W against the dual vectors")
    d.ctx.close()
