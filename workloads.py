"""Seeded synthetic inputs for the SFB hot path.

This module only draws random inputs and casts them to the storage types the
device path reads.  It contains none of the method's arithmetic and is the
one piece shared by the oracle-side tests and the HIP-side tests / bench.

The shapes stand in for the paper's workloads (Section 6.1: Wikipedia tf-idf
for MLR, ImageNet LLC features for DML), which are not available here: dense
Gaussian features scaled by 1/sqrt(D), uniform or Zipf labels, Gaussian
cluster pairs for DML, fixed-density CSR rows for the sparse L2-SVM case.

Draw order for a given seed (numpy.random.default_rng(seed)), fixed so that
any two callers see identical arrays: W0 first, then for each pool batch in
order: features, then labels.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

CONFIGS = {
    # name: model, J, D, P workers, B samples per worker, learning rate, steps, input dtype
    "mlr_tiny":   dict(model="mlr",   J=10,    D=100,   P=4,  B=16,  eta=0.1, steps=5,   dtype="f32"),
    "mlr_medium": dict(model="mlr",   J=1000,  D=4096,  P=8,  B=64,  eta=0.1, steps=100, dtype="f32"),
    "mlr_large":  dict(model="mlr",   J=10000, D=21504, P=16, B=32,  eta=0.1, steps=20,  dtype="bf16",
                       labels="zipf"),
    "dml":        dict(model="dml",   J=600,   D=4096,  P=8,  B=128, eta=0.1, steps=20,  dtype="f32"),
    "l2svm":      dict(model="l2svm", J=2000,  D=8192,  P=16, B=64,  eta=0.1, steps=20,  dtype="f32",
                       density=0.02),
}

SDCA_CONFIGS = {
    # name: classes J, features D, data samples N_data, P workers, B samples per worker, l2 weight lam, steps, dtype
    "sdca_tiny":   dict(J=10,   D=100,  n_data=256,  P=4, B=16, lam=1e-2, steps=8,  dtype="f32"),
    "sdca_medium": dict(J=1000, D=4096, n_data=8192, P=8, B=64, lam=1e-4, steps=20, dtype="f32"),
}

DML_CLUSTERS = 50
DML_CENTRE_VAR = 2.4   # times 1/D
DML_POINT_VAR = 1.0    # times 1/D
ZIPF_EXPONENT = 1.1


def bf16_round(x):
    """Round to the nearest bf16 (ties to even).  Returns (uint16 bits, float32 values)."""
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    b = x32.view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    bits = r.astype(np.uint16)
    back = (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return bits, back.reshape(x32.shape)


def bf16_bits(x32):
    """Bit pattern of float32 values that are already exactly bf16-representable."""
    b = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    if np.any(b & np.uint32(0xFFFF)):
        raise ValueError("values are not bf16-representable")
    return (b >> np.uint32(16)).astype(np.uint16)


@dataclass
class Workload:
    name: str
    model: str
    J: int
    D: int
    P: int
    B: int
    eta: float
    steps: int
    dtype: str                      # storage type of the features: "f32" or "bf16"
    W0: np.ndarray                  # [J, D] float32
    batches: list = field(default_factory=list)

    @property
    def N(self):
        return self.P * self.B

    def batch(self, t):
        """Batch used at step t: the pool is cycled."""
        return self.batches[t % len(self.batches)]


def _cast_features(x64, dtype):
    if dtype == "f32":
        return x64.astype(np.float32)
    if dtype == "bf16":
        return bf16_round(x64)[1]   # float32 array holding exactly bf16-representable values
    raise ValueError(dtype)


def _labels(rng, cfg, n):
    J = cfg["J"]
    if cfg.get("labels") == "zipf":
        # bounded Zipf: P(c) proportional to (c+1)^-1.1 over the J classes
        w = (np.arange(J, dtype=np.float64) + 1.0) ** (-ZIPF_EXPONENT)
        return rng.choice(J, size=n, p=w / w.sum()).astype(np.int32)
    return rng.integers(0, J, size=n).astype(np.int32)


def _mlr_batch(rng, cfg, n):
    D = cfg["D"]
    a = rng.standard_normal((n, D)) / np.sqrt(D)
    y = _labels(rng, cfg, n)
    return {"A": _cast_features(a, cfg["dtype"]), "y": y}


def _dml_batch(rng, cfg, n, centres):
    D = cfg["D"]
    sd = np.sqrt(DML_POINT_VAR / D)
    ca = rng.integers(0, DML_CLUSTERS, size=n)
    shift = rng.integers(1, DML_CLUSTERS, size=n)
    x = centres[ca] + sd * rng.standard_normal((n, D))
    noise_y = sd * rng.standard_normal((n, D))
    sim = rng.integers(0, 2, size=n).astype(np.int32)   # 1 = similar, 0 = dissimilar
    cb = np.where(sim == 1, ca, (ca + shift) % DML_CLUSTERS)
    yv = centres[cb] + noise_y
    return {"X": _cast_features(x, cfg["dtype"]), "Y": _cast_features(yv, cfg["dtype"]), "y": sim}


def _l2svm_batch(rng, cfg, n):
    D = cfg["D"]
    per_row = int(round(cfg["density"] * D))
    col = np.empty((n, per_row), dtype=np.int32)
    for r in range(n):
        col[r] = np.sort(rng.choice(D, size=per_row, replace=False))
    val = np.abs(rng.standard_normal((n, per_row))).astype(np.float32)
    y = _labels(rng, cfg, n)
    rowptr = (np.arange(n + 1, dtype=np.int64) * per_row).astype(np.int32)
    return {"rowptr": rowptr, "col": col.reshape(-1), "val": val.reshape(-1), "D": D, "y": y}


def make(name, seed=0, pool=None, **override):
    """Build the named workload.  ``override`` replaces config fields (J, D, P, B, ...)
    to make ragged or scaled variants of the same recipe."""
    cfg = dict(CONFIGS[name])
    cfg.update(override)
    rng = np.random.default_rng(seed)
    J, D, P, B = cfg["J"], cfg["D"], cfg["P"], cfg["B"]
    n = P * B
    model = cfg["model"]
    if model == "dml":
        W0 = rng.standard_normal((J, D)) * np.sqrt(1.0 / D)       # N(0, variance 1/D)
    else:
        W0 = rng.standard_normal((J, D)) * 0.1                    # N(0, variance 0.01)
    W0 = W0.astype(np.float32)
    n_pool = pool if pool is not None else min(cfg["steps"], 4)
    centres = None
    if model == "dml":
        centres = np.sqrt(DML_CENTRE_VAR / D) * rng.standard_normal((DML_CLUSTERS, D))
    batches = []
    for _ in range(n_pool):
        if model == "mlr":
            batches.append(_mlr_batch(rng, cfg, n))
        elif model == "dml":
            batches.append(_dml_batch(rng, cfg, n, centres))
        elif model == "l2svm":
            batches.append(_l2svm_batch(rng, cfg, n))
        else:
            raise ValueError(model)
    return Workload(name=name, model=model, J=J, D=D, P=P, B=B, eta=cfg["eta"], steps=cfg["steps"],
                    dtype=cfg["dtype"], W0=W0, batches=batches)


def worker_share(model, batch, p, B):
    """Worker p's B samples of a batch (rows [p*B, (p+1)*B)), in the batch's own storage."""
    rows = slice(p * B, (p + 1) * B)
    if model == "mlr":
        return {"A": batch["A"][rows], "y": batch["y"][rows]}
    if model == "dml":
        return {"X": batch["X"][rows], "Y": batch["Y"][rows], "y": batch["y"][rows]}
    rp = batch["rowptr"][p * B:(p + 1) * B + 1]
    lo, hi = int(rp[0]), int(rp[-1])
    return {"rowptr": (rp - rp[0]).astype(np.int32), "col": batch["col"][lo:hi], "val": batch["val"][lo:hi],
            "y": batch["y"][rows], "D": batch["D"]}


def ssp_proposals(P, n_events, seed=0, p_step=0.45):
    """A seeded list of PROPOSED schedule events for a stale-synchronous run: ("step", p) or
    ("deliver", p, q, count).  No rule of the method is applied here: whoever replays the list
    decides which proposals are legal and refuses the others."""
    rng = np.random.default_rng(seed)
    events = []
    for _ in range(n_events):
        if rng.random() < p_step:
            events.append(("step", int(rng.integers(P))))
        else:
            p = int(rng.integers(P))
            q = int((p + 1 + rng.integers(P - 1)) % P) if P > 1 else p
            events.append(("deliver", p, q, int(rng.integers(1, 3))))
    return events


@dataclass
class SdcaWorkload:
    """A fixed data set (SDCA keeps one dual vector per data sample) and, per step, the P*B
    distinct sample indices the workers pick (worker-major).  Class-dependent feature means
    make the problem learnable; no arithmetic of the method is applied here."""
    name: str
    J: int
    D: int
    n_data: int
    P: int
    B: int
    lam: float
    steps: int
    dtype: str
    A: np.ndarray                   # [n_data, D] float32 (bf16-representable when dtype == "bf16")
    y: np.ndarray                   # [n_data] int32
    picks: list = field(default_factory=list)     # per step: [P*B] int32, distinct

    @property
    def N(self):
        return self.P * self.B

    def pick(self, t):
        return self.picks[t % len(self.picks)]


def make_sdca(name, seed=0, **override):
    """Draw order: class means, labels, features, then one index set per step."""
    cfg = dict(SDCA_CONFIGS[name])
    cfg.update(override)
    rng = np.random.default_rng(seed)
    J, D, n_data, P, B = cfg["J"], cfg["D"], cfg["n_data"], cfg["P"], cfg["B"]
    if P * B > n_data:
        raise ValueError("a step picks P*B distinct samples: needs P*B <= n_data")
    means = rng.standard_normal((J, D)) / np.sqrt(D)
    y = rng.integers(0, J, size=n_data).astype(np.int32)
    a = means[y] + rng.standard_normal((n_data, D)) / np.sqrt(D)
    picks = [rng.choice(n_data, size=P * B, replace=False).astype(np.int32) for _ in range(cfg["steps"])]
    return SdcaWorkload(name=name, J=J, D=D, n_data=n_data, P=P, B=B, lam=cfg["lam"], steps=cfg["steps"],
                        dtype=cfg["dtype"], A=_cast_features(a, cfg["dtype"]), y=y, picks=picks)
