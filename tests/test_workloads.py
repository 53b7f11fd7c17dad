"""The seeded input recipes: determinism, shapes, storage types, structure."""
import numpy as np
import pytest

import workloads


def test_same_seed_same_arrays_and_different_seed_differs():
    a, b, c = workloads.make("mlr_tiny"), workloads.make("mlr_tiny"), workloads.make("mlr_tiny", seed=1)
    assert np.array_equal(a.W0, b.W0) and not np.array_equal(a.W0, c.W0)
    for x, y in zip(a.batches, b.batches):
        assert np.array_equal(x["A"], y["A"]) and np.array_equal(x["y"], y["y"])
    assert len(a.batches) == 4 and a.batch(5) is a.batches[1]


def test_mlr_tiny_shapes_and_statistics():
    wl = workloads.make("mlr_tiny")
    assert (wl.J, wl.D, wl.P, wl.B, wl.N, wl.steps, wl.eta) == (10, 100, 4, 16, 64, 5, 0.1)
    b = wl.batch(0)
    assert wl.W0.shape == (10, 100) and wl.W0.dtype == np.float32
    assert b["A"].shape == (64, 100) and b["A"].dtype == np.float32
    assert b["y"].dtype == np.int32 and b["y"].min() >= 0 and b["y"].max() < 10
    assert abs(wl.W0.std() - 0.1) < 0.01                       # N(0, variance 0.01)
    assert abs(b["A"].std() - 0.1) < 0.01                      # N(0,1)/sqrt(100)


def test_bf16_features_are_exactly_representable_and_rounding_is_nearest_even():
    wl = workloads.make("mlr_large", J=16, D=64, P=2, B=4, pool=1)
    a = wl.batch(0)["A"]
    bits = workloads.bf16_bits(a)                               # raises if any low bit is set
    assert bits.dtype == np.uint16 and bits.shape == a.shape
    # ties to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> 1; 1 + 3*2^-8 -> 1 + 2^-6
    _, r = workloads.bf16_round(np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -20]))
    assert list(r) == [1.0, 1 + 2.0 ** -6, 1 + 2.0 ** -7]
    with pytest.raises(ValueError):
        workloads.bf16_bits(np.array([1 + 2.0 ** -12], dtype=np.float32))


def test_zipf_labels_are_bounded_and_head_heavy():
    wl = workloads.make("mlr_large", J=1000, D=8, P=16, B=32, pool=4)
    y = np.concatenate([b["y"] for b in wl.batches])
    assert y.min() >= 0 and y.max() < 1000
    assert (y == 0).mean() > 0.08 and (y < 10).mean() > 0.3     # P(0) ~ 0.13 for J=1000


def test_dml_pairs_have_the_designed_geometry():
    wl = workloads.make("dml", pool=1)
    b = wl.batch(0)
    assert b["X"].shape == (1024, 4096) and b["Y"].shape == (1024, 4096)
    assert set(np.unique(b["y"])) == {0, 1} and 0.4 < b["y"].mean() < 0.6
    d2 = ((b["X"].astype(np.float64) - b["Y"]) ** 2).sum(axis=1)
    assert abs(d2[b["y"] == 1].mean() - 2.0) < 0.1              # similar: 2/D per coordinate
    assert abs(d2[b["y"] == 0].mean() - 6.8) < 0.5              # dissimilar: (2*2.4 + 2)/D
    assert abs(wl.W0.var() * 4096 - 1.0) < 0.05


def test_l2svm_csr_rows_are_sorted_distinct_fixed_density():
    wl = workloads.make("l2svm", pool=1)
    b = wl.batch(0)
    assert b["rowptr"].dtype == np.int32 and b["col"].dtype == np.int32 and b["val"].dtype == np.float32
    assert b["rowptr"][0] == 0 and b["rowptr"][-1] == b["col"].size == 1024 * 164
    assert np.all(np.diff(b["rowptr"]) == 164)
    col = b["col"].reshape(1024, 164)
    assert np.all(np.diff(col, axis=1) > 0) and col.min() >= 0 and col.max() < 8192
    assert np.all(b["val"] >= 0)
