"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bar: leaf ids and labels bit-exact; float32 scores within 1e-5 relative / 1e-6 absolute."""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

RTOL, ATOL = 1e-5, 1e-6


def _run(forest, X, leaves=True):
    import torch
    import paper_2301_13441_amd as pk
    f = pk.forest_load(forest)
    try:
        xd = torch.from_numpy(np.ascontiguousarray(X)).cuda()
        scores, labels = f.predict(xd)
        lv = f.predict_leaves(xd) if leaves and forest.n_trees > 0 else None
        torch.cuda.synchronize()
        return (None if scores is None else scores.cpu().numpy(),
                None if labels is None else labels.cpu().numpy(),
                None if lv is None else lv.cpu().numpy(), f.info)
    finally:
        f.close()


def _check(forest, X, leaves=True):
    ref = oracle.predict(forest, X, want_leaves=leaves, n_threads=8)
    scores, labels, lv, info = _run(forest, X, leaves)
    if lv is not None:
        np.testing.assert_array_equal(lv, ref.leaf_node_id)
    if labels is not None:
        np.testing.assert_array_equal(labels, ref.labels)
    if scores is not None:
        np.testing.assert_allclose(scores, ref.scores, rtol=RTOL, atol=ATOL)
    return info


@pytest.mark.parametrize("name,rows,trees,kind", [
    ("c1", 1000, None, 4),        # the whole small configuration
    ("c2", 1000, 40, 8),          # depth 8: 8 outcome words per (row, tree)
    ("c3", 777, 100, 6),          # ragged tail: 777 = 12 tiles + 9 rows
    ("c4", 600, 200, 6),          # 10 classes, softmax + argmax, 30 % zeros in X
    ("c5", 300, 8, 0),            # deep irregular trees, vector leaves
])
def test_configs_small(name, rows, trees, kind):
    w = wl.make_workload(name, n_rows=rows, n_trees=trees)
    info = _check(w.forest, w.make_x(rows))
    assert info["kernel_kind"] == kind


@pytest.mark.parametrize("depth", [1, 2, 3, 5, 7])
def test_full_depths(depth):
    rng = np.random.default_rng(depth)
    arrs = wl._full_forest(rng, 9, depth, 6, wl._normal_thr,
                           lambda r, s: r.standard_normal(s, dtype=np.float32))
    f = wl.Forest(n_features=6, n_outputs=1, leaf_width=1, tree_output=np.zeros(9, np.int32),
                  aggregate=wl.AGG_SUM, transform=wl.TRANSFORM_SIGMOID, **arrs)
    X = rng.standard_normal((333, 6)).astype(np.float32)
    assert _check(f, X)["kernel_kind"] == depth


@pytest.mark.parametrize("seed", range(4))
def test_irregular_forests_with_ties(seed):
    f = wl.random_forest(500 + seed, n_trees=13, n_features=5, max_depth=9, stop_prob=0.2,
                         n_outputs=3, leaf_width=(1 if seed % 2 else 3), grid_thresholds=True,
                         transform=wl.TRANSFORM_SOFTMAX, aggregate=wl.AGG_MEAN)
    rng = np.random.default_rng(seed)
    X = (rng.integers(-3, 4, size=(200, 5)).astype(np.float32) * np.float32(0.5))
    assert _check(f, X)["kernel_kind"] == 0


def test_special_values_nan_inf_signed_zero():
    w = wl.make_workload("c1", n_rows=256)
    X = w.make_x(256).copy()
    rng = np.random.default_rng(9)
    special = np.asarray([np.nan, np.inf, -np.inf, 0.0, -0.0, 1e-45, -1e-45], np.float32)
    mask = rng.random(X.shape) < 0.3
    X[mask] = special[rng.integers(0, len(special), size=int(mask.sum()))]
    f = w.forest
    thr = f.threshold.copy()
    internal = np.flatnonzero(f.feature >= 0)
    thr[internal[::7]] = np.inf
    thr[internal[3::11]] = -np.inf
    thr[internal[5::13]] = -0.0
    g = wl.Forest(**{**f.__dict__, "threshold": thr})
    _check(g, X)


def test_empty_and_single_row_and_single_leaf_trees():
    import torch
    import paper_2301_13441_amd as pk
    w = wl.make_workload("c1", n_rows=1)
    _check(w.forest, w.make_x(1))
    f = pk.forest_load(w.forest)
    f.predict_raw(0, 0, 0, 0)           # n_rows == 0 is a successful no-op
    f.close()
    # forest of single-leaf trees (root is a leaf) plus one stump
    g = wl.random_forest(77, n_trees=5, n_features=3, max_depth=0)
    X = np.zeros((70, 3), np.float32)
    assert _check(g, X)["kernel_kind"] == 0
    torch.cuda.synchronize()


def test_repeated_runs_are_bit_identical():
    import torch
    import paper_2301_13441_amd as pk
    w = wl.make_workload("c4", n_rows=2000, n_trees=300)
    xd = torch.from_numpy(w.make_x(2000)).cuda()
    f = pk.forest_load(w.forest)
    a, la = f.predict(xd)
    a, la = a.clone(), la.clone()
    for _ in range(3):
        b, lb = f.predict(xd)
        assert torch.equal(a, b) and torch.equal(la, lb)
    f.close()
