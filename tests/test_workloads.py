"""The synthetic workloads have the shapes, sizes and value structure the five benchmark
configurations call for, and are reproducible from their seeds."""
import numpy as np
import pytest

import workloads as wl


@pytest.mark.parametrize("name,T,depth,F,K", [("c1", 10, 4, 28, 1), ("c2", 500, 8, 28, 1),
                                              ("c3", 1000, 6, 50, 1), ("c4", 2000, 6, 128, 10)])
def test_full_depth_configs(name, T, depth, F, K):
    w = wl.make_workload(name, n_rows=8)
    f = w.forest
    assert f.n_trees == T and f.n_features == F and f.n_outputs == K
    per = (1 << (depth + 1)) - 1
    assert f.n_nodes == T * per
    internal = f.feature.reshape(T, per) >= 0
    assert (internal.sum(axis=1) == (1 << depth) - 1).all()
    assert f.feature.max() < F
    assert np.isfinite(f.threshold).all()
    if name == "c4":
        assert (f.tree_output == np.arange(T) % 10).all()
    if name == "c3":
        grid = wl.normal_quantile_grid(255)
        assert np.isin(f.threshold[f.feature >= 0], grid).all()
        assert abs(grid[127]) < 1e-12 and np.all(np.diff(grid) > 0)
        assert f.base_score.tolist() == [0.5] and f.aggregate == wl.AGG_SUM


def test_c5_shapes():
    w = wl.make_workload("c5", n_rows=4)
    f = w.forest
    assert f.n_trees == 128 and f.n_features == 256 and f.leaf_width == 2
    sizes = np.diff(f.tree_offset)
    leaves = (sizes + 1) // 2
    assert (leaves >= 500).all() and (leaves <= 2000).all()
    leaf = f.feature < 0
    np.testing.assert_allclose(f.leaf_value[leaf].sum(axis=1), 1.0, atol=1e-6)
    # depth never exceeds 12: walk down from every root
    for t in range(0, 128, 17):
        a, b = f.tree_offset[t], f.tree_offset[t + 1]
        depth = np.zeros(b - a, dtype=int)
        for n in range(b - a):          # pre-order: parents come before children
            if f.feature[a + n] >= 0:
                depth[f.left[a + n]] = depth[n] + 1
                depth[f.right[a + n]] = depth[n] + 1
        assert depth.max() <= 12


def test_x_is_reproducible_and_prefix_stable():
    w = wl.make_workload("c4", n_rows=70000, n_trees=10)
    a = w.make_x(70000)
    b = wl.make_workload("c4", n_rows=100, n_trees=10).make_x(100)
    np.testing.assert_array_equal(a[:100], b)
    zeros = (a == 0).mean()
    assert 0.29 < zeros < 0.31
    assert not np.signbit(a[a == 0]).any()
    c = wl.make_workload("c2", n_rows=1000).make_x(1000)
    assert c.dtype == np.float32 and c.shape == (1000, 28)
    assert abs(c.mean()) < 0.02 and abs(c.std() - 1) < 0.02
