"""Seeded synthetic workloads: forests (as raw per-node arrays) and feature matrices.

This module only draws random numbers and lays them out as arrays.  It holds none of the
inference arithmetic: no traversal, no packing, no reduction.  Both the CPU oracle's tests
and the GPU path's tests/bench import it so that the two sides see byte-identical inputs.

The five configurations stand in for the paper's evaluation data (YearPrediction, 515 345
samples x 90 features, Section 5.1 "Experimental Setup") and its trained scikit-learn
models, whose hyper-parameters the paper does not state.  Every array comes from
``numpy.random.default_rng(seed)`` with a fixed draw order so a workload is reproducible
from its seed alone.

Forest description (a plain dict of numpy arrays, "caller's node arrays"):
    tree_offset  int64 [T+1]   node range of each tree; the root is the first node of a range
    feature      int32 [n]     split feature of an internal node, -1 for a leaf
    threshold    float32 [n]   split threshold (a row goes LEFT iff x[feature] <= threshold)
    left, right  int32 [n]     tree-local child indices (ignored at leaves)
    leaf_value   float32 [n, leaf_width]   payload of a leaf (ignored at internal nodes)
    tree_output  int32 [T]     output column a scalar-leaf tree adds into
plus scalars: n_features, n_outputs (K), leaf_width, aggregate, base_score, transform, output.
"""
from __future__ import annotations

import statistics
from dataclasses import dataclass, field
from typing import Iterator, Optional

import numpy as np

AGG_SUM, AGG_MEAN = 0, 1
TRANSFORM_NONE, TRANSFORM_SIGMOID, TRANSFORM_SOFTMAX = 0, 1, 2
OUT_SCORES, OUT_LABELS, OUT_BOTH = 0, 1, 2

X_CHUNK_ROWS = 65536  # X is drawn in chunks of this many rows so every row prefix is reproducible

SEEDS = {"c1": 13441001, "c2": 13441002, "c3": 13441003, "c4": 13441004, "c5": 13441005}
FULL_ROWS = {"c1": 1_000, "c2": 1_000_000, "c3": 1_000_000, "c4": 500_000, "c5": 4_000_000}


@dataclass
class Forest:
    n_features: int
    n_outputs: int
    leaf_width: int
    tree_offset: np.ndarray
    feature: np.ndarray
    threshold: np.ndarray
    left: np.ndarray
    right: np.ndarray
    leaf_value: np.ndarray
    tree_output: np.ndarray
    aggregate: int = AGG_SUM
    base_score: Optional[np.ndarray] = None
    transform: int = TRANSFORM_NONE
    output: int = OUT_BOTH

    @property
    def n_trees(self) -> int:
        return len(self.tree_offset) - 1

    @property
    def n_nodes(self) -> int:
        return int(self.tree_offset[-1])


@dataclass
class Workload:
    name: str
    seed: int
    forest: Forest
    n_rows: int
    zero_fraction: float = 0.0
    _rng_state_after_model: dict = field(default_factory=dict, repr=False)

    def x_chunks(self, n_rows: Optional[int] = None) -> Iterator[np.ndarray]:
        """Yield X in row chunks (float32, C-contiguous). Same rows for any prefix length."""
        n = self.n_rows if n_rows is None else n_rows
        rng = np.random.default_rng(self.seed)
        rng.bit_generator.state = self._rng_state_after_model
        F = self.forest.n_features
        done = 0
        while done < n:
            x = rng.standard_normal((X_CHUNK_ROWS, F), dtype=np.float32)
            if self.zero_fraction > 0.0:
                mask = rng.random((X_CHUNK_ROWS, F)) < self.zero_fraction
                x[mask] = np.float32(0.0)
            take = min(X_CHUNK_ROWS, n - done)
            yield x[:take]
            done += take

    def make_x(self, n_rows: Optional[int] = None) -> np.ndarray:
        n = self.n_rows if n_rows is None else n_rows
        out = np.empty((n, self.forest.n_features), dtype=np.float32)
        pos = 0
        for c in self.x_chunks(n):
            out[pos:pos + len(c)] = c
            pos += len(c)
        return out


# --------------------------------------------------------------------------------------
# tree-shape helpers (structure only)
# --------------------------------------------------------------------------------------

def full_tree_arrays(depth: int):
    """Child indices of a full binary tree stored breadth-first (root = 0).

    Returns (is_leaf [n] bool, left [n], right [n]) with n = 2**(depth+1) - 1.
    """
    n_int = (1 << depth) - 1
    n = (1 << (depth + 1)) - 1
    idx = np.arange(n, dtype=np.int32)
    is_leaf = idx >= n_int
    left = np.where(is_leaf, -1, 2 * idx + 1).astype(np.int32)
    right = np.where(is_leaf, -1, 2 * idx + 2).astype(np.int32)
    return is_leaf, left, right


def _full_forest(rng, n_trees, depth, n_features, thr_draw, leaf_draw, leaf_width=1):
    """Forest of full trees; draw order: all features, all thresholds, all leaf payloads."""
    is_leaf, left, right = full_tree_arrays(depth)
    n = len(is_leaf)
    n_int = int((~is_leaf).sum())
    n_leaf = n - n_int
    feats = rng.integers(0, n_features, size=(n_trees, n_int), dtype=np.int64).astype(np.int32)
    thrs = thr_draw(rng, (n_trees, n_int), feats)
    leaves = leaf_draw(rng, (n_trees, n_leaf))
    feature = np.full((n_trees, n), -1, dtype=np.int32)
    feature[:, :n_int] = feats
    threshold = np.zeros((n_trees, n), dtype=np.float32)
    threshold[:, :n_int] = thrs
    leaf_value = np.zeros((n_trees, n, leaf_width), dtype=np.float32)
    leaf_value[:, n_int:, :] = leaves.reshape(n_trees, n_leaf, leaf_width)
    tree_offset = (np.arange(n_trees + 1, dtype=np.int64) * n)
    return dict(
        tree_offset=tree_offset,
        feature=feature.reshape(-1),
        threshold=threshold.reshape(-1),
        left=np.tile(left, n_trees),
        right=np.tile(right, n_trees),
        leaf_value=leaf_value.reshape(-1, leaf_width),
    )


def _normal_thr(rng, shape, feats):
    return rng.standard_normal(shape, dtype=np.float32)


def normal_quantile_grid(n_edges: int = 255) -> np.ndarray:
    """Interior edges k/(n_edges+1) of the standard normal, rounded once to float32."""
    nd = statistics.NormalDist()
    q = [nd.inv_cdf(k / (n_edges + 1)) for k in range(1, n_edges + 1)]
    return np.asarray(q, dtype=np.float64).astype(np.float32)


def _quantile_thr(rng, shape, feats):
    grid = normal_quantile_grid(255)
    k = rng.integers(0, len(grid), size=shape)
    return grid[k]


def _random_tree_structure(rng, max_depth, stop_prob, min_leaves, max_leaves):
    """One tree grown by random stopping, nodes in pre-order; redrawn until the leaf count fits.

    Every attempt draws a block of 2**(max_depth+1)-1 uniforms and consumes them in
    pre-order: a node at depth < max_depth is a leaf iff its uniform < stop_prob.
    """
    cap = (1 << (max_depth + 1)) - 1
    while True:
        u = rng.random(cap)
        is_leaf, left, right = [], [], []
        # explicit stack of (node index, depth, which child of parent, parent)
        stack = [(0, -1, -1)]  # (depth, parent, side)
        pos = 0
        while stack:
            depth, parent, side = stack.pop()
            me = len(is_leaf)
            if parent >= 0:
                (left if side == 0 else right)[parent] = me
            leaf = depth >= max_depth or u[pos] < stop_prob
            pos += 1
            is_leaf.append(leaf)
            left.append(-1)
            right.append(-1)
            if not leaf:
                # push right first so the left subtree is numbered first (pre-order)
                stack.append((depth + 1, me, 1))
                stack.append((depth + 1, me, 0))
        n_leaves = sum(is_leaf)
        if min_leaves <= n_leaves <= max_leaves:
            return (np.asarray(is_leaf, dtype=bool), np.asarray(left, dtype=np.int32),
                    np.asarray(right, dtype=np.int32))


# --------------------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------------------

def make_workload(name: str, n_rows: Optional[int] = None, n_trees: Optional[int] = None) -> Workload:
    """Build configuration ``name`` in {"c1".."c5"}.

    ``n_rows`` / ``n_trees`` may shrink the workload for tests; the model arrays of the
    first ``n_trees`` trees are NOT a prefix of the full model (the draws are blocked per
    array), but the result is still a deterministic function of (name, n_trees).
    """
    seed = SEEDS[name]
    rng = np.random.default_rng(seed)
    rows = FULL_ROWS[name] if n_rows is None else n_rows
    uniform_leaf = lambda r, shape: r.random(shape, dtype=np.float32)
    normal_leaf = lambda r, shape: (r.standard_normal(shape, dtype=np.float32) * np.float32(0.1))
    zero_fraction = 0.0

    if name in ("c1", "c2"):
        T = (10 if name == "c1" else 500) if n_trees is None else n_trees
        depth = 4 if name == "c1" else 8
        F = 28
        arrs = _full_forest(rng, T, depth, F, _normal_thr, uniform_leaf)
        forest = Forest(n_features=F, n_outputs=1, leaf_width=1,
                        tree_output=np.zeros(T, dtype=np.int32),
                        aggregate=AGG_MEAN, base_score=None,
                        transform=TRANSFORM_NONE, output=OUT_BOTH, **arrs)
    elif name == "c3":
        T = 1000 if n_trees is None else n_trees
        F = 50
        arrs = _full_forest(rng, T, 6, F, _quantile_thr, normal_leaf)
        forest = Forest(n_features=F, n_outputs=1, leaf_width=1,
                        tree_output=np.zeros(T, dtype=np.int32),
                        aggregate=AGG_SUM, base_score=np.asarray([0.5], dtype=np.float32),
                        transform=TRANSFORM_NONE, output=OUT_SCORES, **arrs)
    elif name == "c4":
        K = 10
        T = 2000 if n_trees is None else n_trees
        F = 128
        arrs = _full_forest(rng, T, 6, F, _normal_thr, normal_leaf)
        forest = Forest(n_features=F, n_outputs=K, leaf_width=1,
                        tree_output=(np.arange(T) % K).astype(np.int32),
                        aggregate=AGG_SUM, base_score=None,
                        transform=TRANSFORM_SOFTMAX, output=OUT_BOTH, **arrs)
        zero_fraction = 0.3
    elif name == "c5":
        T = 128 if n_trees is None else n_trees
        F = 256
        shapes = [_random_tree_structure(rng, 12, 0.15, 500, 2000) for _ in range(T)]
        sizes = np.asarray([len(s[0]) for s in shapes], dtype=np.int64)
        tree_offset = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
        is_leaf = np.concatenate([s[0] for s in shapes])
        left = np.concatenate([s[1] for s in shapes])
        right = np.concatenate([s[2] for s in shapes])
        n = len(is_leaf)
        feats = rng.integers(0, F, size=n, dtype=np.int64).astype(np.int32)
        thrs = rng.standard_normal(n, dtype=np.float32)
        p = rng.random(n, dtype=np.float32)
        feature = np.where(is_leaf, -1, feats).astype(np.int32)
        threshold = np.where(is_leaf, np.float32(0), thrs).astype(np.float32)
        leaf_value = np.zeros((n, 2), dtype=np.float32)
        leaf_value[is_leaf, 0] = (np.float32(1.0) - p)[is_leaf]
        leaf_value[is_leaf, 1] = p[is_leaf]
        forest = Forest(n_features=F, n_outputs=2, leaf_width=2,
                        tree_offset=tree_offset, feature=feature, threshold=threshold,
                        left=left, right=right, leaf_value=leaf_value,
                        tree_output=np.zeros(T, dtype=np.int32),
                        aggregate=AGG_MEAN, base_score=None,
                        transform=TRANSFORM_NONE, output=OUT_BOTH)
    else:
        raise KeyError(name)

    return Workload(name=name, seed=seed, forest=forest, n_rows=rows,
                    zero_fraction=zero_fraction,
                    _rng_state_after_model=rng.bit_generator.state)


def random_forest(seed: int, n_trees: int, n_features: int, max_depth: int,
                  stop_prob: float = 0.3, n_outputs: int = 1, leaf_width: int = 1,
                  aggregate: int = AGG_SUM, transform: int = TRANSFORM_NONE,
                  output: int = OUT_BOTH, allow_single_leaf: bool = True,
                  grid_thresholds: bool = False) -> Forest:
    """Small irregular forests for tests: random shapes, nodes stored in pre-order.

    ``grid_thresholds`` draws thresholds from a coarse grid {-1,-0.5,0,0.5,1} so that test
    rows drawn from the same grid hit the ``x == threshold`` boundary often.
    """
    rng = np.random.default_rng(seed)
    shapes = []
    for _ in range(n_trees):
        lo = 1 if allow_single_leaf else 2
        shapes.append(_random_tree_structure(rng, max_depth, stop_prob, lo, 1 << max_depth))
    sizes = np.asarray([len(s[0]) for s in shapes], dtype=np.int64)
    tree_offset = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    is_leaf = np.concatenate([s[0] for s in shapes])
    n = len(is_leaf)
    feats = rng.integers(0, n_features, size=n).astype(np.int32)
    if grid_thresholds:
        thrs = (rng.integers(-2, 3, size=n).astype(np.float32) * np.float32(0.5))
    else:
        thrs = rng.standard_normal(n, dtype=np.float32)
    vals = (rng.standard_normal((n, leaf_width), dtype=np.float32) * np.float32(0.5))
    return Forest(
        n_features=n_features, n_outputs=n_outputs, leaf_width=leaf_width,
        tree_offset=tree_offset,
        feature=np.where(is_leaf, -1, feats).astype(np.int32),
        threshold=np.where(is_leaf, np.float32(0), thrs).astype(np.float32),
        left=np.concatenate([s[1] for s in shapes]),
        right=np.concatenate([s[2] for s in shapes]),
        leaf_value=np.where(is_leaf[:, None], vals, np.float32(0)).astype(np.float32),
        tree_output=(rng.integers(0, n_outputs, size=n_trees).astype(np.int32)
                     if leaf_width == 1 else np.zeros(n_trees, dtype=np.int32)),
        aggregate=aggregate, base_score=None, transform=transform, output=output)
