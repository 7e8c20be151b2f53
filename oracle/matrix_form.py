"""Dense operator representation of a decision tree, for tiny trees.  TEST INFRASTRUCTURE ONLY.

Two formulations, both written with plain numpy matmuls so they can be read against the
paper:

* ``paper_form``  -- Table 2 / Fig. 2: W1 in {0,1}^{N_F x N_I} selects the feature each
  internal node tests, W2 in R^{N_I} holds the thresholds, W3 in {0,1}^{N_I x N_L} is 0 where
  leaf L_j lies in the LEFT subtree of internal node I_i and 1 everywhere else (also for
  leaves outside I_i's subtree: the printed sparsity range [1/2, 1 - 1/N_L] only holds under
  that reading).  Inference is matmul(X, W1) -> greater(., W2) -> matmul(., W3) -> argmax.
  Internal nodes are numbered in level order and leaves in in-order (Section 3.1.2).  The
  paper does not state the argmax tie rule; the FIRST maximiser is the one that makes the
  construction exact (the right-most leaf always ties with the true one), and numpy's argmax
  returns the first.
* ``path_form``   -- the equivalent signed form: A = W1, B = W2, T = (X.A <= B),
  C[i][j] = +1 / -1 / 0 when leaf j is in the left subtree / right subtree / not below
  internal node i, D[j] = number of +1 in column j; row r reaches leaf j iff
  (T.C)[r][j] == D[j]; the prediction is onehot . E.

X must be finite here: a 0/1 matmul is only a gather when 0 * x == 0.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np


@dataclass
class TreeMatrices:
    W1: np.ndarray          # [N_F, N_I] 0/1   (A)
    W2: np.ndarray          # [N_I] float32    (B)
    W3: np.ndarray          # [N_I, N_L] 0/1
    C: np.ndarray           # [N_I, N_L] in {-1, 0, +1}
    D: np.ndarray           # [N_L]
    E: np.ndarray           # [N_L, leaf_width] float32
    internal_nodes: List[int]   # caller node index of I_0.. (level order)
    leaf_nodes: List[int]       # caller node index of L_0.. (in-order)


def _level_order_internal(feature, left, right) -> List[int]:
    order, frontier = [], [0]
    while frontier:
        nxt = []
        for n in frontier:
            if feature[n] >= 0:
                order.append(n)
                nxt.append(int(left[n]))
                nxt.append(int(right[n]))
        frontier = nxt
    return order


def _in_order_leaves(feature, left, right) -> List[int]:
    out, stack, n = [], [], 0
    # iterative in-order walk: left subtree, node, right subtree; only leaves are recorded
    while True:
        while feature[n] >= 0:
            stack.append(n)
            n = int(left[n])
        out.append(n)
        if not stack:
            return out
        n = int(right[stack.pop()])


def _leaves_below(node, feature, left, right) -> List[int]:
    out, todo = [], [node]
    while todo:
        n = todo.pop()
        if feature[n] >= 0:
            todo.append(int(left[n]))
            todo.append(int(right[n]))
        else:
            out.append(n)
    return out


def tree_matrices(n_features, feature, threshold, left, right, leaf_value) -> TreeMatrices:
    """Build W1, W2, W3 (Table 2) and C, D, E for one tree given as tree-local arrays."""
    internal = _level_order_internal(feature, left, right)
    leaves = _in_order_leaves(feature, left, right)
    leaf_col = {n: j for j, n in enumerate(leaves)}
    n_i, n_l = len(internal), len(leaves)
    W1 = np.zeros((n_features, n_i), dtype=np.int8)
    W2 = np.zeros((n_i,), dtype=np.float32)
    W3 = np.ones((n_i, n_l), dtype=np.int8)
    C = np.zeros((n_i, n_l), dtype=np.int8)
    for i, n in enumerate(internal):
        W1[int(feature[n]), i] = 1
        W2[i] = threshold[n]
        for leaf in _leaves_below(int(left[n]), feature, left, right):
            W3[i, leaf_col[leaf]] = 0
            C[i, leaf_col[leaf]] = 1
        for leaf in _leaves_below(int(right[n]), feature, left, right):
            C[i, leaf_col[leaf]] = -1
    D = (C == 1).sum(axis=0).astype(np.int32)
    E = np.asarray([leaf_value[n] for n in leaves], dtype=np.float32).reshape(n_l, -1)
    return TreeMatrices(W1, W2, W3, C, D, E, internal, leaves)


def paper_form_leaf(X: np.ndarray, m: TreeMatrices) -> np.ndarray:
    """matmul -> greater -> matmul -> argmax; returns the in-order leaf number per row."""
    G = X.astype(np.float64) @ m.W1.astype(np.float64)           # (1) reorganisation as matmul
    S = (G.astype(np.float32) > m.W2[None, :])                    # (2) element-wise greater
    P = S.astype(np.int32) @ m.W3.astype(np.int32)                # (3) matmul ...
    return np.argmax(P, axis=1).astype(np.int32)                  #     ... and (first) argmax


def path_form_onehot(X: np.ndarray, m: TreeMatrices) -> np.ndarray:
    """(X.A <= B) . C == D; returns the boolean [rows, N_L] match matrix."""
    G = X.astype(np.float64) @ m.W1.astype(np.float64)
    T = (G.astype(np.float32) <= m.W2[None, :])
    M = T.astype(np.int32) @ m.C.astype(np.int32)
    return M == m.D[None, :]


def split_trees(forest):
    """Yield tree-local (feature, threshold, left, right, leaf_value) slices of a forest."""
    for t in range(len(forest.tree_offset) - 1):
        a, b = int(forest.tree_offset[t]), int(forest.tree_offset[t + 1])
        yield (forest.feature[a:b], forest.threshold[a:b], forest.left[a:b],
               forest.right[a:b], forest.leaf_value[a:b])


def forest_raw_scores(forest, X: np.ndarray, use: str = "path") -> np.ndarray:
    """Per-column fp64 raw value (base + sum or mean) through a matrix formulation."""
    K, W = forest.n_outputs, forest.leaf_width
    acc = np.zeros((X.shape[0], K), dtype=np.float64)
    cnt = np.zeros((K,), dtype=np.float64)
    for t, (f, thr, l, r, v) in enumerate(split_trees(forest)):
        m = tree_matrices(forest.n_features, f, thr, l, r, v)
        if use == "path":
            onehot = path_form_onehot(X, m).astype(np.float64)
        else:
            leaf = paper_form_leaf(X, m)
            onehot = np.zeros((X.shape[0], len(m.leaf_nodes)), dtype=np.float64)
            onehot[np.arange(X.shape[0]), leaf] = 1.0
        contrib = onehot @ m.E.astype(np.float64)                 # gather from E
        if W == 1:
            k = int(forest.tree_output[t]) if forest.tree_output is not None else 0
            acc[:, k] += contrib[:, 0]
            cnt[k] += 1
        else:
            acc += contrib
            cnt += 1
    if forest.aggregate == 1:
        acc = acc / np.where(cnt > 0, cnt, 1.0)[None, :]   # a column no tree feeds stays an empty sum
    if forest.base_score is not None:
        acc = forest.base_score.astype(np.float64)[None, :] + acc
    return acc
