"""CPU oracle package.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the bench's cpu_baseline leg may import this package; the
product path (the HIP library and its Python binding) never does, and this package never
imports the product.

* ``predict``      -- the plain per-row tree traversal, in C (forest_oracle.c), fp64 sums.
* ``matrix_form``  -- the paper's dense operator representation (Table 2: W1, W2, W3 with
                      matmul / greater / matmul / argmax) and the signed path-matrix form
                      (A, B, C, D, E), written with numpy for tiny forests.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "forest_oracle.c")
_LIB = os.path.join(_HERE, "libforest_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile forest_oracle.c with gcc into libforest_oracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-pthread", "-fno-fast-math",
               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32, i64, p = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
        lib.oracle_predict.restype = ctypes.c_int
        lib.oracle_predict.argtypes = [i32, i32, i32, i32, p, p, p, p, p, p, p, i32, p, i32,
                                       p, i64, p, p, p, p, i32]
        _lib = lib
    return _lib


@dataclass
class OracleResult:
    scores: np.ndarray        # float32 [n_rows, K]
    labels: np.ndarray        # int32 [n_rows]
    leaf_node_id: Optional[np.ndarray]  # int32 [n_rows, T], caller's tree-local node index
    raw: np.ndarray           # float64 [n_rows, K], unrounded value before the transform


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def predict(forest, X: np.ndarray, want_leaves: bool = False, n_threads: int = 1) -> OracleResult:
    """Run the traversal oracle on host arrays.  ``forest`` is any object with the fields of
    ``workloads.Forest`` (duck-typed; this package does not import the generator)."""
    lib = _load()
    X = np.ascontiguousarray(X, dtype=np.float32)
    n_rows = X.shape[0]
    assert X.ndim == 2 and X.shape[1] == forest.n_features
    K, T = forest.n_outputs, len(forest.tree_offset) - 1
    keep = dict(
        tree_offset=np.ascontiguousarray(forest.tree_offset, dtype=np.int64),
        feature=np.ascontiguousarray(forest.feature, dtype=np.int32),
        threshold=np.ascontiguousarray(forest.threshold, dtype=np.float32),
        left=np.ascontiguousarray(forest.left, dtype=np.int32),
        right=np.ascontiguousarray(forest.right, dtype=np.int32),
        leaf_value=np.ascontiguousarray(forest.leaf_value, dtype=np.float32),
        tree_output=(None if forest.tree_output is None
                     else np.ascontiguousarray(forest.tree_output, dtype=np.int32)),
        base_score=(None if forest.base_score is None
                    else np.ascontiguousarray(forest.base_score, dtype=np.float32)),
    )
    scores = np.empty((n_rows, K), dtype=np.float32)
    labels = np.empty((n_rows,), dtype=np.int32)
    raw = np.empty((n_rows, K), dtype=np.float64)
    leaves = np.empty((n_rows, T), dtype=np.int32) if want_leaves else None
    rc = lib.oracle_predict(
        T, forest.n_features, K, forest.leaf_width,
        _ptr(keep["tree_offset"]), _ptr(keep["feature"]), _ptr(keep["threshold"]),
        _ptr(keep["left"]), _ptr(keep["right"]), _ptr(keep["leaf_value"]),
        _ptr(keep["tree_output"]), int(forest.aggregate), _ptr(keep["base_score"]),
        int(forest.transform), _ptr(X), n_rows, _ptr(scores), _ptr(labels), _ptr(leaves),
        _ptr(raw), int(n_threads))
    if rc != 0:
        raise ValueError("oracle_predict rejected its arguments")
    return OracleResult(scores=scores, labels=labels, leaf_node_id=leaves, raw=raw)
