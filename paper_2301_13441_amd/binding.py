"""ctypes binding with the same names as the C ABI (argument marshalling only)."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

AGG_SUM, AGG_MEAN = 0, 1
TRANSFORM_NONE, TRANSFORM_SIGMOID, TRANSFORM_SOFTMAX = 0, 1, 2
OUT_SCORES, OUT_LABELS, OUT_BOTH = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libforest_hip.so")
_lib = None

_p = ctypes.c_void_p
_i32, _i64 = ctypes.c_int32, ctypes.c_int64


class ForestError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {code} ({_strerror(code)})")
        self.code = code


class _Desc(ctypes.Structure):
    _fields_ = [("n_trees", _i32), ("n_features", _i32), ("n_outputs", _i32), ("leaf_width", _i32),
                ("tree_offset", _p), ("feature", _p), ("threshold", _p), ("left", _p), ("right", _p),
                ("leaf_value", _p), ("tree_output", _p), ("aggregate", _i32), ("base_score", _p),
                ("transform", _i32), ("output", _i32)]


class _Info(ctypes.Structure):
    _fields_ = [("n_trees", _i32), ("n_features", _i32), ("n_outputs", _i32), ("leaf_width", _i32),
                ("n_internal", _i64), ("n_leaves", _i64), ("max_depth", _i32), ("kernel_kind", _i32),
                ("packed_bytes", _i64), ("x_in_registers", _i32), ("kernel_path", _i32), ("rows_per_workgroup", _i32),
                ("workspace_bytes", _i64), ("small_batch_rows", _i64), ("workgroup_waves", _i32), ("rank_banks", _i32)]


class _View(ctypes.Structure):
    _fields_ = [("n_trees", _i32), ("kernel_kind", _i32), ("kernel_path", _i32), ("rank_registers", _i32),
                ("tree_n_internal", _p), ("tree_depth", _p),
                ("tree_is_full", _p), ("node_base", _p), ("leaf_base", _p), ("split_feature", _p),
                ("split_threshold", _p), ("child_left", _p), ("child_right", _p), ("leaf_node", _p),
                ("leaf_value", _p), ("rank_threshold", _p), ("rank_threshold_base", _p),
                ("rank_bucket", _p), ("rank_bucket_start", _p),
                ("workgroup_waves", _i32), ("wave_tree", _p), ("program_groups", _p),
                ("bank_batches", _i32), ("bank_waves", _i32), ("bank_regs", _i32), ("bank_trees", _i32),
                ("bank_unit", _i32), ("bank_max_units", _i32), ("bank_prog_entries", _i64), ("bank_prog", _p),
                ("bank_stream_base", _p), ("bank_span", _p), ("bank_child", _p), ("bank_leaf", _p), ("bank_batch", _p),
                ("bank_tree", _p), ("bank_reg", _p), ("bank_passes", _i32),
                ("bank_todo_items", _i64), ("bank_pass", _p), ("bank_pass_wave", _p),
                ("bank_todo", _p), ("fast_window", _i32), ("fast_tab_entries", _i64), ("fast_feat", _p), ("fast_tab", _p),
                ("order_leaf_node", _p), ("order_leaf_tree", _p)]


# include/forest.h: the inference ABI
EXPORTS = ["forest_load", "forest_free", "forest_info", "forest_out_bytes", "forest_out_layout",
           "forest_predict", "forest_predict_static", "forest_predict_leaves", "forest_strerror"]
# include/forest_testing.h: host-only views into the model compiler, for its tests
TESTING_EXPORTS = ["forest_pack", "forest_pack_view", "forest_pack_free", "forest_rank_code",
                   "forest_staged_position", "forest_probe_compare_rate"]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the in-tree HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2301_13441_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(_LIB_PATH)
    lib.forest_load.restype = ctypes.c_int
    lib.forest_load.argtypes = [ctypes.POINTER(_Desc), ctypes.POINTER(_p)]
    lib.forest_free.restype = None
    lib.forest_free.argtypes = [_p]
    lib.forest_info.restype = ctypes.c_int
    lib.forest_info.argtypes = [_p, ctypes.POINTER(_Info)]
    lib.forest_out_bytes.restype = _i64
    lib.forest_out_bytes.argtypes = [_p, _i64]
    lib.forest_out_layout.restype = ctypes.c_int
    lib.forest_out_layout.argtypes = [_p, _i64, ctypes.POINTER(_i64), ctypes.POINTER(_i64)]
    lib.forest_predict.restype = ctypes.c_int
    lib.forest_predict.argtypes = [_p, _p, _i64, _p, _p]
    lib.forest_predict_static.restype = ctypes.c_int
    lib.forest_predict_static.argtypes = [_p, _p, _i64, _p, _p]
    lib.forest_predict_leaves.restype = ctypes.c_int
    lib.forest_predict_leaves.argtypes = [_p, _p, _i64, _p, _p]
    lib.forest_pack.restype = ctypes.c_int
    lib.forest_pack.argtypes = [ctypes.POINTER(_Desc), ctypes.POINTER(_p)]
    lib.forest_pack_view.restype = ctypes.c_int
    lib.forest_pack_view.argtypes = [_p, ctypes.POINTER(_View)]
    lib.forest_pack_free.restype = None
    lib.forest_pack_free.argtypes = [_p]
    lib.forest_rank_code.restype = ctypes.c_int
    lib.forest_rank_code.argtypes = [_i32, ctypes.POINTER(ctypes.c_uint16), ctypes.POINTER(ctypes.c_uint16)]
    lib.forest_staged_position.restype = ctypes.c_int
    lib.forest_staged_position.argtypes = [_i32, _i32, ctypes.POINTER(_i32)]
    lib.forest_strerror.restype = ctypes.c_char_p
    lib.forest_strerror.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def _strerror(code: int) -> str:
    try:
        return load_library().forest_strerror(int(code)).decode()
    except Exception:  # pragma: no cover
        return "?"


def _desc_from(forest):
    """Marshal an object with the fields of the C forest_desc (numpy arrays) into the struct.
    Returns (struct, keepalive list)."""
    keep = []

    def arr(a, dt):
        if a is None:
            return None
        a = np.ascontiguousarray(a, dtype=dt)
        keep.append(a)
        return a.ctypes.data_as(_p)

    d = _Desc()
    d.n_trees = len(forest.tree_offset) - 1
    d.n_features = int(forest.n_features)
    d.n_outputs = int(forest.n_outputs)
    d.leaf_width = int(forest.leaf_width)
    d.tree_offset = arr(forest.tree_offset, np.int64)
    d.feature = arr(forest.feature, np.int32)
    d.threshold = arr(forest.threshold, np.float32)
    d.left = arr(forest.left, np.int32)
    d.right = arr(forest.right, np.int32)
    d.leaf_value = arr(forest.leaf_value, np.float32)
    d.tree_output = arr(getattr(forest, "tree_output", None), np.int32)
    d.aggregate = int(forest.aggregate)
    d.base_score = arr(getattr(forest, "base_score", None), np.float32)
    d.transform = int(forest.transform)
    d.output = int(forest.output)
    return d, keep


def forest_pack(forest) -> dict:
    """Run the host model compiler only and return its tables as numpy arrays (no GPU needed)."""
    lib = load_library()
    d, keep = _desc_from(forest)
    h = _p()
    rc = lib.forest_pack(ctypes.byref(d), ctypes.byref(h))
    if rc != 0:
        raise ForestError(rc, "forest_pack")
    try:
        v = _View()
        rc = lib.forest_pack_view(h, ctypes.byref(v))
        if rc != 0:
            raise ForestError(rc, "forest_pack_view")
        T = v.n_trees

        def get(ptr, n, dt):
            if n == 0:
                return np.zeros(0, dtype=dt)
            return np.ctypeslib.as_array(ctypes.cast(ptr, ctypes.POINTER(np.ctypeslib.as_ctypes_type(dt))),
                                         shape=(n,)).copy()

        node_base = get(v.node_base, T + 1, np.int64)
        leaf_base = get(v.leaf_base, T + 1, np.int64)
        ni, nl = int(node_base[-1]), int(leaf_base[-1])
        rank = {}
        if v.rank_threshold_base:
            F = int(forest.n_features)
            tbase = get(v.rank_threshold_base, F + 1, np.int32)
            bucket = get(v.rank_bucket, 4 * F, np.int32).reshape(F, 4)  # lo, scale as raw bits
            n_start = int((bucket[:, 2] + 1).sum()) if F else 0
            rank = dict(rank_threshold=get(v.rank_threshold, int(tbase[-1]), np.float32),
                        rank_threshold_base=tbase,
                        rank_bucket_lo=bucket[:, 0].copy().view(np.float32),
                        rank_bucket_scale=bucket[:, 1].copy().view(np.float32),
                        rank_bucket_count=bucket[:, 2].copy(), rank_bucket_base=bucket[:, 3].copy(),
                        rank_bucket_start=get(v.rank_bucket_start, n_start, np.int32))
            rank.update(fast_window=int(v.fast_window),
                        fast_feat=get(v.fast_feat, int(forest.n_features) * 8, np.uint32).reshape(-1, 8),
                        fast_tab=get(v.fast_tab, int(v.fast_tab_entries), np.uint16))
        if v.wave_tree:
            rank["workgroup_waves"] = int(v.workgroup_waves)
            rank["wave_tree"] = get(v.wave_tree, int(v.workgroup_waves) + 1, np.int32)
            rank["program_groups"] = get(v.program_groups, T, np.int32)
        if v.bank_batches > 0:
            nb, nw, nt = int(v.bank_batches), int(v.bank_waves), int(v.bank_trees)
            span = get(v.bank_span, nb * nw * 2, np.int32).reshape(nb, nw, 2)
            batch = get(v.bank_batch, nb * 4, np.int32).reshape(nb, 4)
            unit = int(v.bank_unit)
            n_slots = int(batch[-1, 0] + batch[-1, 1])
            rank.update(bank_batches=nb, bank_waves=nw, bank_regs=int(v.bank_regs), bank_trees=nt,
                        bank_unit=unit, bank_max_units=int(v.bank_max_units),
                        bank_prog=get(v.bank_prog, int(v.bank_prog_entries), np.uint32),
                        bank_stream_base=get(v.bank_stream_base, nw, np.int32), bank_span=span,
                        bank_child=get(v.bank_child, n_slots, np.uint32),
                        bank_leaf=get(v.bank_leaf, n_slots, np.uint32), bank_batch=batch,
                        bank_tree=get(v.bank_tree, nb * nt * 4, np.int32).reshape(nb, nt, 4),
                        bank_reg=get(v.bank_reg, nw * int(v.bank_regs), np.int32).reshape(nw, -1),
                        bank_pass=get(v.bank_pass, int(v.bank_passes) * 2, np.int32).reshape(-1, 2),
                        bank_pass_wave=get(v.bank_pass_wave, int(v.bank_passes) * nw * 4, np.int32).reshape(-1, nw, 4),
                        bank_todo=get(v.bank_todo, int(v.bank_todo_items) * 4, np.int32).reshape(-1, 4))
        else:
            rank["bank_batches"] = 0
        rank["order_leaf_node"] = get(v.order_leaf_node, nl, np.int32)
        rank["order_leaf_tree"] = get(v.order_leaf_tree, nl, np.int32)
        return dict(
            **rank,
            n_trees=T, kernel_kind=v.kernel_kind, kernel_path=v.kernel_path,
            rank_registers=v.rank_registers,
            tree_n_internal=get(v.tree_n_internal, T, np.int32),
            tree_depth=get(v.tree_depth, T, np.int32),
            tree_is_full=get(v.tree_is_full, T, np.int32),
            node_base=node_base, leaf_base=leaf_base,
            split_feature=get(v.split_feature, ni, np.int32),
            split_threshold=get(v.split_threshold, ni, np.float32),
            child_left=get(v.child_left, ni, np.int32),
            child_right=get(v.child_right, ni, np.int32),
            leaf_node=get(v.leaf_node, nl, np.int32),
            leaf_value=get(v.leaf_value, nl * int(forest.leaf_width), np.float32).reshape(nl, -1),
        )
    finally:
        lib.forest_pack_free(h)


def forest_rank_code(q: int) -> tuple[int, int, int]:
    """(number of codes, f16 bits of code(q), f16 bits of the split entry for threshold q)."""
    code, entry = ctypes.c_uint16(), ctypes.c_uint16()
    n = load_library().forest_rank_code(int(q), ctypes.byref(code), ctypes.byref(entry))
    if n < 0:
        raise ForestError(n, _strerror(n))
    return n, code.value, entry.value


def forest_staged_position(depth: int, pos: int) -> int:
    """Level-order ordinal of the node at bit position `pos` of a depth-4..6 full tree, -1 for none."""
    node = ctypes.c_int32()
    rc = load_library().forest_staged_position(int(depth), int(pos), ctypes.byref(node))
    if rc != 0:
        raise ForestError(rc, _strerror(rc))
    return node.value


def forest_probe_compare_rate(iterations: int, device_word, stream=None) -> int:
    """Enqueues the compare-issue probe on `stream` (torch stream; default: the current one) and
    returns the number of comparisons it makes; `device_word` is an int32 device tensor."""
    import torch
    lib = load_library()
    lib.forest_probe_compare_rate.restype = ctypes.c_int
    lib.forest_probe_compare_rate.argtypes = [_i32, _p, _p, ctypes.POINTER(_i64)]
    s = torch.cuda.current_stream(device_word.device) if stream is None else stream
    n = _i64()
    rc = lib.forest_probe_compare_rate(int(iterations), _p(s.cuda_stream), _p(device_word.data_ptr()), ctypes.byref(n))
    if rc != 0:
        raise ForestError(rc, "forest_probe_compare_rate")
    return int(n.value)


def _check_x(X, n_features: int) -> None:
    """The kernels trust the shape they are given: refuse anything but a contiguous float32
    [n_rows, n_features] tensor in device memory before a pointer reaches them."""
    import torch
    if not (isinstance(X, torch.Tensor) and X.is_cuda and X.dtype == torch.float32 and X.dim() == 2
            and X.shape[1] == n_features and X.is_contiguous()):
        raise ValueError(f"X must be a contiguous float32 CUDA tensor of shape [n_rows, {n_features}]")


class Forest:
    """Owner of a loaded model handle.  predict()/predict_leaves() take torch CUDA tensors."""

    def __init__(self, handle, lib):
        self._h = handle
        self._lib = lib
        info = _Info()
        rc = lib.forest_info(handle, ctypes.byref(info))
        if rc != 0:
            raise ForestError(rc, "forest_info")
        self.info = {name: getattr(info, name) for name, _ in _Info._fields_}
        self.n_outputs = info.n_outputs
        self.n_features = info.n_features
        self.n_trees = info.n_trees

    def close(self):
        if self._h is not None:
            self._lib.forest_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def out_bytes(self, n_rows: int) -> int:
        n = self._lib.forest_out_bytes(self._h, n_rows)
        if n < 0:
            raise ForestError(int(n), "forest_out_bytes")
        return int(n)

    def out_layout(self, n_rows: int):
        so, lo = _i64(), _i64()
        rc = self._lib.forest_out_layout(self._h, n_rows, ctypes.byref(so), ctypes.byref(lo))
        if rc != 0:
            raise ForestError(rc, "forest_out_layout")
        return so.value, lo.value

    def predict_raw(self, x_ptr: int, n_rows: int, out_ptr: int, stream: int = 0, static: bool = False) -> None:
        """forest_predict (static: forest_predict_static) on raw device pointers."""
        fn = self._lib.forest_predict_static if static else self._lib.forest_predict
        rc = fn(self._h, _p(x_ptr), n_rows, _p(out_ptr), _p(stream))
        if rc != 0:
            raise ForestError(rc, "forest_predict_static" if static else "forest_predict")

    def predict(self, X, out=None, stream=None, static: bool = False):
        """X: torch float32 CUDA tensor [n_rows, F], contiguous.  Returns (scores, labels) views
        into one uint8 output buffer (either may be None, per the model's output kind).  With
        `static` the call goes through forest_predict_static (pass `out`: it allocates nothing)."""
        import torch
        _check_x(X, self.n_features)
        n = X.shape[0]
        nbytes = self.out_bytes(n)
        if out is None:
            out = torch.empty(max(nbytes, 4), dtype=torch.uint8, device=X.device)
        if not (out.is_cuda and out.device == X.device and out.is_contiguous()
                and out.numel() * out.element_size() >= nbytes):
            raise ValueError(f"out must be a contiguous tensor of at least {nbytes} bytes on {X.device}")
        s = torch.cuda.current_stream(X.device) if stream is None else stream
        self.predict_raw(X.data_ptr(), n, out.data_ptr(), s.cuda_stream, static=static)
        so, lo = self.out_layout(n)
        flat = out.view(torch.uint8).reshape(-1)
        scores = labels = None
        if so >= 0:
            scores = flat[so:so + 4 * n * self.n_outputs].view(torch.float32).reshape(n, self.n_outputs)
        if lo >= 0:
            labels = flat[lo:lo + 4 * n].view(torch.int32)
        return scores, labels

    def predict_leaves(self, X, stream=None):
        import torch
        _check_x(X, self.n_features)
        n = X.shape[0]
        out = torch.empty((n, self.n_trees), dtype=torch.int32, device=X.device)
        s = torch.cuda.current_stream(X.device) if stream is None else stream
        rc = self._lib.forest_predict_leaves(self._h, _p(X.data_ptr()), n, _p(out.data_ptr()),
                                             _p(s.cuda_stream))
        if rc != 0:
            raise ForestError(rc, "forest_predict_leaves")
        return out


def forest_load(forest) -> Forest:
    """forest_load: validate, pack and upload to the current HIP device."""
    lib = load_library()
    d, keep = _desc_from(forest)
    h = _p()
    rc = lib.forest_load(ctypes.byref(d), ctypes.byref(h))
    if rc != 0:
        raise ForestError(rc, "forest_load")
    return Forest(h, lib)
