"""ctypes binding of the linear-model family, same names as include/linear.h (argument
marshalling only; every step runs in the HIP kernel)."""
from __future__ import annotations

import ctypes

import numpy as np

from .binding import load_library

_p = ctypes.c_void_p
_i32, _i64 = ctypes.c_int32, ctypes.c_int64

LINEAR_EXPORTS = ["linear_load", "linear_free", "linear_out_bytes", "linear_out_layout", "linear_predict",
                  "linear_strerror"]


class _LinearDesc(ctypes.Structure):
    _fields_ = [("n_features", _i32), ("n_outputs", _i32), ("weight", _p), ("bias", _p),
                ("transform", _i32), ("output", _i32)]


class LinearError(RuntimeError):
    def __init__(self, code: int, what: str):
        lib = _lib()
        super().__init__(f"{what}: {code} ({lib.linear_strerror(int(code)).decode()})")
        self.code = code


_ready = False


def _lib():
    global _ready
    lib = load_library()
    if not _ready:
        lib.linear_load.restype = ctypes.c_int
        lib.linear_load.argtypes = [ctypes.POINTER(_LinearDesc), ctypes.POINTER(_p)]
        lib.linear_free.restype = None
        lib.linear_free.argtypes = [_p]
        lib.linear_out_bytes.restype = _i64
        lib.linear_out_bytes.argtypes = [_p, _i64]
        lib.linear_out_layout.restype = ctypes.c_int
        lib.linear_out_layout.argtypes = [_p, _i64, ctypes.POINTER(_i64), ctypes.POINTER(_i64)]
        lib.linear_predict.restype = ctypes.c_int
        lib.linear_predict.argtypes = [_p, _p, _i64, _p, _p]
        lib.linear_strerror.restype = ctypes.c_char_p
        lib.linear_strerror.argtypes = [ctypes.c_int]
        _ready = True
    return lib


def linear_desc(model):
    """Marshal an object with the fields of the C linear_desc.  Returns (struct, keepalive)."""
    keep = []

    def arr(a):
        if a is None:
            return None
        a = np.ascontiguousarray(a, dtype=np.float32)
        keep.append(a)
        return a.ctypes.data_as(_p)

    d = _LinearDesc()
    d.n_features = int(model.n_features)
    d.n_outputs = int(model.n_outputs)
    d.weight = arr(model.weight)
    d.bias = arr(getattr(model, "bias", None))
    d.transform = int(model.transform)
    d.output = int(model.output)
    return d, keep


def _check_x(X, n_features: int) -> None:
    """The kernels trust the shape they are given: refuse anything but a contiguous float32
    [n_rows, n_features] tensor in device memory before a pointer reaches them."""
    import torch
    if not (isinstance(X, torch.Tensor) and X.is_cuda and X.dtype == torch.float32 and X.dim() == 2
            and X.shape[1] == n_features and X.is_contiguous()):
        raise ValueError(f"X must be a contiguous float32 CUDA tensor of shape [n_rows, {n_features}]")


class Linear:
    """Owner of a loaded linear model handle.  predict() takes torch CUDA tensors."""

    def __init__(self, handle, n_features, n_outputs):
        self._h = handle
        self.n_features = n_features
        self.n_outputs = n_outputs

    def close(self):
        if self._h is not None:
            _lib().linear_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def out_bytes(self, n_rows: int) -> int:
        n = _lib().linear_out_bytes(self._h, n_rows)
        if n < 0:
            raise LinearError(int(n), "linear_out_bytes")
        return int(n)

    def out_layout(self, n_rows: int):
        so, lo = _i64(), _i64()
        rc = _lib().linear_out_layout(self._h, n_rows, ctypes.byref(so), ctypes.byref(lo))
        if rc != 0:
            raise LinearError(rc, "linear_out_layout")
        return so.value, lo.value

    def predict_raw(self, x_ptr: int, n_rows: int, out_ptr: int, stream: int = 0) -> None:
        rc = _lib().linear_predict(self._h, _p(x_ptr), n_rows, _p(out_ptr), _p(stream))
        if rc != 0:
            raise LinearError(rc, "linear_predict")

    def predict(self, X, out=None, stream=None):
        """X: torch float32 CUDA tensor [n_rows, F], contiguous.  Returns (scores, labels) views
        into one uint8 output buffer (either may be None, per the model's output kind)."""
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
        self.predict_raw(X.data_ptr(), n, out.data_ptr(), s.cuda_stream)
        so, lo = self.out_layout(n)
        flat = out.view(torch.uint8).reshape(-1)
        scores = labels = None
        if so >= 0:
            scores = flat[so:so + 4 * n * self.n_outputs].view(torch.float32).reshape(n, self.n_outputs)
        if lo >= 0:
            labels = flat[lo:lo + 4 * n].view(torch.int32)
        return scores, labels


def linear_load(model) -> Linear:
    """linear_load: validate, widen and upload to the current HIP device."""
    lib = _lib()
    d, keep = linear_desc(model)
    h = _p()
    rc = lib.linear_load(ctypes.byref(d), ctypes.byref(h))
    del keep
    if rc != 0:
        raise LinearError(rc, "linear_load")
    return Linear(h, int(model.n_features), int(model.n_outputs))
