"""MI355X-native tree-ensemble inference (dense operator representation, hand-written HIP).

Thin ctypes binding over the C ABI declared in include/forest.h and include/linear.h.  PyTorch is used only for
device memory and streams.  There is no CPU fallback: without the built HIP library, or
without a GPU at load time, the calls raise.
"""
from .binding import (Forest, ForestError, forest_load, forest_pack, lib_path, load_library,
                      AGG_SUM, AGG_MEAN, TRANSFORM_NONE, TRANSFORM_SIGMOID, TRANSFORM_SOFTMAX,
                      OUT_SCORES, OUT_LABELS, OUT_BOTH)

from .linear_binding import Linear, LinearError, linear_load

__all__ = ["Linear", "LinearError", "linear_load", "Forest", "ForestError", "forest_load", "forest_pack", "lib_path", "load_library",
           "AGG_SUM", "AGG_MEAN", "TRANSFORM_NONE", "TRANSFORM_SIGMOID", "TRANSFORM_SOFTMAX",
           "OUT_SCORES", "OUT_LABELS", "OUT_BOTH"]
