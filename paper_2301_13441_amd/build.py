"""Builds the HIP library in-tree for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libforest_hip.so")
SOURCES = ["forest_pack.cpp", "forest_api_host.cpp", "forest_api.cpp", "forest_kernels.hip", "forest_kernels_reg.hip",
           "forest_kernels_rank.hip", "forest_kernels_ranklds.hip", "forest_kernels_rankbank.hip", "forest_kernels_split.hip",
           "forest_probe.hip",
           "linear_api.cpp", "linear_kernels.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fno-fast-math", "-ffp-contract=off", "-Wall", "-Wno-unused-command-line-argument",
]


def _compile(src: str, extra, verbose: bool) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, *extra, "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return obj


RANKLDS = "forest_kernels_ranklds.hip"
CONSERVATIVE = "-DFOREST_RANKLDS_CONSERVATIVE"


def ranklds_variant_flags(flags: list[str], verbose: bool = False) -> list[str]:
    """The extra flags the LDS rank kernel is built with.  Its streaming form keeps the split
    program in pinned scalar registers with a load in flight between statements, which is sound
    only if the compiler's own code leaves those registers alone: that is checked here on the
    generated assembly, BEFORE anything is linked.  If the check fails the conservative form is
    built instead (every statement loads and waits for its own entries), with a warning."""
    try:
        from . import check_stream_registers
    except ImportError:  # run as a script
        import check_stream_registers
    try:
        n = check_stream_registers.check(HIPCC, flags, os.path.join(CSRC, RANKLDS), OBJ)
        if verbose:
            print(f"stream registers: {n} loops clean", flush=True)
        return []
    except Exception as exc:  # noqa: BLE001 - any failure of the check selects the safe form
        print(f"WARNING: {RANKLDS}: streaming form not verified ({exc}); building the conservative form",
              file=sys.stderr, flush=True)
        return [CONSERVATIVE]


def build(verbose: bool = False, extra: list[str] | None = None) -> str:
    os.makedirs(OBJ, exist_ok=True)
    extra = list(extra or [])
    with ThreadPoolExecutor(max_workers=len(SOURCES) + 1) as pool:
        variant = pool.submit(ranklds_variant_flags, [*FLAGS, *extra], verbose)
        others = [s for s in SOURCES if s != RANKLDS]
        objs = list(pool.map(lambda s: _compile(s, extra, verbose), others))
        objs.append(_compile(RANKLDS, [*extra, *variant.result()], verbose))
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
    print(LIB)
