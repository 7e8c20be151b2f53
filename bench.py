#!/usr/bin/env python3
"""Benchmark of the whole hot path: one step = forest_predict over one batch of synthetic rows.

Prints ONE JSON line.  `value` is rows/s with X already resident in HBM.  The `roofline`
object prices the dominant (only) kernel against the vector-ALU peak: the method evaluates
every internal node of every tree for every row, one comparison each, and the packed model
stays on chip, so the rate of the compare instruction is what bounds it.  The rank kernels
compare two rows per lane with one packed-f16 instruction, so their peak is two comparisons
per lane and clock; the fp32 kernels' peak is one.
`cpu_baseline` is the CPU oracle timed on this machine's host cores on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X: 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz vector instructions per second and
# lane.  The fp32 vector peak of 157.3 TFLOP/s is this number x 2 (FMA) x 2 (packed fp32).  A
# float32 compare is neither fused nor packed: one comparison per lane-op.  A packed-f16
# compare (v_pk_fma_f16 with clamp on exactly coded ranks) is two comparisons per lane-op.
ALU_PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9
HBM_PEAK = 8.0e12

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE, scaled by a
# copy kernel of known size); see profiles/.  None until measured for a workload.
MEASURED_TRAFFIC = {
    # profiles/forest_rank_kernel_c2.md: FETCH_SIZE 66,233 x 2.000 (copy-kernel scale) KiB read,
    # WRITE_SIZE 7,812.5 x 1.000 KiB written
    "c2": 135.6e6 + 8.0e6,
    # profiles/linear_kernels.md: FETCH_SIZE 703,161 x 2.000 KiB, WRITE_SIZE 15,625 x 1.000 KiB
    "l2": 1440.0e6 + 16.0e6,
}

# Busy fractions of the units the forest kernels use, from rocprofv3 --pmc runs of this script
# (SQ_INSTS_VALU x 4 cycles, SQ_VALU_MFMA_BUSY_CYCLES, SQ_LDS_IDX_ACTIVE over the SIMD / CU cycles
# of the launch); see the profile named.  They are measurements of the committed kernels, not
# taken live, and are reported next to the live roofline fraction.
MEASURED_UNIT_BUSY = {
    "c2": {"valu_issue": 0.81, "mfma": 0.54, "profile": "profiles/forest_rank_kernel_c2.md"},
    "c3": {"valu_issue": 0.80, "profile": "profiles/forest_rank_kernel_c3_c4.md"},
    "c4": {"valu_issue": 0.82, "profile": "profiles/forest_rank_kernel_c3_c4.md"},
    "c5": {"valu_issue": 0.56, "lds": 0.67, "profile": "profiles/forest_ranklds_kernel_c5.md"},
}


def bench_linear(args) -> int:
    """The linear-model family (one matmul + bias + transform + label): bound by reading X once
    from HBM, so its roofline is the HBM one."""
    import numpy as np
    import torch

    import paper_2301_13441_amd as pk
    from workloads.linear import make_linear_workload

    w = make_linear_workload(args.workload, n_rows=args.rows)
    n_rows, F, K = w.n_rows, w.model.n_features, w.model.n_outputs
    m = pk.linear_load(w.model)
    xd = torch.empty((n_rows, F), dtype=torch.float32, device="cuda")
    sample_rows = min(n_rows, 262144)
    parts = []
    pos = 0
    for chunk in w.x_chunks(n_rows):
        xd[pos:pos + len(chunk)].copy_(torch.from_numpy(chunk))
        if pos < sample_rows:
            parts.append(chunk[:max(0, sample_rows - pos)].copy())
        pos += len(chunk)
    x_sample = np.concatenate(parts)[:sample_rows]
    out = torch.empty(max(m.out_bytes(n_rows), 4), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    for _ in range(args.warmup):
        m.predict(xd, out=out)
    torch.cuda.synchronize()
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        starts[i].record(stream)
        m.predict(xd, out=out)
        stops[i].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kernel_ms = [a.elapsed_time(b) for a, b in zip(starts, stops)]
    kernel_s = float(np.mean(kernel_ms)) * 1e-3
    scores, labels = m.predict(xd, out=out)
    torch.cuda.synchronize()
    algo_bytes = n_rows * 4.0 * F + m.out_bytes(n_rows)
    roofline = {
        "bound": "hbm",
        "kernel": "linear_predict (matmul + bias + transform + label, one kernel)",
        "achieved": algo_bytes / kernel_s / 1e9,
        "peak": HBM_PEAK / 1e9,
        "unit": "GB/s",
        "frac": algo_bytes / kernel_s / HBM_PEAK,
        "kernel_ms_avg": kernel_s * 1e3,
        "kernel_ms_min": float(np.min(kernel_ms)),
        "algorithmic_bytes": algo_bytes,
        "flops": 2.0 * F * K * n_rows,
        "traffic": MEASURED_TRAFFIC.get(args.workload),
    }
    cpu_baseline = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle.linear_oracle import predict_linear
        t1 = time.perf_counter()
        ref = predict_linear(w.model, x_sample)
        dt = time.perf_counter() - t1
        cpu_baseline = {"value": sample_rows / dt, "unit": "rows/s", "cores": os.cpu_count() or 1,
                        "kind": "oracle", "sample": f"first {sample_rows} rows of {args.workload}, one pass "
                                                    "(numpy float64 matmul, its BLAS threads)"}
        parity = {"rows_checked": sample_rows}
        if scores is not None:
            got = scores[:sample_rows].cpu().numpy()
            err = np.abs(got - ref.scores)
            parity["scores_within_tol"] = bool((err <= 1e-6 + 1e-5 * np.abs(ref.scores)).all())
            parity["max_abs_err"] = float(err.max())
        if labels is not None:
            parity["labels_equal"] = bool((labels[:sample_rows].cpu().numpy() == ref.labels).all())
    line = {
        "metric": "rows/sec scored (fp32 X), 1 MI355X",
        "value": n_rows * args.steps / wall,
        "unit": "rows/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64 products and sums of f32 inputs, rounded to f32 once",
        "data": "synthetic (seeded; stands in for the paper's linear models on YearPrediction)",
        "config": {"workload": args.workload, "n_rows": n_rows, "n_features": F, "n_outputs": K},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "parity": parity,
    }
    print(json.dumps(line))
    m.close()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5", "l1", "l2", "l3", "l4"],
                    help="c1..c5: tree ensembles (c2 is the headline); l1..l4: linear models")
    ap.add_argument("--rows", type=int, default=None, help="override the row count (testing)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 "
              "(rows are independent: more GPUs = shard X by rows, replicate the packed model)",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2301_13441_amd as pk
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    if args.workload.startswith("l"):
        return bench_linear(args)

    w = wl.make_workload(args.workload, n_rows=args.rows)
    n_rows, F = w.n_rows, w.forest.n_features
    f = pk.forest_load(w.forest)
    info = f.info

    # X: generated on the host in chunks, copied to HBM before the timed region
    xd = torch.empty((n_rows, F), dtype=torch.float32, device="cuda")
    sample_rows = min(n_rows, 262144)
    parts = []
    pos = 0
    for chunk in w.x_chunks(n_rows):
        xd[pos:pos + len(chunk)].copy_(torch.from_numpy(chunk))
        if pos < sample_rows:
            parts.append(chunk[:max(0, sample_rows - pos)].copy())
        pos += len(chunk)
    x_sample = np.concatenate(parts)[:sample_rows]
    out = torch.empty(max(f.out_bytes(n_rows), 4), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()

    stream = torch.cuda.current_stream()
    for _ in range(args.warmup):
        f.predict(xd, out=out)
    torch.cuda.synchronize()

    starts = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        starts[i].record(stream)
        f.predict(xd, out=out)
        stops[i].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kernel_ms = [a.elapsed_time(b) for a, b in zip(starts, stops)]
    kernel_s = float(np.mean(kernel_ms)) * 1e-3

    scores, labels = f.predict(xd, out=out)
    torch.cuda.synchronize()

    compares = float(info["n_internal"]) * n_rows          # one per (row, internal node)
    achieved = compares / kernel_s
    algo_bytes = n_rows * (4.0 * F) + f.out_bytes(n_rows)
    packed = info["kernel_path"] in (2, 3)  # rank kernels: two comparisons per packed-f16 lane-op
    peak = ALU_PEAK_LANE_OPS * (2 if packed else 1)
    roofline = {
        "bound": "alu",
        "kernel": "forest_predict (fused compare + leaf resolution + reduction)",
        "achieved": achieved / 1e12,
        "peak": peak / 1e12,
        "unit": "Tcompare/s",
        "frac": achieved / peak,
        "peak_basis": "256 CU x 4 SIMD x 16 lanes x 2.4 GHz x "
                      + ("2 comparisons per packed-f16 lane-op" if packed else "1 float32 comparison per lane-op"),
        # against one float32 compare per (row, node) and lane-op, the floor a plain fp32 kernel has
        "frac_vs_fp32_compare_peak": achieved / ALU_PEAK_LANE_OPS,
        "kernel_ms_avg": kernel_s * 1e3,
        "kernel_ms_min": float(np.min(kernel_ms)),
        "algorithmic_bytes": algo_bytes,
        "hbm_GBps": algo_bytes / kernel_s / 1e9,
        "hbm_frac": algo_bytes / kernel_s / HBM_PEAK,
        "traffic": MEASURED_TRAFFIC.get(args.workload),
        "unit_busy_measured": MEASURED_UNIT_BUSY.get(args.workload),
    }

    cpu_baseline = None
    parity = None
    if not args.no_cpu_baseline:
        import oracle
        cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16")))
        t1 = time.perf_counter()
        ref = oracle.predict(w.forest, x_sample, n_threads=cores)
        dt = time.perf_counter() - t1
        cpu_baseline = {"value": sample_rows / dt, "unit": "rows/s", "cores": cores, "kind": "oracle",
                        "sample": f"first {sample_rows} rows of {args.workload}, one pass, "
                                  f"{cores} threads over contiguous row blocks"}
        parity = {"rows_checked": sample_rows}
        if scores is not None:
            got = scores[:sample_rows].cpu().numpy()
            err = np.abs(got - ref.scores)
            parity["scores_within_tol"] = bool((err <= 1e-6 + 1e-5 * np.abs(ref.scores)).all())
            parity["max_abs_err"] = float(err.max())
        if labels is not None:
            parity["labels_equal"] = bool((labels[:sample_rows].cpu().numpy() == ref.labels).all())

    line = {
        "metric": "rows/sec scored (fp32 X), 1 MI355X",
        "value": n_rows * args.steps / wall,
        "unit": "rows/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": ("f16 threshold ranks (exact rewrite of the f32 compare), f64 accumulate"
                  if info["kernel_path"] in (2, 3) else "f32 compare, f64 accumulate"),
        "data": "synthetic (seeded; stands in for YearPrediction and the paper's unstated models)",
        "config": {"workload": args.workload, "n_rows": n_rows, "n_features": F,
                   "n_trees": info["n_trees"], "max_depth": info["max_depth"],
                   "n_internal_nodes": info["n_internal"], "n_outputs": info["n_outputs"],
                   "kernel_kind": info["kernel_kind"], "kernel_path": info["kernel_path"],
                   "packed_bytes": info["packed_bytes"]},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "parity": parity,
    }
    print(json.dumps(line))
    f.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
