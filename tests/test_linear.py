"""Linear-model family: ABI checks that need no GPU, and GPU parity against the CPU oracle
through the C ABI.  Bar: labels bit-exact, float32 scores within 1e-5 relative / 1e-6 absolute
(both sides accumulate in float64 and round once)."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle.linear_oracle import predict_linear
from paper_2301_13441_amd import linear_binding as lb
from workloads import OUT_BOTH, OUT_LABELS, OUT_SCORES, TRANSFORM_NONE, TRANSFORM_SIGMOID, TRANSFORM_SOFTMAX
from workloads.linear import LinearModel, make_linear_workload

RTOL, ATOL = 1e-5, 1e-6


def _rand_model(seed, F, K, transform, output=OUT_BOTH):
    rng = np.random.default_rng(seed)
    return LinearModel(F, K, (rng.standard_normal((F, K)) / np.sqrt(F)).astype(np.float32),
                       (rng.standard_normal(K) * 0.2).astype(np.float32), transform, output)


# ---------------------------------------------------------------- no GPU needed
def test_library_exports_every_declared_symbol():
    header = open(os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                               "include", "linear.h")).read()
    declared = set(re.findall(r"\b(linear_[a-z_]+)\s*\(", header))
    assert declared == set(lb.LINEAR_EXPORTS)
    lib = lb._lib()
    for name in declared:
        assert hasattr(lib, name)


def test_validation_happens_before_any_device_call():
    lib = lb._lib()
    h = ctypes.c_void_p()

    def load(model):
        d, keep = lb.linear_desc(model)
        return lib.linear_load(ctypes.byref(d), ctypes.byref(h))

    good = _rand_model(0, 4, 3, TRANSFORM_SOFTMAX)
    assert lib.linear_load(None, ctypes.byref(h)) == -1
    assert load(LinearModel(0, 3, good.weight, good.bias, TRANSFORM_NONE)) == -1            # F < 1
    assert load(LinearModel(4, 1, good.weight[:, :1], good.bias[:1], TRANSFORM_SOFTMAX)) == -1  # softmax, K = 1
    assert load(LinearModel(4, 3, good.weight, good.bias, 7)) == -1                          # bad enum
    assert load(LinearModel(4, 33, np.zeros((4, 33), np.float32), None, TRANSFORM_NONE)) == -7  # K limit
    bad = good.weight.copy()
    bad[2, 1] = np.nan
    assert load(LinearModel(4, 3, bad, good.bias, TRANSFORM_NONE)) == -4
    assert h.value is None                                                                  # *out untouched
    assert lib.linear_out_bytes(None, 5) == -1
    assert lib.linear_predict(None, None, 5, None, None) == -1
    assert lib.linear_strerror(-7).decode().startswith("model exceeds")
    lib.linear_free(None)


# ---------------------------------------------------------------- GPU parity
def _run(model, X):
    import torch
    m = lb.linear_load(model)
    try:
        xd = torch.from_numpy(np.ascontiguousarray(X)).cuda()
        scores, labels = m.predict(xd)
        torch.cuda.synchronize()
        return (None if scores is None else scores.cpu().numpy(),
                None if labels is None else labels.cpu().numpy())
    finally:
        m.close()


def _check(model, X):
    ref = predict_linear(model, X)
    scores, labels = _run(model, X)
    if model.output != OUT_SCORES:
        np.testing.assert_array_equal(labels, ref.labels)
    else:
        assert labels is None
    if model.output != OUT_LABELS:
        np.testing.assert_allclose(scores, ref.scores, rtol=RTOL, atol=ATOL)
    else:
        assert scores is None


@pytest.mark.gpu
@pytest.mark.parametrize("name,rows", [("l1", 1000), ("l2", 70001), ("l3", 50003), ("l4", 65537)])
def test_configs(name, rows):
    w = make_linear_workload(name, n_rows=rows)
    _check(w.model, w.make_x())


@pytest.mark.gpu
@pytest.mark.parametrize("F", [1, 3, 31, 32, 33, 64, 90, 257])
@pytest.mark.parametrize("K,transform", [(1, TRANSFORM_NONE), (1, TRANSFORM_SIGMOID), (2, TRANSFORM_SOFTMAX),
                                          (7, TRANSFORM_SOFTMAX), (10, TRANSFORM_NONE), (17, TRANSFORM_SOFTMAX),
                                          (32, TRANSFORM_SIGMOID)])
def test_shapes_ragged_in_every_direction(F, K, transform):
    model = _rand_model(100 * F + K, F, K, transform)
    rng = np.random.default_rng(F + K)
    for rows in (1, 63, 64, 65, 300):
        _check(model, rng.standard_normal((rows, F)).astype(np.float32))


@pytest.mark.gpu
@pytest.mark.parametrize("F", [4, 8, 28, 100, 124, 128])
def test_rows_of_whole_16_byte_pieces(F):
    """Feature counts that are multiples of 4 on both sides of the whole-row / chunked kernel
    boundary, full and partial tiles."""
    for K, transform in ((1, TRANSFORM_SIGMOID), (10, TRANSFORM_SOFTMAX)):
        model = _rand_model(7 * F + K, F, K, transform)
        rng = np.random.default_rng(F * K)
        for rows in (1, 63, 64, 65, 129, 1000):
            _check(model, rng.standard_normal((rows, F)).astype(np.float32))


@pytest.mark.gpu
@pytest.mark.parametrize("F", [28, 40, 64, 90, 100, 130])
def test_x_that_starts_off_a_16_byte_boundary_and_absent_bias(F):
    """X may start at any float: 4, 8 or 12 bytes past a 16-byte boundary the kernels fall back
    to narrower loads.  The bias pointer may be NULL (zeros)."""
    import torch
    rng = np.random.default_rng(F)
    model = LinearModel(F, 3, rng.standard_normal((F, 3)).astype(np.float32), None, TRANSFORM_SOFTMAX, OUT_BOTH)
    m = lb.linear_load(model)
    try:
        for off in (0, 1, 2, 3):
            for rows in (1, 65, 300):
                X = rng.standard_normal((rows, F)).astype(np.float32)
                buf = torch.empty(rows * F + 4, dtype=torch.float32, device="cuda")
                xd = buf[off:off + rows * F].view(rows, F)
                xd.copy_(torch.from_numpy(X))
                assert xd.data_ptr() % 16 == 4 * off
                scores, labels = m.predict(xd)
                torch.cuda.synchronize()
                ref = predict_linear(model, X)
                np.testing.assert_array_equal(labels.cpu().numpy(), ref.labels)
                np.testing.assert_allclose(scores.cpu().numpy(), ref.scores, rtol=RTOL, atol=ATOL)
    finally:
        m.close()


@pytest.mark.gpu
def test_output_kinds_ties_and_empty_batch():
    import torch
    X = np.random.default_rng(5).standard_normal((130, 6)).astype(np.float32)
    for output in (OUT_SCORES, OUT_LABELS, OUT_BOTH):
        _check(_rand_model(9, 6, 4, TRANSFORM_SOFTMAX, output), X)
    # exact ties between columns: the first maximum wins
    tie = LinearModel(6, 3, np.zeros((6, 3), np.float32), np.float32([0.5, 0.5, 0.25]), TRANSFORM_SOFTMAX, OUT_BOTH)
    _check(tie, X)
    m = lb.linear_load(tie)
    m.predict_raw(0, 0, 0, 0)   # n_rows == 0 is a successful no-op
    with pytest.raises(lb.LinearError) as e:   # more rows than one call takes
        m.predict_raw(256, 10**9 + 1, 256, 0)
    assert e.value.code == -7
    for bad in (torch.zeros((10, 5), dtype=torch.float32, device="cuda"),      # wrong feature count
                torch.zeros((10, 6), dtype=torch.float32),                     # host memory
                torch.zeros((10, 6), dtype=torch.float16, device="cuda")):     # wrong dtype
        with pytest.raises(ValueError):
            m.predict(bad)
    m.close()
    torch.cuda.synchronize()


@pytest.mark.gpu
def test_large_magnitudes_and_cancellation():
    """Float64 accumulation: sums that cancel to a small value keep their digits."""
    rng = np.random.default_rng(8)
    F = 64
    w = np.tile(np.float32([1.0, -1.0]), F // 2).reshape(F, 1)
    model = LinearModel(F, 1, w, np.float32([0.0]), TRANSFORM_NONE, OUT_SCORES)
    base = (rng.standard_normal((500, F // 2)) * 1e4).astype(np.float32)
    X = np.empty((500, F), np.float32)
    X[:, 0::2] = base
    X[:, 1::2] = base + rng.standard_normal((500, F // 2)).astype(np.float32) * np.float32(1e-3)
    _check(model, X)


@pytest.mark.gpu
@pytest.mark.parametrize("name", ["l2", "l3", "l4"])
def test_full_size_sampled(name):
    """The bench's launch configuration at full size; the oracle checks sampled rows."""
    import torch
    w = make_linear_workload(name)
    m = lb.linear_load(w.model)
    try:
        n = w.n_rows
        xd = torch.empty((n, w.model.n_features), dtype=torch.float32, device="cuda")
        pos = 0
        keep = {}
        rng = np.random.default_rng(17)
        for ci, chunk in enumerate(w.x_chunks()):
            xd[pos:pos + len(chunk)].copy_(torch.from_numpy(chunk))
            if ci % 7 == 0 or pos + len(chunk) == n:
                idx = np.unique(np.concatenate([rng.integers(0, len(chunk), 200), [0, len(chunk) - 1]]))
                keep[pos] = (idx, chunk[idx].copy())
            pos += len(chunk)
        scores, labels = m.predict(xd)
        torch.cuda.synchronize()
        for start, (idx, rows) in keep.items():
            ref = predict_linear(w.model, rows)
            sel = torch.from_numpy(start + idx).cuda()
            np.testing.assert_allclose(scores[sel].cpu().numpy(), ref.scores, rtol=RTOL, atol=ATOL)
            if labels is not None:
                np.testing.assert_array_equal(labels[sel].cpu().numpy(), ref.labels)
    finally:
        m.close()


@pytest.mark.gpu
def test_input_larger_than_2_to_31_elements():
    """Row offsets past 2^31 elements of X in both kernels (whole-row tiles: 30 features;
    chunked: 130 features); the oracle checks the ends and seeded rows between."""
    import torch
    for F, K, n in ((30, 3, 75_000_000), (130, 2, 17_000_000)):
        assert n * F > 2**31
        model = _rand_model(F, F, K, TRANSFORM_SOFTMAX)
        gen = torch.Generator(device="cuda").manual_seed(F)
        xd = torch.empty((n, F), dtype=torch.float32, device="cuda")
        step = 5_000_000
        for pos in range(0, n, step):
            xd[pos:pos + step].normal_(generator=gen)
        rng = np.random.default_rng(F)
        pick = np.unique(np.concatenate([np.arange(200), np.arange(n - 200, n), rng.integers(0, n, 3000),
                                         rng.integers(2**31 // F, n, 3000)]))
        idx = torch.from_numpy(pick).cuda()
        xs = xd[idx].cpu().numpy()
        m = lb.linear_load(model)
        try:
            scores, labels = m.predict(xd)
            torch.cuda.synchronize()
            got_scores, got_labels = scores[idx].cpu().numpy(), labels[idx].cpu().numpy()
        finally:
            m.close()
        del xd, scores, labels
        ref = predict_linear(model, xs)
        np.testing.assert_array_equal(got_labels, ref.labels)
        np.testing.assert_allclose(got_scores, ref.scores, rtol=RTOL, atol=ATOL)
