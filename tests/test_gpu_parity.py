"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bar: leaf ids and labels bit-exact; float32 scores within 1e-5 relative / 1e-6 absolute."""
import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

RTOL, ATOL = 1e-5, 1e-6


def _run(forest, X, leaves=True):
    import torch
    import paper_2301_13441_amd as pk
    f = pk.forest_load(forest)
    try:
        xd = torch.from_numpy(np.ascontiguousarray(X)).cuda()
        scores, labels = f.predict(xd)
        lv = f.predict_leaves(xd) if leaves and forest.n_trees > 0 else None
        torch.cuda.synchronize()
        return (None if scores is None else scores.cpu().numpy(),
                None if labels is None else labels.cpu().numpy(),
                None if lv is None else lv.cpu().numpy(), f.info)
    finally:
        f.close()


def _check(forest, X, leaves=True):
    ref = oracle.predict(forest, X, want_leaves=leaves, n_threads=8)
    scores, labels, lv, info = _run(forest, X, leaves)
    if lv is not None:
        np.testing.assert_array_equal(lv, ref.leaf_node_id)
    if labels is not None:
        np.testing.assert_array_equal(labels, ref.labels)
    if scores is not None:
        np.testing.assert_allclose(scores, ref.scores, rtol=RTOL, atol=ATOL)
    return info


@pytest.mark.parametrize("name,rows,trees,kind", [
    ("c1", 1000, None, 4),        # the whole small configuration
    ("c2", 1000, 40, 8),          # depth 8: 8 outcome words per (row, tree)
    ("c3", 777, 100, 6),          # ragged tail: 777 = 12 tiles + 9 rows
    ("c4", 600, 200, 6),          # 10 classes, softmax + argmax, 30 % zeros in X
    ("c5", 300, 9, 0),            # deep irregular trees, vector leaves (9 trees over 8 waves)
])
def test_configs_small(name, rows, trees, kind):
    w = wl.make_workload(name, n_rows=rows, n_trees=trees)
    info = _check(w.forest, w.make_x(rows))
    assert info["kernel_kind"] == kind


@pytest.mark.parametrize("depth", [1, 2, 3, 5, 7])
def test_full_depths(depth):
    rng = np.random.default_rng(depth)
    arrs = wl._full_forest(rng, 9, depth, 6, wl._normal_thr,
                           lambda r, s: r.standard_normal(s, dtype=np.float32))
    f = wl.Forest(n_features=6, n_outputs=1, leaf_width=1, tree_output=np.zeros(9, np.int32),
                  aggregate=wl.AGG_SUM, transform=wl.TRANSFORM_SIGMOID, **arrs)
    X = rng.standard_normal((333, 6)).astype(np.float32)
    assert _check(f, X)["kernel_kind"] == depth


@pytest.mark.parametrize("seed", range(4))
def test_irregular_forests_with_ties(seed):
    f = wl.random_forest(500 + seed, n_trees=13, n_features=5, max_depth=9, stop_prob=0.2,
                         n_outputs=3, leaf_width=(1 if seed % 2 else 3), grid_thresholds=True,
                         transform=wl.TRANSFORM_SOFTMAX, aggregate=wl.AGG_MEAN)
    rng = np.random.default_rng(seed)
    X = (rng.integers(-3, 4, size=(200, 5)).astype(np.float32) * np.float32(0.5))
    info = _check(f, X)
    assert info["kernel_kind"] == 0 and info["kernel_path"] == 3


@pytest.mark.parametrize("seed", range(8))
def test_register_bank_kernel_on_large_batches(seed):
    """Irregular trees with one scalar column or at most two-wide vector leaves: batches of
    small_batch_rows rows or more run the register-bank kernel (whole trees evaluated by the wave
    that holds each node's rank register, one lane per (row, tree) in the walk)."""
    rng = np.random.default_rng(300 + seed)
    K = 1 + seed % 2
    F = int(rng.choice([2, 31, 256]))
    T = int(rng.choice([1, 3, 4, 5, 22]))
    f = wl.random_forest(1300 + seed, n_trees=T, n_features=F, max_depth=int(rng.integers(1, 11)),
                         stop_prob=float(rng.choice([0.05, 0.2])), n_outputs=K, leaf_width=K,
                         grid_thresholds=bool(seed % 4 == 0), aggregate=int(seed % 3 == 0),
                         transform=(wl.TRANSFORM_SOFTMAX if K == 2 and seed % 4 == 1 else wl.TRANSFORM_NONE))
    rows = 65536 + int(rng.integers(0, 300))
    X = rng.standard_normal((rows, F)).astype(np.float32)
    if seed % 4 == 0:
        X = np.round(X * 2) / 2
    X[5, :] = np.nan
    X[6, :] = np.inf
    X[7, :] = -np.inf
    info = _check(f, X)
    if info["kernel_kind"] == 0:     # a draw of shallow trees that all came out full runs the rank kernel
        assert info["kernel_path"] == 3 and info["rank_banks"] == 1


def test_register_bank_kernel_lookup_paths():
    """The register-bank kernel's rank lookups, every path in one model: a feature whose 13,000
    thresholds take two registers, one with 7,000 (one register, codes of both signs), one with 3
    (no window), one whose 500 thresholds crowd into a millionth of its range (buckets fuller
    than a window), features in a second block of 64 columns with the block between unused, rows
    of 70 floats at a 4-byte aligned address, values on and between thresholds, NaN and Inf."""
    import torch
    import paper_2301_13441_amd as pk
    rng = np.random.default_rng(77)
    F, n = 200, 65536 + 77
    f = wl.random_forest(4242, n_trees=600, n_features=F, max_depth=7, stop_prob=0.05)
    internal = np.flatnonzero(f.feature >= 0)
    assert internal.size > 30000
    feat = f.feature.copy()
    thr = f.threshold.copy()
    cut = [0, 13000, 20000, 20300, 22300, internal.size]
    feat[internal[cut[0]:cut[1]]] = 0
    thr[internal[cut[0]:cut[1]]] = rng.permutation(13000).astype(np.float32)
    feat[internal[cut[1]:cut[2]]] = 1
    thr[internal[cut[1]:cut[2]]] = rng.permutation(7000).astype(np.float32) * np.float32(0.5)
    feat[internal[cut[2]:cut[3]]] = 2
    thr[internal[cut[2]:cut[3]]] = rng.choice(np.float32([-0.5, 0.0, 0.75]), cut[3] - cut[2])
    feat[internal[cut[3]:cut[4]]] = 3
    thr[internal[cut[3]:cut[4]]] = np.float32(1.0) + rng.integers(0, 500, cut[4] - cut[3]).astype(np.float32) * np.float32(1e-6)
    thr[internal[cut[3]:cut[3] + 2]] = np.float32([-1e30, 1e30])
    feat[internal[cut[4]:]] = 130 + rng.integers(0, 70, internal.size - cut[4]).astype(np.int32)   # columns 64..127 unused
    g = wl.Forest(**{**f.__dict__, "feature": feat, "threshold": thr})
    X = rng.standard_normal((n, F)).astype(np.float32)
    X[:, 0] = rng.integers(-2, 26004, n).astype(np.float32) * np.float32(0.5)
    X[:, 1] = rng.integers(-4, 14008, n).astype(np.float32) * np.float32(0.25)
    X[:, 2] = rng.choice(np.float32([-1.0, -0.5, -0.25, 0.0, 0.5, 0.75, 1.0]), n)
    X[:, 3] = np.float32(1.0) + rng.integers(-5, 505, n).astype(np.float32) * np.float32(1e-6)
    X[::97, 3] = rng.choice(np.float32([-2e30, -1e30, 0.0, 1e30, 2e30]), len(X[::97]))
    X[11, :] = np.nan
    X[12, :] = np.inf
    X[13, :] = -np.inf
    buf = torch.zeros(n * F + 1, dtype=torch.float32, device="cuda")
    xd = buf[1:].view(n, F)
    xd.copy_(torch.from_numpy(X))
    assert xd.data_ptr() % 8 == 4
    ref = oracle.predict(g, X, want_leaves=True, n_threads=8)
    h = pk.forest_load(g)
    try:
        assert h.info["kernel_path"] == 3 and h.info["rank_banks"] == 1
        scores, labels = h.predict(xd)
        leaves = h.predict_leaves(xd)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(leaves.cpu().numpy(), ref.leaf_node_id)
        np.testing.assert_allclose(scores.cpu().numpy(), ref.scores, rtol=RTOL, atol=ATOL)
    finally:
        h.close()


@pytest.mark.parametrize("seed", range(64))
def test_random_models_and_batches(seed):
    """Everything drawn at once: full or irregular trees, feature and tree counts, depth, output
    columns, scalar or vector leaves, aggregate, base scores, transform, output kind, batch size
    (single rows, ragged tiles, batches that cut the trees into shares and batches that do not)."""
    rng = np.random.default_rng(7000 + seed)
    K = int(rng.choice([1, 1, 2, 3, 5, 12]))
    vector = bool(K > 1 and rng.random() < 0.4)
    transform = int(rng.choice([wl.TRANSFORM_NONE, wl.TRANSFORM_SIGMOID] if K == 1 else
                               [wl.TRANSFORM_NONE, wl.TRANSFORM_SIGMOID, wl.TRANSFORM_SOFTMAX]))
    kw = dict(n_outputs=K, transform=transform, aggregate=int(rng.choice([wl.AGG_SUM, wl.AGG_MEAN])),
              output=int(rng.choice([wl.OUT_SCORES, wl.OUT_LABELS, wl.OUT_BOTH])))
    F = int(rng.choice([1, 2, 7, 28, 60, 130, 260]))
    T = int(rng.integers(1, 70))
    if rng.random() < 0.5 and not vector:
        f = _full_forest(8000 + seed, T, int(rng.integers(1, 9)), F, **{k: v for k, v in kw.items() if k != "n_outputs"},
                         n_outputs=K)
    else:
        f = wl.random_forest(8000 + seed, n_trees=T, n_features=F, max_depth=int(rng.integers(1, 12)),
                             stop_prob=float(rng.choice([0.05, 0.2, 0.4])), leaf_width=(K if vector else 1),
                             grid_thresholds=bool(rng.random() < 0.3), **kw)
    if rng.random() < 0.5:
        f = wl.Forest(**{**f.__dict__, "base_score": rng.standard_normal(K).astype(np.float32)})
    rows = int(rng.choice([1, 2, 63, 64, 65, 127, 128, 129, 500, 1111, 70000]))
    X = rng.standard_normal((rows, F)).astype(np.float32)
    if rng.random() < 0.3:
        X = np.round(X * 2) / 2          # many x == threshold cases on grid thresholds
    _check(f, X, leaves=rows <= 2000)


@pytest.mark.parametrize("what", ["depth", "features", "outputs", "all"])
def test_models_at_the_documented_limits(what):
    """64 tests on the longest path, 4096 features, 32 output columns: each alone and together."""
    from test_pack import _chain_forest
    depth, F, K = {"depth": (64, 5, 1), "features": (6, 4096, 2), "outputs": (6, 9, 32), "all": (64, 4096, 32)}[what]
    n_trees = 700 if what == "features" else 7     # 4200 nodes: most of the 4096 features are tested somewhere
    for vector in (False, True):
        if vector and K == 1:
            continue
        f = _chain_forest(depth, F, n_trees=n_trees, n_outputs=K, leaf_width=(K if vector else 1), seed=depth + F + K,
                          transform=(wl.TRANSFORM_SOFTMAX if K > 1 else wl.TRANSFORM_SIGMOID))
        rng = np.random.default_rng(F)
        _check(f, rng.standard_normal((300, F)).astype(np.float32))


@pytest.mark.parametrize("n_features,path", [(20, 3), (300, 0)])
def test_very_large_trees(n_features, path):
    """Two trees of about 100,000 internal nodes each (depth 17): the streaming walks of the LDS
    rank kernel and of the plain irregular-tree kernel keep nothing per tree but one chunk."""
    f = wl.random_forest(1700 + n_features, n_trees=2, n_features=n_features, max_depth=17, stop_prob=0.004,
                         n_outputs=2, leaf_width=2, transform=wl.TRANSFORM_SOFTMAX)
    assert f.n_nodes > 150_000
    rng = np.random.default_rng(n_features)
    info = _check(f, rng.standard_normal((200, n_features)).astype(np.float32))
    assert info["kernel_path"] == path, info


def test_special_values_nan_inf_signed_zero():
    w = wl.make_workload("c1", n_rows=256)
    X = w.make_x(256).copy()
    rng = np.random.default_rng(9)
    special = np.asarray([np.nan, np.inf, -np.inf, 0.0, -0.0, 1e-45, -1e-45], np.float32)
    mask = rng.random(X.shape) < 0.3
    X[mask] = special[rng.integers(0, len(special), size=int(mask.sum()))]
    f = w.forest
    thr = f.threshold.copy()
    internal = np.flatnonzero(f.feature >= 0)
    thr[internal[::7]] = np.inf
    thr[internal[3::11]] = -np.inf
    thr[internal[5::13]] = -0.0
    g = wl.Forest(**{**f.__dict__, "threshold": thr})
    _check(g, X)


def test_empty_and_single_row_and_single_leaf_trees():
    import torch
    import paper_2301_13441_amd as pk
    w = wl.make_workload("c1", n_rows=1)
    _check(w.forest, w.make_x(1))
    f = pk.forest_load(w.forest)
    f.predict_raw(0, 0, 0, 0)           # n_rows == 0 is a successful no-op
    f.close()
    # forest of single-leaf trees (root is a leaf) plus one stump
    g = wl.random_forest(77, n_trees=5, n_features=3, max_depth=0)
    X = np.zeros((70, 3), np.float32)
    assert _check(g, X)["kernel_kind"] == 0
    torch.cuda.synchronize()


@pytest.mark.parametrize("name,trees", [
    ("c2", 200),   # rank kernel, depth 8, one column
    ("c3", 300),   # rank kernel, depth 6
    ("c4", 200),   # wide rank kernel, 10 columns, softmax
    ("c5", 128),   # LDS rank kernel, vector leaves, 8 waves
])
@pytest.mark.parametrize("rows", [1, 2, 65, 129, 1000])
def test_small_batches_cut_the_trees_into_shares(name, trees, rows):
    """Below forest_info.small_batch_rows rows a call also splits the trees over workgroups and
    sums fp64 partial sums in a second kernel: same answers as the oracle at every batch size."""
    w = wl.make_workload(name, n_rows=rows, n_trees=trees)
    info = _check(w.forest, w.make_x(rows))
    assert info["small_batch_rows"] == 512 * info["rows_per_workgroup"] > rows
    assert info["workspace_bytes"] >= 8 * rows * w.forest.n_outputs * 2


def test_small_batches_other_families():
    # float32 register family (too many rank registers)
    rng = np.random.default_rng(5)
    f = _full_forest(3, 80, 8, 128, feature_bias=0.9)
    for rows in (1, 100, 300):
        info = _check(f, rng.standard_normal((rows, 128)).astype(np.float32))
        assert info["kernel_path"] == 1
    # LDS rank family in small workgroups: irregular trees with 20 output columns
    g = wl.random_forest(901, n_trees=96, n_features=7, max_depth=7, stop_prob=0.15, n_outputs=20,
                         leaf_width=20, transform=wl.TRANSFORM_SOFTMAX, aggregate=wl.AGG_MEAN)
    for rows in (1, 70, 500):
        info = _check(g, rng.standard_normal((rows, 7)).astype(np.float32))
        assert info["kernel_path"] == 3 and info["workgroup_waves"] == 2
    # plain LDS family: irregular trees over more features than the rank tile has rows
    g = wl.random_forest(902, n_trees=96, n_features=300, max_depth=7, stop_prob=0.1, n_outputs=20,
                         leaf_width=20, transform=wl.TRANSFORM_SOFTMAX, aggregate=wl.AGG_MEAN)
    for rows in (1, 70, 500):
        info = _check(g, rng.standard_normal((rows, 300)).astype(np.float32))
        assert info["kernel_path"] == 0


@pytest.mark.parametrize("rows", [300, 70000])   # a split launch (three kernels) and a plain one
def test_predict_replays_from_a_captured_graph(rows):
    """forest_predict allocates nothing and records only kernels, so a caller can capture it;
    every replay, with eager work and synchronisations in between, must match the oracle."""
    import torch
    import paper_2301_13441_amd as pk
    w = wl.make_workload("c3", n_rows=rows, n_trees=100)
    f = pk.forest_load(w.forest)
    try:
        rng = np.random.default_rng(rows)
        xs = [w.make_x(rows)] + [rng.standard_normal((rows, w.forest.n_features)).astype(np.float32)
                                 for _ in range(2)]
        static_x = torch.zeros((rows, w.forest.n_features), dtype=torch.float32, device="cuda")
        out = torch.zeros(max(f.out_bytes(rows), 4), dtype=torch.uint8, device="cuda")
        static_x.copy_(torch.from_numpy(xs[0]))
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            f.predict(static_x, out=out)          # warm-up outside the capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            scores, labels = f.predict(static_x, out=out)
        for x in xs:
            static_x.copy_(torch.from_numpy(x))
            out.zero_()                           # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            ref = oracle.predict(w.forest, x, want_leaves=False, n_threads=8)
            np.testing.assert_allclose(scores.cpu().numpy(), ref.scores, rtol=RTOL, atol=ATOL)
    finally:
        f.close()


@pytest.mark.parametrize("n_streams", [2, 6])   # within the handle's workspaces, and more streams than it has
def test_small_batches_from_several_streams_on_one_handle(n_streams):
    """Calls on one handle from different streams may overlap whatever the batch size: every
    stream gets a workspace of its own, and a stream that finds none left runs unsplit."""
    import torch
    import paper_2301_13441_amd as pk
    w = wl.make_workload("c2", n_rows=1, n_trees=200)
    F = w.forest.n_features
    f = pk.forest_load(w.forest)
    try:
        rng = np.random.default_rng(n_streams)
        streams = [torch.cuda.Stream() for _ in range(n_streams)]
        rows = [int(r) for r in rng.integers(1, 3000, size=n_streams)]
        xs = [rng.standard_normal((r, F)).astype(np.float32) for r in rows]
        xd = [torch.from_numpy(x).cuda() for x in xs]
        outs = [torch.zeros(max(f.out_bytes(r), 4), dtype=torch.uint8, device="cuda") for r in rows]
        torch.cuda.synchronize()
        got = [None] * n_streams
        for rep in range(20):                     # many calls in flight on every stream
            for i, st in enumerate(streams):
                got[i] = f.predict(xd[i], out=outs[i], stream=st)
        torch.cuda.synchronize()
        for i in range(n_streams):
            ref = oracle.predict(w.forest, xs[i], n_threads=8)
            np.testing.assert_array_equal(got[i][1].cpu().numpy(), ref.labels)
            np.testing.assert_allclose(got[i][0].cpu().numpy(), ref.scores, rtol=RTOL, atol=ATOL)
    finally:
        f.close()


def test_hand_off_from_torch_ops_on_the_same_stream():
    """Hybrid use (Section 4.5): the features are the output of tensor ops on the device and
    the forest consumes them on the same stream, without a host round trip in between."""
    import torch
    import paper_2301_13441_amd as pk
    w = wl.make_workload("c4", n_rows=2000, n_trees=60)
    f = pk.forest_load(w.forest)
    try:
        torch.manual_seed(3)
        a = torch.randn((2000, 32), device="cuda")
        wgt = torch.randn((32, w.forest.n_features), device="cuda")
        feats = torch.relu(a @ wgt).contiguous()      # stays on the device
        scores, labels = f.predict(feats)             # enqueued behind the matmul, no sync
        torch.cuda.synchronize()
        ref = oracle.predict(w.forest, feats.cpu().numpy(), want_leaves=False, n_threads=8)
        np.testing.assert_array_equal(labels.cpu().numpy(), ref.labels)
        np.testing.assert_allclose(scores.cpu().numpy(), ref.scores, rtol=RTOL, atol=ATOL)
    finally:
        f.close()


@pytest.mark.parametrize("case", ["clustered", "one_threshold", "huge_range"])
def test_rank_lookup_with_awkward_threshold_sets(case):
    """Threshold sets that defeat a uniform bucket grid (one crowded bucket, a single threshold,
    a range that overflows float32) must still rank every value exactly."""
    rng = np.random.default_rng(21)
    w = wl.make_workload("c2", n_rows=1, n_trees=40)
    f = w.forest
    thr = f.threshold.copy()
    internal = np.flatnonzero(f.feature >= 0)
    if case == "clustered":
        thr[internal] = np.float32(1.0) + rng.integers(0, 300, internal.size).astype(np.float32) * np.float32(1e-6)
        thr[internal[:3]] = np.float32([-1e30, 0.0, 1e30])
    elif case == "one_threshold":
        thr[internal] = np.float32(0.25)
    else:
        thr[internal[::2]] = np.float32(3e38)
        thr[internal[1::2]] = np.float32(-3e38)
    g = wl.Forest(**{**f.__dict__, "threshold": thr})
    X = rng.standard_normal((700, f.n_features)).astype(np.float32)
    X[:200] = np.float32(1.0) + rng.integers(-5, 305, (200, f.n_features)).astype(np.float32) * np.float32(1e-6)
    X[200:230] = np.float32(0.25)
    X[230:260] = rng.choice(np.float32([3e38, -3e38, np.inf, -np.inf, 0.0]), (30, f.n_features))
    assert _check(g, X)["kernel_path"] == 2


def test_forest_without_trees_returns_the_base_scores():
    f = wl.Forest(n_features=3, n_outputs=3, leaf_width=1, tree_offset=np.zeros(1, np.int64),
                  feature=np.zeros(0, np.int32), threshold=np.zeros(0, np.float32), left=np.zeros(0, np.int32),
                  right=np.zeros(0, np.int32), leaf_value=np.zeros((0, 1), np.float32),
                  tree_output=np.zeros(0, np.int32), aggregate=wl.AGG_SUM,
                  base_score=np.float32([0.25, 1.5, -2.0]), transform=wl.TRANSFORM_SOFTMAX, output=wl.OUT_BOTH)
    X = np.random.default_rng(1).standard_normal((200, 3)).astype(np.float32)
    scores, labels, _, info = _run(f, X, leaves=False)
    ref = oracle.predict(f, X, want_leaves=False)
    np.testing.assert_array_equal(labels, ref.labels)
    np.testing.assert_allclose(scores, ref.scores, rtol=RTOL, atol=ATOL)
    assert np.all(labels == 1) and info["n_trees"] == 0


def test_large_batches_from_two_streams_at_once():
    """Batches of small_batch_rows rows or more touch no state of the handle: two streams may
    run them on one handle concurrently."""
    import torch
    import paper_2301_13441_amd as pk
    w = wl.make_workload("c3", n_rows=70000, n_trees=64)
    f = pk.forest_load(w.forest)
    try:
        assert f.info["small_batch_rows"] <= 70000
        rng = np.random.default_rng(4)
        xs = [w.make_x(70000), rng.standard_normal((70000, w.forest.n_features)).astype(np.float32)]
        xd = [torch.from_numpy(x).cuda() for x in xs]
        outs = [torch.empty(f.out_bytes(70000), dtype=torch.uint8, device="cuda") for _ in xs]
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        torch.cuda.synchronize()
        res = []
        for _ in range(3):                      # interleave launches on the two streams
            res = [f.predict(xd[i], out=outs[i], stream=streams[i]) for i in range(2)]
        torch.cuda.synchronize()
        for i in range(2):
            ref = oracle.predict(w.forest, xs[i], want_leaves=False, n_threads=8)
            np.testing.assert_allclose(res[i][0].cpu().numpy(), ref.scores, rtol=RTOL, atol=ATOL)
    finally:
        f.close()


def test_null_pointers_are_refused_before_any_launch():
    import paper_2301_13441_amd as pk
    w = wl.make_workload("c1", n_rows=10)
    f = pk.forest_load(w.forest)
    try:
        with pytest.raises(pk.ForestError) as e:
            f.predict_raw(0, 10, 0, 0)
        assert e.value.code == -1
        # more rows than one call takes: refused by the size calls and by predict, nothing runs
        for call in (lambda: f.out_bytes(10**9 + 1), lambda: f.out_layout(2**40),
                     lambda: f.predict_raw(256, 10**9 + 1, 256, 0)):
            with pytest.raises(pk.ForestError) as e:
                call()
            assert e.value.code == -7
        assert f.out_bytes(10**9) == 10**9 * 8
        # the binding refuses tensors the kernels would read out of bounds or misinterpret
        import torch
        F = w.forest.n_features
        good = torch.zeros((10, F), dtype=torch.float32, device="cuda")
        for bad in (torch.zeros((10, F - 1), dtype=torch.float32, device="cuda"),       # too few columns
                    torch.zeros((10, F), dtype=torch.float64, device="cuda"),           # wrong dtype
                    torch.zeros((10, F), dtype=torch.float32),                          # host memory
                    torch.zeros((10, 2 * F), dtype=torch.float32, device="cuda")[:, ::2],  # strided
                    torch.zeros((10 * F,), dtype=torch.float32, device="cuda")):        # not a matrix
            with pytest.raises(ValueError):
                f.predict(bad)
            with pytest.raises(ValueError):
                f.predict_leaves(bad)
        with pytest.raises(ValueError):
            f.predict(good, out=torch.empty(8, dtype=torch.uint8, device="cuda"))      # output too small
        f.predict(good)
    finally:
        f.close()


def test_repeated_runs_are_bit_identical():
    import torch
    import paper_2301_13441_amd as pk
    w = wl.make_workload("c4", n_rows=2000, n_trees=300)
    xd = torch.from_numpy(w.make_x(2000)).cuda()
    f = pk.forest_load(w.forest)
    a, la = f.predict(xd)
    a, la = a.clone(), la.clone()
    for _ in range(3):
        b, lb = f.predict(xd)
        assert torch.equal(a, b) and torch.equal(la, lb)
    f.close()


# ----------------------------------------------------------------------------- kernel families

def _full_forest(seed, n_trees, depth, n_features, feature_bias=None, n_outputs=1, **kw):
    rng = np.random.default_rng(seed)
    arrs = wl._full_forest(rng, n_trees, depth, n_features, wl._normal_thr,
                           lambda r, s: r.standard_normal(s, dtype=np.float32))
    if feature_bias is not None:  # send most nodes to feature 0
        internal = arrs["feature"] >= 0
        hit = internal & (rng.random(arrs["feature"].shape) < feature_bias)
        arrs["feature"] = np.where(hit, 0, arrs["feature"]).astype(np.int32)
    out = (rng.integers(0, n_outputs, size=n_trees).astype(np.int32))
    return wl.Forest(n_features=n_features, n_outputs=n_outputs, leaf_width=1, tree_output=out,
                     **arrs, **{"aggregate": wl.AGG_SUM, **kw})


@pytest.mark.parametrize("what,path", [
    ("rank_three_segments", 2),   # > 2 * 12287 distinct thresholds on one feature
    ("rank_wide", 2),             # 128 features -> 128 rank registers (the 3-waves variant)
    ("reg_fallback", 1),          # too many rank registers -> float32 feature registers
    ("ranklds_full_wide", 3),     # full trees over > 128 features: ranks in LDS
    ("ranklds_irregular", 3),     # irregular trees, 3 output columns
    ("ranklds_scalar_columns", 3),  # 10 output columns, scalar leaves: one sum per (wave, column), 12 waves
    ("ranklds_narrow", 3),        # 10-wide vector leaves over 64 features: workgroups of 8 waves
    ("ranklds_four_waves", 3),    # 12-wide vector leaves over 256 features: 4 waves
    ("ranklds_two_waves", 3),     # 32-wide vector leaves: 2 waves
    ("lds_many_outputs", 0),      # full trees over 300 features, 20 columns: more rank rows than the tile holds
    ("lds_generic_many_outputs", 0),
    ("lds_generic_large_trees", 0),   # more than 256 rank rows and trees of ~7000 nodes: plain family, any size
])
def test_kernel_families(what, path):
    rng = np.random.default_rng(42)
    if what == "rank_three_segments":
        f = _full_forest(1, 100, 8, 1)
    elif what == "rank_wide":
        f = _full_forest(2, 30, 7, 128, n_outputs=3, transform=wl.TRANSFORM_SOFTMAX)
    elif what == "reg_fallback":
        f = _full_forest(3, 100, 8, 128, feature_bias=0.9)
    elif what == "ranklds_full_wide":
        f = _full_forest(4, 12, 5, 200)
    elif what == "ranklds_irregular":
        f = wl.random_forest(6, n_trees=37, n_features=11, max_depth=10, stop_prob=0.12, n_outputs=3,
                             transform=wl.TRANSFORM_SOFTMAX)
    elif what == "ranklds_scalar_columns":
        f = wl.random_forest(8, n_trees=45, n_features=64, max_depth=9, stop_prob=0.15, n_outputs=10,
                             transform=wl.TRANSFORM_SOFTMAX)
        f.tree_output[f.tree_output == 4] = 5      # a column no tree feeds, inside the waves' runs
    elif what == "ranklds_narrow":
        f = wl.random_forest(8, n_trees=45, n_features=64, max_depth=9, stop_prob=0.15, n_outputs=10, leaf_width=10,
                             transform=wl.TRANSFORM_SOFTMAX)
    elif what == "ranklds_four_waves":
        f = wl.random_forest(9, n_trees=9, n_features=256, max_depth=13, stop_prob=0.02, n_outputs=12, leaf_width=12,
                             transform=wl.TRANSFORM_SOFTMAX)
    elif what == "ranklds_two_waves":
        f = wl.random_forest(10, n_trees=5, n_features=130, max_depth=13, stop_prob=0.02, n_outputs=32, leaf_width=32,
                             transform=wl.TRANSFORM_SOFTMAX)
    elif what == "lds_many_outputs":
        f = _full_forest(5, 60, 4, 300, n_outputs=20, transform=wl.TRANSFORM_SOFTMAX)
    elif what == "lds_generic_large_trees":
        f = wl.random_forest(11, n_trees=6, n_features=300, max_depth=13, stop_prob=0.02, n_outputs=5, leaf_width=5,
                             transform=wl.TRANSFORM_SOFTMAX)
    else:
        f = wl.random_forest(7, n_trees=41, n_features=300, max_depth=8, stop_prob=0.1, n_outputs=20,
                             transform=wl.TRANSFORM_SOFTMAX)
    X = rng.standard_normal((517, f.n_features)).astype(np.float32)
    # rows that sit exactly on thresholds of their feature
    thr = f.threshold[f.feature == 0]
    X[:64, 0] = np.resize(thr, 64)
    info = _check(f, X)
    assert info["kernel_path"] == path, info
    if what.startswith("ranklds"):
        waves = {"ranklds_narrow": 8, "ranklds_four_waves": 4, "ranklds_two_waves": 2}.get(what, 12)
        assert info["workgroup_waves"] == waves, info


@pytest.mark.parametrize("depth", [1, 2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("leaves", ["one_column", "columns", "vector"])
def test_wide_rank_kernel_every_depth(depth, leaves):
    """65 to 128 rank registers: the kernel that places its matrix-core operands by hand.  Every
    depth has its own number of outcome groups per word (1, 2 or 4) and words per tree (1 to 8);
    scalar leaves into one or several columns and vector leaves take different loops."""
    rng = np.random.default_rng(1000 + depth)
    n_trees = {1: 400, 2: 200, 3: 100, 4: 60, 7: 13, 8: 13}.get(depth, 37)   # > 64 features tested at every depth
    if leaves == "vector":
        arrs = wl._full_forest(rng, n_trees, depth, 100, wl._normal_thr,
                               lambda r, s: r.standard_normal((s[0], s[1] * 3), dtype=np.float32), leaf_width=3)
        f = wl.Forest(n_features=100, n_outputs=3, leaf_width=3, tree_output=np.zeros(n_trees, np.int32),
                      aggregate=wl.AGG_MEAN, transform=wl.TRANSFORM_NONE, **arrs)
    elif leaves == "columns":
        f = _full_forest(2000 + depth, n_trees, depth, 100, n_outputs=4, transform=wl.TRANSFORM_SOFTMAX)
    else:
        f = _full_forest(3000 + depth, n_trees, depth, 100, transform=wl.TRANSFORM_SIGMOID)
    X = rng.standard_normal((389, 100)).astype(np.float32)
    thr = f.threshold[f.feature == 3]
    if thr.size:
        X[:64, 3] = np.resize(thr, 64)      # rows that sit exactly on thresholds
    import paper_2301_13441_amd as pk
    assert 64 < pk.forest_pack(f)["rank_registers"] <= 128
    info = _check(f, X)
    assert info["kernel_path"] == 2 and info["kernel_kind"] == depth, info


@pytest.mark.parametrize("full", [True, False])
def test_every_rank_code_against_every_neighbouring_threshold(full):
    """One feature with integer thresholds 0 .. n - 1 spread over more than two rank registers,
    and rows at every threshold and halfway between neighbours: every code of a register is
    compared with the entries next to it, and with entries far away through the other nodes of
    the row's trees.  Register and LDS rank kernels."""
    rng = np.random.default_rng(5)
    if full:
        f = _full_forest(12, 3600, 3, 1)
    else:
        f = wl.random_forest(12, n_trees=900, n_features=1, max_depth=6, stop_prob=0.05)
    internal = np.flatnonzero(f.feature >= 0)
    n = internal.size
    assert n > 2 * 12287
    f.threshold[internal] = rng.permutation(n).astype(np.float32)
    X = np.arange(-1.0, n + 0.5, 0.5, dtype=np.float32).reshape(-1, 1)
    info = _check(f, X)
    assert info["kernel_path"] == (2 if full else 3), info


@pytest.mark.parametrize("full", [True, False])
def test_x_at_a_four_byte_aligned_address(full):
    """X is only promised to be float32-aligned: rows of 13 floats starting one float into an
    allocation (the kernels read neighbouring features of a row with wider loads)."""
    import torch
    import paper_2301_13441_amd as pk
    F, n = 13, 700
    f = _full_forest(31, 20, 5, F) if full else wl.random_forest(31, n_trees=20, n_features=F, max_depth=9, stop_prob=0.1)
    X = np.random.default_rng(8).standard_normal((n, F)).astype(np.float32)
    buf = torch.zeros(n * F + 1, dtype=torch.float32, device="cuda")
    xd = buf[1:].view(n, F)
    xd.copy_(torch.from_numpy(X))
    assert xd.data_ptr() % 8 == 4 and xd.is_contiguous()
    ref = oracle.predict(f, X, n_threads=8)
    h = pk.forest_load(f)
    try:
        scores, labels = h.predict(xd)
        torch.cuda.synchronize()
        assert h.info["kernel_path"] == (2 if full else 3)
        np.testing.assert_allclose(scores.cpu().numpy(), ref.scores, rtol=RTOL, atol=ATOL)
    finally:
        h.close()


def test_duplicate_thresholds_and_unused_features():
    w = wl.make_workload("c3", n_rows=700, n_trees=60)      # thresholds from a 255-value grid
    f = w.forest
    feat = np.where(f.feature >= 0, f.feature % 7, f.feature).astype(np.int32)  # 43 features unused
    g = wl.Forest(**{**f.__dict__, "feature": feat})
    X = w.make_x(700).copy()
    grid = wl.normal_quantile_grid(255)
    X[:300, :7] = grid[np.random.default_rng(3).integers(0, 255, size=(300, 7))]  # x == threshold
    assert _check(g, X)["kernel_path"] == 2


# ----------------------------------------------------------------------------- full-size runs

def _full_size(name):
    """The bench's launch configuration (full row count, device-resident X): scores and labels of
    EVERY row are compared with the oracle, and the leaf ids of every tree on the first 65 536
    rows plus 65 536 seeded random rows.  X is drawn chunk by chunk; each chunk goes to the device
    and through the oracle, so the host never holds more than one chunk and the sampled rows."""
    import os
    import torch
    import paper_2301_13441_amd as pk
    w = wl.make_workload(name)
    n, F, K = w.n_rows, w.forest.n_features, w.forest.n_outputs
    threads = max(1, min(os.cpu_count() or 1, 16))
    rng = np.random.default_rng(wl.SEEDS[name] + 7)
    n_head = min(n, 65536)
    pick = np.unique(np.concatenate([np.arange(n_head), rng.integers(0, n, size=65536)]))
    xd = torch.empty((n, F), dtype=torch.float32, device="cuda")
    xs = np.empty((len(pick), F), dtype=np.float32)
    ref_scores = np.empty((n, K), dtype=np.float32)
    ref_labels = np.empty((n,), dtype=np.int32)
    pos = 0
    for chunk in w.x_chunks(n):
        xd[pos:pos + len(chunk)].copy_(torch.from_numpy(chunk))
        sel = pick[(pick >= pos) & (pick < pos + len(chunk))]
        xs[np.searchsorted(pick, sel)] = chunk[sel - pos]
        ref = oracle.predict(w.forest, chunk, n_threads=threads)
        ref_scores[pos:pos + len(chunk)] = ref.scores
        ref_labels[pos:pos + len(chunk)] = ref.labels
        pos += len(chunk)
    f = pk.forest_load(w.forest)
    try:
        scores, labels = f.predict(xd)
        torch.cuda.synchronize()
        got_scores = None if scores is None else scores.cpu().numpy()
        got_labels = None if labels is None else labels.cpu().numpy()
        # leaf ids: every tree, on the sampled rows (a batch large enough to run the same kernels)
        lv = f.predict_leaves(xd[torch.from_numpy(pick).cuda()].contiguous())
        torch.cuda.synchronize()
        got_leaves = lv.cpu().numpy()
        info = f.info
    finally:
        f.close()
    assert len(pick) >= info["small_batch_rows"]
    if got_labels is not None:
        np.testing.assert_array_equal(got_labels, ref_labels)
    if got_scores is not None:
        np.testing.assert_allclose(got_scores, ref_scores, rtol=RTOL, atol=ATOL)
    del got_scores, got_labels, ref_scores, ref_labels
    ref_leaves = oracle.predict(w.forest, xs, want_leaves=True, n_threads=threads).leaf_node_id
    np.testing.assert_array_equal(got_leaves, ref_leaves)
    return info


@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
def test_full_size_all_rows(name):
    info = _full_size(name)
    assert info["n_trees"] == {"c2": 500, "c3": 1000, "c4": 2000, "c5": 128}[name]


def test_input_larger_than_2_to_31_elements():
    """Row offsets past 2^31 elements (and 2^33 bytes) of X: 80,000,000 rows of 28 features,
    drawn on the device; the oracle checks the first and last rows and seeded rows between,
    most of them beyond the 2^31st element."""
    import torch
    import paper_2301_13441_amd as pk
    w = wl.make_workload("c2", n_rows=1, n_trees=8)
    F = w.forest.n_features
    n = 80_000_000
    assert n * F > 2**31
    gen = torch.Generator(device="cuda").manual_seed(99)
    xd = torch.empty((n, F), dtype=torch.float32, device="cuda")
    step = 10_000_000
    for pos in range(0, n, step):
        xd[pos:pos + step].normal_(generator=gen)
    rng = np.random.default_rng(99)
    pick = np.unique(np.concatenate([np.arange(300), np.arange(n - 300, n), rng.integers(0, n, 4000),
                                     rng.integers(2**31 // F, n, 4000)]))
    idx = torch.from_numpy(pick).cuda()
    xs = xd[idx].cpu().numpy()
    f = pk.forest_load(w.forest)
    try:
        scores, labels = f.predict(xd)
        torch.cuda.synchronize()
        got_scores, got_labels = scores[idx].cpu().numpy(), labels[idx].cpu().numpy()
    finally:
        f.close()
    ref = oracle.predict(w.forest, xs, n_threads=8)
    np.testing.assert_array_equal(got_labels, ref.labels)
    np.testing.assert_allclose(got_scores, ref.scores, rtol=RTOL, atol=ATOL)


def test_compare_rate_probe_runs_and_counts():
    """The bench's measurement aid: runs to completion, leaves its word alone, counts what it did."""
    import torch
    from paper_2301_13441_amd import binding
    word = torch.full((1,), 7, dtype=torch.int32, device="cuda")
    n = binding.forest_probe_compare_rate(100, word)
    torch.cuda.synchronize()
    assert n == 256 * 8 * 256 * 2 * 16 * 100 and int(word.item()) == 7
