"""Host model compiler (no GPU): numbering of Section 3.1.2, the structure Table 2 implies,
error codes, kernel-family choice.  Runs the packer through the C ABI (forest_pack)."""
import ctypes

import numpy as np
import pytest

import paper_2301_13441_amd as pk
from paper_2301_13441_amd import binding
import workloads as wl
import oracle
from oracle import matrix_form as mf


def _lib():
    return pk.load_library()


def test_library_exports_every_declared_symbol():
    import os
    import re
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    lib = _lib()
    for header, names in (("forest.h", binding.EXPORTS), ("forest_testing.h", binding.TESTING_EXPORTS)):
        declared = set(re.findall(r"\b(forest_[a-z_]+)\s*\(", open(os.path.join(inc, header)).read()))
        assert declared == set(names), header
        for name in declared:
            assert getattr(lib, name) is not None
    assert lib.forest_strerror(-2) == b"malformed tree"


@pytest.mark.parametrize("seed", range(6))
def test_numbering_matches_level_order_and_in_order(seed):
    f = wl.random_forest(900 + seed, n_trees=7, n_features=5, max_depth=6, stop_prob=0.25)
    v = pk.forest_pack(f)
    assert v["kernel_kind"] == 0
    for t, (ft, thr, l, r, val) in enumerate(mf.split_trees(f)):
        m = mf.tree_matrices(5, ft, thr, l, r, val)     # independent numbering, written from the paper
        a, b = v["node_base"][t], v["node_base"][t + 1]
        la, lb = v["leaf_base"][t], v["leaf_base"][t + 1]
        assert b - a == len(m.internal_nodes) == v["tree_n_internal"][t]
        assert lb - la == len(m.leaf_nodes) == (b - a) + 1            # N_L = N_I + 1
        assert v["leaf_node"][la:lb].tolist() == m.leaf_nodes          # leaves in in-order
        assert v["split_feature"][a:b].tolist() == [int(ft[n]) for n in m.internal_nodes]
        np.testing.assert_array_equal(v["split_threshold"][a:b], m.W2)  # W2 in level order
        np.testing.assert_array_equal(v["leaf_value"][la:lb], m.E)
        # child references reproduce C: leaf j is left of I_i iff reachable through child_left
        ord_of = {n: i for i, n in enumerate(m.internal_nodes)}
        leaf_of = {n: j for j, n in enumerate(m.leaf_nodes)}
        for i, n in enumerate(m.internal_nodes):
            for side, table in ((l, "child_left"), (r, "child_right")):
                c = int(side[n])
                want = ord_of[c] if ft[c] >= 0 else ~leaf_of[c]
                assert v[table][a + i] == want


def test_full_trees_are_detected_with_their_depth():
    for name, kind in (("c1", 4), ("c2", 8), ("c3", 6), ("c4", 6)):
        w = wl.make_workload(name, n_rows=1, n_trees=6)
        v = pk.forest_pack(w.forest)
        assert v["kernel_kind"] == kind
        assert (v["tree_is_full"] == 1).all() and (v["tree_depth"] == kind).all()
    w = wl.make_workload("c5", n_rows=1, n_trees=3)
    v = pk.forest_pack(w.forest)
    assert v["kernel_kind"] == 0 and (v["tree_is_full"] == 0).all() and v["tree_depth"].max() <= 12


def _bad(forest, code):
    with pytest.raises(pk.ForestError) as e:
        pk.forest_pack(forest)
    assert e.value.code == code, e.value


def test_error_paths_need_no_gpu():
    base = wl.random_forest(1, n_trees=3, n_features=4, max_depth=4, allow_single_leaf=False)
    internal = np.flatnonzero(base.feature >= 0)

    def clone(**kw):
        return wl.Forest(**{**base.__dict__, **{k: np.array(v) if isinstance(v, np.ndarray) else v
                                                  for k, v in kw.items()}})

    f = clone(feature=base.feature.copy()); f.feature[internal[0]] = 4
    _bad(f, -3)                                           # feature >= n_features
    f = clone(threshold=base.threshold.copy()); f.threshold[internal[1]] = np.nan
    _bad(f, -4)                                           # NaN threshold
    f = clone(left=base.left.copy()); f.left[internal[0]] = 10_000
    _bad(f, -2)                                           # child out of range
    f = clone(left=base.left.copy()); f.left[internal[0]] = 0
    _bad(f, -2)                                           # cycle back to the root
    f = clone(right=base.right.copy()); f.right[internal[0]] = f.left[internal[0]]
    _bad(f, -2)                                           # node reached twice (and one unreachable)
    _bad(clone(leaf_width=2), -1)                         # leaf_width is 1 or K
    _bad(clone(aggregate=7), -1)
    _bad(clone(transform=wl.TRANSFORM_SOFTMAX), -1)       # softmax needs K >= 2
    _bad(clone(n_outputs=33, leaf_width=1), -7)           # documented limit
    _bad(clone(tree_output=np.asarray([0, 5, 0], np.int32)), -1)
    off = base.tree_offset.copy(); off[1] = off[0]
    _bad(clone(tree_offset=off), -2)                      # empty tree
    # +-Inf thresholds are legal
    f = clone(threshold=base.threshold.copy()); f.threshold[internal[0]] = np.inf
    pk.forest_pack(f)
    # null pointers
    lib = _lib()
    h = ctypes.c_void_p()
    assert lib.forest_pack(None, ctypes.byref(h)) == -1
    assert lib.forest_load(None, ctypes.byref(h)) == -1
    assert lib.forest_out_bytes(None, 5) == -1
    assert lib.forest_predict(None, None, 5, None, None) == -1
    lib.forest_free(None)
    lib.forest_pack_free(None)


def _chain_forest(depth, n_features, n_trees=3, n_outputs=1, leaf_width=1, seed=0, **kw):
    """Trees that are one long path: internal node i has a leaf on one side (which side is
    drawn) and node i + 1 on the other; `depth` tests on the longest path."""
    rng = np.random.default_rng(seed)
    n = 2 * depth + 1
    feature, threshold, left, right = [], [], [], []
    for _ in range(n_trees):
        f = np.full(n, -1, np.int32); t = np.zeros(n, np.float32)
        l = np.full(n, -1, np.int32); r = np.full(n, -1, np.int32)
        for i in range(depth):                      # internal nodes 0..depth-1, leaves depth..2*depth
            f[i] = rng.integers(0, n_features); t[i] = rng.standard_normal()
            nxt, leaf = (i + 1 if i + 1 < depth else 2 * depth), depth + i
            l[i], r[i] = (nxt, leaf) if rng.random() < 0.5 else (leaf, nxt)
        feature.append(f); threshold.append(t); left.append(l); right.append(r)
    vals = rng.standard_normal((n_trees * n, leaf_width)).astype(np.float32)
    feat = np.concatenate(feature)
    vals[feat >= 0] = 0
    return wl.Forest(n_features=n_features, n_outputs=n_outputs, leaf_width=leaf_width,
                     tree_offset=np.arange(n_trees + 1, dtype=np.int64) * n, feature=feat,
                     threshold=np.concatenate(threshold), left=np.concatenate(left), right=np.concatenate(right),
                     leaf_value=vals, tree_output=(rng.integers(0, n_outputs, n_trees).astype(np.int32)
                                                   if leaf_width == 1 else np.zeros(n_trees, np.int32)), **kw)


def test_documented_limits_are_the_limits():
    """Just inside every documented limit packs; just outside is refused with the limit code."""
    pk.forest_pack(_chain_forest(64, 5))
    _bad(_chain_forest(65, 5), -7)                          # FOREST_MAX_DEPTH
    pk.forest_pack(_chain_forest(3, 4096))
    _bad(_chain_forest(3, 4097), -7)                        # FOREST_MAX_FEATURES
    pk.forest_pack(_chain_forest(3, 6, n_outputs=32))
    _bad(_chain_forest(3, 6, n_outputs=33), -7)             # FOREST_MAX_OUTPUTS


def test_load_without_device_reports_hip_error_not_crash():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a device is present")
    w = wl.make_workload("c1", n_rows=1)
    with pytest.raises(pk.ForestError) as e:
        pk.forest_load(w.forest)
    assert e.value.code == -6


def test_kernel_family_choice():
    import sys, os
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    from test_gpu_parity import _full_forest
    v = pk.forest_pack(_full_forest(1, 100, 8, 1))
    assert v["kernel_path"] == 2 and v["rank_registers"] == 3       # 25500 thresholds on one feature: 3 segments
    v = pk.forest_pack(_full_forest(1, 40, 8, 2))
    assert v["kernel_path"] == 2 and v["rank_registers"] == 2       # 5096 and 5104 thresholds: one segment each
    v = pk.forest_pack(_full_forest(2, 30, 7, 128))
    assert v["kernel_path"] == 2 and v["rank_registers"] == 128
    v = pk.forest_pack(_full_forest(3, 100, 8, 128, feature_bias=0.9))
    assert v["kernel_path"] == 1                                     # 130 rank registers would be needed
    assert pk.forest_pack(_full_forest(4, 12, 5, 200))["kernel_path"] == 3      # too wide for registers
    assert pk.forest_pack(_full_forest(5, 60, 4, 9, n_outputs=20))["kernel_path"] == 3     # 20 columns of scalar leaves
    assert pk.forest_pack(_full_forest(5, 60, 4, 300, n_outputs=20))["kernel_path"] == 0   # more than 256 rank rows
    irregular = wl.random_forest(9, n_trees=5, n_features=6, max_depth=7)
    assert pk.forest_pack(irregular)["kernel_path"] == 3
    many = wl.random_forest(9, n_trees=5, n_features=6, max_depth=7, n_outputs=20)
    v = pk.forest_pack(many)
    assert v["kernel_path"] == 3 and v["workgroup_waves"] == 12       # scalar leaves: one sum per (wave, column)
    many = wl.random_forest(9, n_trees=5, n_features=6, max_depth=7, n_outputs=20, leaf_width=20)
    v = pk.forest_pack(many)
    assert v["kernel_path"] == 3 and v["workgroup_waves"] == 2        # 20-wide leaves: three workgroups of 2 waves per CU
    wide = wl.random_forest(9, n_trees=40, n_features=300, max_depth=9, stop_prob=0.05)
    assert pk.forest_pack(wide)["kernel_path"] == 0                   # more than 256 rank rows: plain family
    w = wl.make_workload("c5", n_rows=1, n_trees=4)
    v = pk.forest_pack(w.forest)
    assert v["kernel_path"] == 3 and v["rank_registers"] == 256
    w = wl.make_workload("c2", n_rows=1)
    v = pk.forest_pack(w.forest)
    assert v["kernel_path"] == 2 and v["rank_registers"] == 28       # ~4550 thresholds per feature


def test_lds_rank_family_cuts_the_trees_into_balanced_runs():
    """Irregular trees: each wave of a workgroup gets a contiguous run of trees, the runs cover
    every tree once, and the longest run is the shortest any contiguous cut allows (brute force
    over all cuts on a small forest; never longer than the equal-count cut on c5)."""
    import itertools
    small = wl.random_forest(21, n_trees=9, n_features=6, max_depth=9, stop_prob=0.1, n_outputs=3)
    for forest in (small, wl.make_workload("c5", n_rows=1).forest):
        v = pk.forest_pack(forest)
        assert v["kernel_path"] == 3
        waves, cut, groups = v["workgroup_waves"], v["wave_tree"], v["program_groups"].astype(np.int64)
        T = forest.n_trees
        assert waves in (8, 12) and len(cut) == waves + 1
        assert cut[0] == 0 and cut[-1] == T and (np.diff(cut) >= 0).all()
        cost = groups + 2
        run = lambda a, b: int(cost[a:b].sum())
        longest = max(run(cut[w], cut[w + 1]) for w in range(waves))
        equal = max(run(T * w // waves, T * (w + 1) // waves) for w in range(waves))
        assert longest <= equal
        if T <= 9:
            best = min(max(run(a, b) for a, b in zip((0,) + c, c + (T,)))
                       for c in itertools.combinations_with_replacement(range(T + 1), waves - 1))
            assert longest == best
        else:
            print("c5: longest run", longest, "equal-count cut", equal, "mean", cost.sum() / waves)


def _bucket_of(x, lo, scale, count):
    """bucket_index of the library, in float32 like the kernels."""
    with np.errstate(all="ignore"):   # inf * 0 = NaN is a bucket-0 case, as in the library
        t = (np.float32(x) - np.float32(lo)) * np.float32(scale)
    if not t > 0:
        return 0
    if t >= np.float32(count):
        return int(count) - 1
    return int(t)


@pytest.mark.parametrize("case", ["normal", "grid", "with_infinities", "one_threshold", "clustered"])
def test_rank_bucket_tables_bracket_every_rank(case):
    """The rank families turn x into #{thresholds < x} through a bucket table: for every feature
    the table entry of x's bucket and the next one must bracket the true rank, for values between,
    on and beyond the thresholds."""
    rng = np.random.default_rng(11)
    if case == "grid":
        f = wl.make_workload("c3", n_rows=1, n_trees=60).forest
    else:
        f = wl.make_workload("c2", n_rows=1, n_trees=30).forest
        thr = f.threshold.copy()
        internal = np.flatnonzero(f.feature >= 0)
        if case == "with_infinities":
            thr[internal[::9]] = np.inf
            thr[internal[4::13]] = -np.inf
        elif case == "one_threshold":
            thr[internal] = np.float32(0.25)
        elif case == "clustered":   # almost every threshold in one bucket of the uniform grid
            thr[internal] = (np.float32(1.0) + rng.integers(0, 50, internal.size).astype(np.float32) * np.float32(1e-6))
            thr[internal[:3]] = np.float32([-1e30, 0.0, 1e30])
        f = wl.Forest(**{**f.__dict__, "threshold": thr})
    v = binding.forest_pack(f)
    assert v["kernel_path"] in (2, 3)
    tb = v["rank_threshold_base"]
    for feat in range(f.n_features):
        thr = v["rank_threshold"][tb[feat]:tb[feat + 1]]
        want = np.unique(f.threshold[f.feature == feat])
        np.testing.assert_array_equal(thr, want)      # distinct, ascending
        lo, scale = v["rank_bucket_lo"][feat], v["rank_bucket_scale"][feat]
        count, base = v["rank_bucket_count"][feat], v["rank_bucket_base"][feat]
        start = v["rank_bucket_start"][base:base + count + 1]
        assert count >= 1 and start[0] == 0 and start[-1] == len(thr)
        assert np.all(np.diff(start) >= 0)
        probes = [np.float32(x) for x in (-np.inf, np.inf, 0.0, -0.0, 1e-45, -3e38, 3e38)]
        finite = thr[np.isfinite(thr)]
        for t in finite[:: max(1, len(finite) // 40)]:
            probes += [t, np.nextafter(t, np.float32(-np.inf)), np.nextafter(t, np.float32(np.inf))]
        probes += list(rng.standard_normal(40).astype(np.float32) * np.float32(2.0))
        for x in probes:
            rank = int(np.sum(thr < x))
            b = _bucket_of(x, lo, scale, count)
            assert start[b] <= rank <= start[b + 1], (case, feat, float(x), b)


def _simulate_bank_program(f, v, X):
    """Leaf node reached per (row, caller tree), computed from the register-bank program alone:
    every entry of every wave's stream is decoded back to (feature, threshold) and compared as
    float32, the outcome goes to the entry's bit of the batch buffer, then the child references
    are followed from each tree's root.  Nothing of the kernels' rank arithmetic is used."""
    n_codes, _, _ = binding.forest_rank_code(0)
    seg = n_codes - 1
    entry_to_j = {binding.forest_rank_code(q)[2]: q for q in range(n_codes)}
    tbase = v["rank_threshold_base"]
    n_thr = np.diff(tbase)
    regs_of = (n_thr + seg - 1) // seg
    vfirst = np.concatenate([[0], np.cumsum(regs_of)])
    reg_feature = np.repeat(np.arange(len(n_thr)), regs_of)
    nb, nw, nt, U = v["bank_batches"], v["bank_waves"], v["bank_trees"], v["bank_unit"]
    T = len(f.tree_offset) - 1
    out = np.full((len(X), T), -1, dtype=np.int64)
    cursor = v["bank_stream_base"].astype(np.int64).copy()
    for b in range(nb):
        n_units = int(v["bank_span"][b, :, 0].sum())
        assert n_units <= v["bank_max_units"]
        bits = np.zeros((len(X), n_units * U), dtype=bool)
        for w in range(nw):
            units, base = (int(z) for z in v["bank_span"][b, w])
            for k in range(units * U):
                e = int(v["bank_prog"][cursor[w] + k])
                reg = int(v["bank_reg"][w, e & 0xff])
                jl = entry_to_j[e >> 16]
                slot = (base + k // U) * U + 8 * ((k // 8) % (U // 8)) + 7 - k % 8
                if jl == seg:              # padding: compares against the largest code, never true
                    continue
                feat = int(reg_feature[reg])
                thr = v["rank_threshold"][tbase[feat] + (reg - vfirst[feat]) * seg + jl]
                bits[:, slot] = ~(X[:, feat] <= thr)
            cursor[w] += units * U
        slot_base, n_slots, steps = (int(z) for z in v["bank_batch"][b, :3])
        assert n_slots == n_units * U
        child = v["bank_child"][slot_base:slot_base + n_slots].astype(np.int64)
        leaves = v["bank_leaf"][slot_base:slot_base + n_slots].astype(np.int64)
        for j in range(nt):
            root, leaf_base, caller, valid = (int(z) for z in v["bank_tree"][b, j])
            if not valid:
                continue
            if root & 0x8000:  # a single leaf
                leaf = np.full(len(X), leaf_base, dtype=np.int64)
            else:
                at = np.full(len(X), root, dtype=np.int64)
                for _ in range(steps):
                    assert (at % 4 == 0).all() and (at // 4 < n_slots).all()
                    at = np.where(bits[np.arange(len(X)), at // 4], child[at // 4] >> 16, child[at // 4] & 0xffff)
                picked = np.where(bits[np.arange(len(X)), at // 4], leaves[at // 4] >> 16, leaves[at // 4] & 0xffff)
                assert (picked != 0xffff).all()  # the walk has reached a node whose chosen child is a leaf
                leaf = leaf_base + picked
            assert (v["order_leaf_tree"][leaf] == caller).all()
            out[:, caller] = v["order_leaf_node"][leaf]
    return out


@pytest.mark.parametrize("seed", range(6))
def test_register_bank_program_reaches_the_oracles_leaves(seed):
    rng = np.random.default_rng(40 + seed)
    F = int(rng.choice([3, 40, 256]))
    f = wl.random_forest(950 + seed, n_trees=int(rng.integers(1, 14)), n_features=F, max_depth=int(rng.integers(1, 10)),
                         stop_prob=0.15, n_outputs=(2 if seed % 2 else 1), leaf_width=(2 if seed % 2 else 1),
                         grid_thresholds=bool(seed % 3 == 0))
    v = pk.forest_pack(f)
    assert v["kernel_path"] == 3 and v["bank_batches"] == -(-(len(f.tree_offset) - 1) // v["bank_trees"])
    X = rng.standard_normal((150, F)).astype(np.float32)
    if seed % 3 == 0:
        X = np.round(X * 2) / 2
    X[0, :] = np.nan
    ref = oracle.predict(f, X, want_leaves=True)
    np.testing.assert_array_equal(_simulate_bank_program(f, v, X), ref.leaf_node_id)
    # every internal node sits in exactly one slot, and each wave holds at most bank_regs registers
    used = int((v["bank_leaf"] != 0x80008000).sum())
    assert used == int(v["tree_n_internal"].sum())


def _bank_lookup_codes(v, f, x):
    """Ranks of the values `x` of feature `f` as the register-bank kernel's fast lookup finds them
    (numpy float32 arithmetic in the kernel's order); -1 where the window does not settle the
    rank and the kernel takes the general lookup instead."""
    lo, scale, last = (v["fast_feat"][f, :3].copy().view(np.float32))
    n, tab_off, thr_off, fast = (int(z) for z in v["fast_feat"][f, 3:7])
    assert fast == 1
    W = v["fast_window"]
    thr = v["rank_threshold"][thr_off // 4: thr_off // 4 + n]
    with np.errstate(invalid="ignore", over="ignore"):
        t = (x.astype(np.float32) - lo) * scale
        t = np.where(np.isnan(t), np.float32(0), t)  # maximum and minimum drop a NaN operand
        bucket = np.minimum(np.maximum(t, np.float32(0)), last).astype(np.int64)
    at = v["fast_tab"][tab_off // 2 + bucket].astype(np.int64)
    assert (at >= 0).all() and (at <= n - W).all()
    win = thr[at[:, None] + np.arange(W)[None, :]]
    below = win < x[:, None]
    rank = at + below.sum(axis=1)
    unsettled = (~below[:, 0] & (at != 0)) | (below[:, -1] & (at != n - W)) | np.isnan(x)
    return np.where(unsettled, -1, rank)


@pytest.mark.parametrize("seed", range(4))
def test_register_bank_prologue_plan_and_fast_lookup(seed):
    """Every rank register is looked up exactly once, by the wave that holds it, in the pass that
    stages its feature; and the fast lookup's table and window give rank(x) = #{thresholds < x}
    wherever the window settles it, which is almost everywhere."""
    rng = np.random.default_rng(90 + seed)
    F = int(rng.choice([5, 70, 256]))
    f = wl.random_forest(990 + seed, n_trees=12, n_features=F, max_depth=10, stop_prob=0.1,
                         grid_thresholds=bool(seed % 2))
    v = pk.forest_pack(f)
    assert v["kernel_path"] == 3 and v["bank_batches"] > 0
    tbase = v["rank_threshold_base"]
    seen = set()
    for p, (f0, f1) in enumerate(v["bank_pass"]):
        assert 0 < f1 - f0 <= 64 and f0 % 64 == 0
        for w in range(v["bank_waves"]):
            begin, n_fast, n_slow, _ = (int(z) for z in v["bank_pass_wave"][p, w])
            for i in range(begin, begin + n_fast + n_slow):
                slot, feat, first, length = (int(z) for z in v["bank_todo"][i])
                assert f0 <= feat < f1 and 0 <= slot < v["bank_regs"]
                n = int(tbase[feat + 1] - tbase[feat])
                assert first % 12287 == 0 and length == min(n - first, 12287)
                assert (int(v["fast_feat"][feat, 6]) == 1) == (i < begin + n_fast)
                reg = int(v["bank_reg"][w, slot])
                assert reg not in seen
                seen.add(reg)
    assert seen == set(range(v["rank_registers"]))
    settled = total = 0
    for feat in range(F):
        n = int(tbase[feat + 1] - tbase[feat])
        if int(v["fast_feat"][feat, 6]) != 1:
            assert n < v["fast_window"] or n > 6143
            continue
        thr = v["rank_threshold"][tbase[feat]:tbase[feat + 1]]
        x = np.concatenate([rng.standard_normal(400).astype(np.float32) * 2, thr, np.nextafter(thr, np.float32(np.inf)),
                            np.nextafter(thr, np.float32(-np.inf)),
                            np.array([np.nan, np.inf, -np.inf, 0.0, -0.0, 3e38, -3e38], dtype=np.float32)])
        got = _bank_lookup_codes(v, feat, x)
        want = np.searchsorted(thr, x, side="left")  # #{thr < x}
        ok = got >= 0
        np.testing.assert_array_equal(got[ok], want[ok])
        assert not ok[np.isnan(x)].any()
        settled += int(ok.sum())
        total += len(x)
    assert total == 0 or settled >= 0.98 * total


def test_register_bank_program_only_where_it_fits():
    # one tree of thousands of internal nodes: its batch buffer would not fit the LDS budget
    big = wl.random_forest(7, n_trees=1, n_features=20, max_depth=14, stop_prob=0.02, allow_single_leaf=False)
    v = pk.forest_pack(big)
    assert v["tree_n_internal"][0] > 2400 and v["kernel_path"] == 3 and v["bank_batches"] == 0
    # many output columns keep the LDS-resident kernel
    wide = wl.random_forest(8, n_trees=9, n_features=20, max_depth=6, n_outputs=5, leaf_width=5)
    assert pk.forest_pack(wide)["bank_batches"] == 0


def test_pinned_stream_register_check_catches_a_violation():
    """The build does not ship the streaming form of the LDS rank kernel when compiler-generated
    code touches the pinned stream registers between two evaluation statements (it builds the
    conservative form instead, tests/test_build.py); the checker itself is tested here on a
    miniature of the assembly's structure."""
    from paper_2301_13441_amd import check_stream_registers as chk
    clean = "\n".join([
        ".LBB0_1:                                ; =>This Loop Header: Depth=1",
        "\t;;#ASMSTART", "\tv_and_or_b32 v112, s36, v1, v2", "\ts_load_dwordx16 s[36:51], s[2:3], 0x80", "\t;;#ASMEND",
        "\tv_add_u32 v3, v3, v4",
        ".LBB0_2:                                ;   in Loop: Header=BB0_1 Depth=1",
        "\ts_add_u32 s2, s2, 0x80", "\ts_cbranch_scc1 .LBB0_1",
        ".LBB0_3:", "\ts_mov_b32 s40, 0", "\ts_endpgm"])
    assert chk.check_assembly(clean) == 1
    dirty = clean.replace("\ts_add_u32 s2, s2, 0x80", "\ts_add_u32 s2, s2, 0x80\n\ts_mov_b32 s44, s7")
    with pytest.raises(RuntimeError, match="pinned stream register"):
        chk.check_assembly(dirty)
    with pytest.raises(RuntimeError, match="no stream loop"):
        chk.check_assembly("\ts_endpgm")


def test_bench_refuses_more_than_one_gpu():
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_rank_codes_compare_exactly():
    """The rank families replace x <= tau by a comparison of f16 codes (dtype rewriting,
    Section 4.3.1): for every local rank q and threshold index j of a rank register,
    clamp(fma(code(q), 4, entry(j))) rounded once to f16 must be 1 iff q > j and 0 otherwise.
    Checked for all pairs, with the fused multiply-add taken exactly in float64 (the operands are
    f16 values, so 4 * code + entry is exact there) and rounded to f16 by numpy."""
    n, _, _ = binding.forest_rank_code(0)
    codes = np.empty(n, np.uint16)
    entries = np.empty(n, np.uint16)
    for q in range(n):
        _, codes[q], entries[q] = binding.forest_rank_code(q)
    c = codes.view(np.float16).astype(np.float64)
    e = entries.view(np.float16).astype(np.float64)
    assert np.isfinite(c).all() and np.isfinite(e).all()
    assert (np.diff(c) > 0).all()                       # strictly increasing in q
    assert np.array_equal(e, -4.0 * c)
    with pytest.raises(binding.ForestError):
        binding.forest_rank_code(n)
    with pytest.raises(binding.ForestError):
        binding.forest_rank_code(-1)
    q = np.arange(n)
    with np.errstate(over="ignore"):
        for j0 in range(0, n, 512):
            j = np.arange(j0, min(j0 + 512, n))
            fused = (4.0 * c[:, None] + e[None, j]).astype(np.float16)      # one rounding, +-Inf on overflow
            bit = np.clip(fused.astype(np.float64), 0.0, 1.0)
            assert np.array_equal(bit, (q[:, None] > j[None, :]).astype(np.float64)), j0
    # one register covers one threshold fewer than there are codes
    f = _chain_forest(3, 1, n_trees=n // 3 + 1)
    internal = np.flatnonzero(f.feature >= 0)
    assert internal.size >= n
    f.threshold[internal] = np.minimum(np.arange(internal.size), n - 2).astype(np.float32)   # n - 1 distinct
    assert pk.forest_pack(f)["rank_registers"] == 1
    f.threshold[internal] = np.minimum(np.arange(internal.size), n - 1).astype(np.float32)   # n distinct
    assert pk.forest_pack(f)["rank_registers"] == 2


def test_compare_rate_probe_refuses_bad_arguments_before_any_launch():
    import ctypes
    lib = binding.load_library()
    lib.forest_probe_compare_rate.restype = ctypes.c_int
    lib.forest_probe_compare_rate.argtypes = [ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                              ctypes.POINTER(ctypes.c_int64)]
    n = ctypes.c_int64(-1)
    assert lib.forest_probe_compare_rate(0, None, ctypes.c_void_p(16), ctypes.byref(n)) < 0
    assert lib.forest_probe_compare_rate(1 << 25, None, ctypes.c_void_p(16), ctypes.byref(n)) < 0
    assert lib.forest_probe_compare_rate(10, None, None, ctypes.byref(n)) < 0
    assert lib.forest_probe_compare_rate(10, None, ctypes.c_void_p(16), None) < 0
    assert n.value == -1


def test_staged_positions_of_full_trees_and_the_table_walk():
    """Depths 4..8 on the rank path keep a tree's outcome bits in fields a table walk reads three
    levels at a time (Section 3.1.2: all internal nodes are evaluated; the leaf reached is the one
    whose root path agrees with the outcomes); depths 7 and 8 do so for levels 0..4 and keep the
    subtrees rooted at level 5 in fields of their own behind position 32.  The position map must be a bijection onto the tree's nodes, and the walk over it
    -- simulated here exactly as the kernel takes it -- must end on the leaf the heap walk ends on,
    for every depth and many outcome patterns."""
    rng = np.random.default_rng(46)

    def path3(t):       # path through a complete 3-level subtree, local heap order
        p = 1
        for _ in range(3):
            p = 2 * p + ((t >> (p - 1)) & 1)
        return p - 8

    for depth in (4, 5, 6, 7, 8):
        n_pos, n_int = 1 << depth, (1 << depth) - 1
        node_at = [binding.forest_staged_position(depth, pos) for pos in range(n_pos)]
        assert sorted(v for v in node_at if v >= 0) == list(range(n_int))
        assert node_at[0] == -1 and [node_at[p] for p in range(1, 8)] == list(range(7))
        levels = depth if depth <= 6 else 5            # levels the fields cover
        lower = levels - 3
        field = (1 << lower) - 1
        for trial in range(300):
            outcome = rng.integers(0, 2, n_int)            # by level-order ordinal; 1 = right
            h = 1
            for _ in range(depth):
                h = 2 * h + int(outcome[h - 1])
            want = h - n_pos                                # in-order leaf ordinal
            bits = sum(int(outcome[v]) << pos for pos, v in enumerate(node_at) if v >= 0)
            top = path3((bits >> 1) & 0x7f)
            start = 8 + field * top
            inner = path3((bits >> start) & ((1 << field) - 1)) >> (3 - lower)
            got = top * (1 << lower) + inner                # path through `levels` levels
            if depth > 6:                                   # the field of the level-5 subtree the path leads to
                deep = depth - 5
                width = (1 << deep) - 1
                inner = path3((bits >> (32 + width * got)) & ((1 << width) - 1)) >> (3 - deep)
                got = got * (1 << deep) + inner
            assert got == want
    for depth, pos in ((3, 0), (9, 0), (4, 16), (6, -1)):
        with pytest.raises(binding.ForestError):
            binding.forest_staged_position(depth, pos)
