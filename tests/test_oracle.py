"""Pins for the CPU oracle: everything here is checked against something other than the
oracle itself -- a hand-derived worked example, scikit-learn's own predictors, closed forms,
the dense matrix formulation of Table 2, and invariants of that formulation."""
import json
import os

import numpy as np
import pytest

import oracle
from oracle import matrix_form as mf
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "depth2_worked_example.json")


def _one_tree_forest(tree, n_features, **kw):
    n = len(tree["feature"])
    return wl.Forest(
        n_features=n_features, n_outputs=1, leaf_width=1,
        tree_offset=np.asarray([0, n], dtype=np.int64),
        feature=np.asarray(tree["feature"], dtype=np.int32),
        threshold=np.asarray(tree["threshold"], dtype=np.float32),
        left=np.asarray(tree["left"], dtype=np.int32),
        right=np.asarray(tree["right"], dtype=np.int32),
        leaf_value=np.asarray(tree["leaf_value"], dtype=np.float32).reshape(n, 1),
        tree_output=np.zeros(1, dtype=np.int32), **kw)


def _concat(forests, **kw):
    off, parts = [0], {k: [] for k in ("feature", "threshold", "left", "right", "leaf_value")}
    for f in forests:
        off.append(off[-1] + f.n_nodes)
        for k in parts:
            parts[k].append(getattr(f, k))
    base = forests[0]
    T = len(forests)
    args = dict(n_features=base.n_features, n_outputs=base.n_outputs, leaf_width=base.leaf_width,
                tree_offset=np.asarray(off, dtype=np.int64),
                tree_output=np.zeros(T, dtype=np.int32))
    args.update({k: np.concatenate(v) for k, v in parts.items()})
    args.update(kw)
    return wl.Forest(**args)


# ----------------------------------------------------------------------------- worked example

def test_worked_example_traversal_and_matrices():
    g = json.load(open(GOLDEN))
    forest = _one_tree_forest(g["tree"], g["n_features"])
    X = np.asarray([r["x"] for r in g["rows"]], dtype=np.float32)
    res = oracle.predict(forest, X, want_leaves=True)
    assert res.leaf_node_id[:, 0].tolist() == [r["leaf_node"] for r in g["rows"]]
    assert res.scores[:, 0].tolist() == [r["value"] for r in g["rows"]]

    t = g["tree"]
    m = mf.tree_matrices(g["n_features"], np.asarray(t["feature"]), np.asarray(t["threshold"], np.float32),
                         np.asarray(t["left"]), np.asarray(t["right"]),
                         np.asarray(t["leaf_value"], np.float32))
    assert m.W1.tolist() == g["W1"]
    assert m.W2.tolist() == g["W2"]
    assert m.W3.tolist() == g["W3"]
    assert m.C.tolist() == g["C"]
    assert m.D.tolist() == g["D"]
    assert m.E[:, 0].tolist() == g["E"]
    # intermediate tensors of the operator graph, row by row
    G = X.astype(np.float64) @ m.W1
    S = (G.astype(np.float32) > m.W2).astype(int)
    assert S.tolist() == [r["S"] for r in g["rows"]]
    assert (S @ m.W3.astype(int)).tolist() == [r["P"] for r in g["rows"]]
    assert ((1 - S) @ m.C.astype(int)).tolist() == [r["TC"] for r in g["rows"]]
    assert mf.paper_form_leaf(X, m).tolist() == [r["leaf"] for r in g["rows"]]
    onehot = mf.path_form_onehot(X, m)
    assert onehot.sum(axis=1).tolist() == [1, 1, 1, 1]
    assert onehot.argmax(axis=1).tolist() == [r["leaf"] for r in g["rows"]]


def test_worked_example_two_tree_mean_and_half_tie():
    g = json.load(open(GOLDEN))
    f = _concat([_one_tree_forest(g["tree"], 3), _one_tree_forest(g["stump"], 3)],
                aggregate=wl.AGG_MEAN)
    X = np.asarray([r["x"] for r in g["rows"]], dtype=np.float32)
    res = oracle.predict(f, X)
    assert res.scores[:, 0].tolist() == g["forest_mean"]
    assert res.labels.tolist() == g["forest_label"]


# ----------------------------------------------------------------------------- conventions

def _stump(thr, lo=1.0, hi=2.0):
    return _one_tree_forest(dict(feature=[0, -1, -1], threshold=[thr, 0, 0], left=[1, -1, -1],
                                 right=[2, -1, -1], leaf_value=[0, lo, hi]), 1)


def test_stump_is_a_step_function_with_closed_boundary():
    f = _stump(0.25)
    X = np.asarray([[-1.0], [0.25], [np.nextafter(np.float32(0.25), np.float32(1))], [3.0]], np.float32)
    assert oracle.predict(f, X).scores[:, 0].tolist() == [1.0, 1.0, 2.0, 2.0]


def test_nan_goes_right_and_signed_zero_and_infinities():
    X = np.asarray([[np.nan], [-0.0], [0.0], [np.inf], [-np.inf]], np.float32)
    assert oracle.predict(_stump(0.0), X).scores[:, 0].tolist() == [2.0, 1.0, 1.0, 2.0, 1.0]
    assert oracle.predict(_stump(-0.0), X).scores[:, 0].tolist() == [2.0, 1.0, 1.0, 2.0, 1.0]
    # +Inf threshold: everything but NaN goes left; -Inf threshold: only -Inf goes left
    assert oracle.predict(_stump(np.inf), X).scores[:, 0].tolist() == [2.0, 1.0, 1.0, 1.0, 1.0]
    assert oracle.predict(_stump(-np.inf), X).scores[:, 0].tolist() == [2.0, 2.0, 2.0, 2.0, 1.0]


def test_infinite_thresholds_reach_outermost_leaves():
    w = wl.make_workload("c1", n_rows=64)
    f = w.forest
    X = w.make_x(64)
    internal = f.feature >= 0
    for thr, pick in ((np.inf, "first"), (-np.inf, "last")):
        g = wl.Forest(**{**f.__dict__, "threshold": np.where(internal, np.float32(thr), f.threshold)})
        res = oracle.predict(g, X, want_leaves=True)
        # full depth-4 tree stored breadth-first: leaves are nodes 15..30
        want = 15 if pick == "first" else 30
        assert (res.leaf_node_id == want).all()


# ----------------------------------------------------------------------------- scikit-learn

def _sk_forest(estimators, n_features, K, leaf_width, scale=1.0, value_of=None, **kw):
    off, feat, thr, left, right, val = [0], [], [], [], [], []
    for est in estimators:
        tr = est.tree_
        n = tr.node_count
        off.append(off[-1] + n)
        is_leaf = tr.children_left < 0
        feat.append(np.where(is_leaf, -1, tr.feature).astype(np.int32))
        thr.append(np.where(is_leaf, 0, tr.threshold).astype(np.float32))
        left.append(tr.children_left.astype(np.int32))
        right.append(tr.children_right.astype(np.int32))
        v = tr.value.reshape(n, -1)[:, :leaf_width] if value_of is None else value_of(tr)
        val.append((v * scale).astype(np.float32))
    T = len(estimators)
    return wl.Forest(n_features=n_features, n_outputs=K, leaf_width=leaf_width,
                     tree_offset=np.asarray(off, np.int64), feature=np.concatenate(feat),
                     threshold=np.concatenate(thr), left=np.concatenate(left),
                     right=np.concatenate(right), leaf_value=np.concatenate(val),
                     tree_output=np.zeros(T, np.int32), **kw)


def _grid_data(seed, n, F):
    rng = np.random.default_rng(seed)
    # integer-valued features: every learned threshold is k + 0.5, exact in float32
    return rng.integers(0, 12, size=(n, F)).astype(np.float32), rng


def test_against_sklearn_decision_tree_and_apply():
    sk = pytest.importorskip("sklearn.tree")
    X, rng = _grid_data(1, 600, 5)
    y = X[:, 0] * 2 - X[:, 3] + rng.standard_normal(600)
    est = sk.DecisionTreeRegressor(max_depth=7, random_state=0).fit(X, y)
    f = _sk_forest([est], 5, 1, 1)
    Xt, _ = _grid_data(2, 500, 5)
    res = oracle.predict(f, Xt, want_leaves=True)
    assert (res.leaf_node_id[:, 0] == est.apply(Xt)).all()
    np.testing.assert_allclose(res.scores[:, 0], est.predict(Xt), rtol=1e-6, atol=1e-6)


def test_against_sklearn_random_forest_classifier_proba():
    ske = pytest.importorskip("sklearn.ensemble")
    X, rng = _grid_data(3, 800, 6)
    y = ((X[:, 1] + X[:, 2] > 11).astype(int) + (X[:, 4] > 8).astype(int))
    rf = ske.RandomForestClassifier(n_estimators=12, max_depth=6, random_state=0).fit(X, y)
    K = len(rf.classes_)
    f = _sk_forest(rf.estimators_, 6, K, K, aggregate=wl.AGG_MEAN)
    Xt, _ = _grid_data(4, 400, 6)
    res = oracle.predict(f, Xt, want_leaves=True)
    np.testing.assert_allclose(res.scores, rf.predict_proba(Xt), rtol=1e-6, atol=1e-6)
    assert (res.leaf_node_id == rf.apply(Xt)).all()
    proba = rf.predict_proba(Xt)
    srt = np.sort(proba, axis=1)
    clear = (srt[:, -1] - srt[:, -2]) > 1e-6
    assert (res.labels[clear] == np.argmax(proba, axis=1)[clear]).all()


def test_against_sklearn_gradient_boosting_regressor():
    ske = pytest.importorskip("sklearn.ensemble")
    X, rng = _grid_data(5, 700, 4)
    y = np.sin(X[:, 0]) * 3 + X[:, 1] * 0.2 + 0.1 * rng.standard_normal(700)
    gb = ske.GradientBoostingRegressor(n_estimators=30, max_depth=3, learning_rate=0.1,
                                       random_state=0).fit(X, y)
    f = _sk_forest([e[0] for e in gb.estimators_], 4, 1, 1, scale=gb.learning_rate,
                   aggregate=wl.AGG_SUM,
                   base_score=np.asarray([gb.init_.constant_[0, 0]], np.float32))
    Xt, _ = _grid_data(6, 300, 4)
    np.testing.assert_allclose(oracle.predict(f, Xt).scores[:, 0], gb.predict(Xt), rtol=2e-6, atol=2e-6)


def test_against_sklearn_gradient_boosting_classifier_binary():
    """Per-class sums + sigmoid + label of a boosted binary classifier: probability of class 1
    is sigmoid(raw), raw = log-odds of the prior + learning rate x sum of the trees' leaf values."""
    ske = pytest.importorskip("sklearn.ensemble")
    X, rng = _grid_data(11, 900, 5)
    y = ((X[:, 0] + X[:, 3] > 11) ^ (X[:, 1] > 9)).astype(int)
    gb = ske.GradientBoostingClassifier(n_estimators=25, max_depth=3, learning_rate=0.2,
                                        random_state=0).fit(X, y)
    prior = gb.init_.class_prior_
    f = _sk_forest([e[0] for e in gb.estimators_], 5, 1, 1, scale=gb.learning_rate, aggregate=wl.AGG_SUM,
                   base_score=np.asarray([np.log(prior[1] / prior[0])], np.float32),
                   transform=wl.TRANSFORM_SIGMOID)
    Xt, _ = _grid_data(12, 500, 5)
    res = oracle.predict(f, Xt)
    proba = gb.predict_proba(Xt)[:, 1]
    np.testing.assert_allclose(res.scores[:, 0], proba, rtol=2e-6, atol=2e-6)
    np.testing.assert_allclose(res.raw[:, 0], gb.decision_function(Xt), rtol=2e-6, atol=2e-6)
    clear = np.abs(proba - 0.5) > 1e-6
    assert clear.sum() > 400
    assert (res.labels[clear] == gb.predict(Xt)[clear]).all()


def test_against_sklearn_gradient_boosting_classifier_multiclass():
    """Three classes: one scalar-leaf tree per class and round feeding its class's column, base
    score = log prior, softmax over the per-class sums, label = argmax of the raw sums."""
    ske = pytest.importorskip("sklearn.ensemble")
    X, rng = _grid_data(13, 900, 5)
    y = (X[:, 0] + X[:, 1] > 11).astype(int) + (X[:, 2] > 8).astype(int)
    gb = ske.GradientBoostingClassifier(n_estimators=12, max_depth=3, learning_rate=0.3,
                                        random_state=0).fit(X, y)
    n_rounds, K = gb.estimators_.shape
    assert K == 3
    ests = [gb.estimators_[i, k] for i in range(n_rounds) for k in range(K)]   # round-major
    f = _sk_forest(ests, 5, K, 1, scale=gb.learning_rate, aggregate=wl.AGG_SUM,
                   base_score=np.log(gb.init_.class_prior_).astype(np.float32),
                   transform=wl.TRANSFORM_SOFTMAX)
    f.tree_output = np.asarray([k for _ in range(n_rounds) for k in range(K)], np.int32)
    Xt, _ = _grid_data(14, 500, 5)
    res = oracle.predict(f, Xt)
    proba = gb.predict_proba(Xt)
    np.testing.assert_allclose(res.scores, proba, rtol=5e-6, atol=2e-6)
    srt = np.sort(proba, axis=1)
    clear = (srt[:, -1] - srt[:, -2]) > 1e-5
    assert clear.sum() > 400
    assert (res.labels[clear] == gb.predict(Xt)[clear]).all()


# ----------------------------------------------------------------------------- matrix formulation

@pytest.mark.parametrize("seed", range(8))
def test_matrix_forms_agree_with_traversal_on_tiny_forests(seed):
    f = wl.random_forest(100 + seed, n_trees=6, n_features=4, max_depth=5, stop_prob=0.3,
                         grid_thresholds=True)
    rng = np.random.default_rng(seed)
    # rows on the threshold grid: x == threshold happens all the time
    X = (rng.integers(-3, 4, size=(300, 4)).astype(np.float32) * np.float32(0.5))
    res = oracle.predict(f, X, want_leaves=True)
    for t, (ft, thr, l, r, v) in enumerate(mf.split_trees(f)):
        m = mf.tree_matrices(4, ft, thr, l, r, v)
        # Table 2 structure: one selected feature per internal node; W3 row i has exactly
        # |leaves(Left(I_i))| zeros; sparsity (non-zero ratio) within [1/2, 1 - 1/N_L]
        n_i, n_l = m.W3.shape
        assert n_l == n_i + 1
        if n_i:
            assert (m.W1.sum(axis=0) == 1).all()
            nz = m.W3.mean()
            assert 0.5 - 1e-12 <= nz <= 1 - 1 / n_l + 1e-12
            assert ((m.C == 1).sum(axis=0) == m.D).all()
            # in-order numbering makes Left(i) a contiguous leaf range directly left of Right(i)
            for i in range(n_i):
                lf = np.flatnonzero(m.C[i] == 1)
                rt = np.flatnonzero(m.C[i] == -1)
                assert (np.diff(lf) == 1).all() and (np.diff(rt) == 1).all()
                assert lf[-1] + 1 == rt[0]
        onehot = mf.path_form_onehot(X, m)
        assert (onehot.sum(axis=1) == 1).all()            # exactly one leaf per (row, tree)
        leaf_path = onehot.argmax(axis=1)
        leaf_paper = mf.paper_form_leaf(X, m)
        assert (leaf_path == leaf_paper).all()
        assert (np.asarray(m.leaf_nodes)[leaf_paper] == res.leaf_node_id[:, t]).all()
    np.testing.assert_array_equal(mf.forest_raw_scores(f, X, "path"), res.raw)
    np.testing.assert_array_equal(mf.forest_raw_scores(f, X, "paper"), res.raw)


def test_matrix_form_exhaustive_outcomes_depth3():
    # every one of the 2^3 leaf paths of a full depth-3 tree with distinct features per level
    is_leaf, left, right = wl.full_tree_arrays(3)
    feature = np.where(is_leaf, -1, np.asarray([0, 1, 1, 2, 2, 2, 2] + [0] * 8)).astype(np.int32)
    thr = np.zeros(15, np.float32)
    val = np.arange(15, dtype=np.float32)
    m = mf.tree_matrices(3, feature, thr, left, right, val)
    X = np.asarray([[a, b, c] for a in (-1, 1) for b in (-1, 1) for c in (-1, 1)], np.float32)
    assert mf.paper_form_leaf(X, m).tolist() == list(range(8))
    assert mf.path_form_onehot(X, m).argmax(axis=1).tolist() == list(range(8))


def test_multiclass_and_vector_leaf_matrix_agreement():
    f = wl.random_forest(7, n_trees=9, n_features=5, max_depth=4, n_outputs=3, leaf_width=1,
                         transform=wl.TRANSFORM_SOFTMAX)
    g = wl.random_forest(8, n_trees=5, n_features=5, max_depth=4, n_outputs=3, leaf_width=3,
                         aggregate=wl.AGG_MEAN)
    X = np.random.default_rng(0).standard_normal((200, 5)).astype(np.float32)
    for forest in (f, g):
        res = oracle.predict(forest, X)
        np.testing.assert_allclose(mf.forest_raw_scores(forest, X), res.raw, rtol=0, atol=1e-15)


# ----------------------------------------------------------------------------- reduction / transforms

def test_constant_leaves_closed_form():
    w = wl.make_workload("c1", n_rows=32)
    X = w.make_x(32)
    f = w.forest
    c = np.float32(0.375)
    const = np.where((f.feature < 0)[:, None], c, f.leaf_value).astype(np.float32)
    mean = wl.Forest(**{**f.__dict__, "leaf_value": const})
    assert (oracle.predict(mean, X).scores == c).all()
    summed = wl.Forest(**{**f.__dict__, "leaf_value": const, "aggregate": wl.AGG_SUM,
                          "base_score": np.asarray([0.5], np.float32)})
    assert (oracle.predict(summed, X).scores == np.float32(0.5 + 10 * 0.375)).all()


def _constant_leaf_trees(columns, c, K, **kw):
    """Single-split trees (x0 <= 0) whose two leaves both hold c; tree t feeds columns[t]."""
    T = len(columns)
    return wl.Forest(n_features=1, n_outputs=K, leaf_width=1,
                     tree_offset=np.arange(0, 3 * T + 1, 3, dtype=np.int64),
                     feature=np.tile(np.asarray([0, -1, -1], np.int32), T),
                     threshold=np.zeros(3 * T, np.float32),
                     left=np.tile(np.asarray([1, -1, -1], np.int32), T),
                     right=np.tile(np.asarray([2, -1, -1], np.int32), T),
                     leaf_value=np.tile(np.asarray([[0.0], [c], [c]], np.float32), (T, 1)),
                     tree_output=np.asarray(columns, np.int32), **kw)


def test_mean_divides_by_the_trees_that_feed_a_column():
    """Closed form: eleven scalar-leaf trees with constant leaves c feed three of four columns
    unevenly (3 / 4 / 4 trees).  MEAN gives base + c in every fed column -- dividing by all eleven
    trees would give 3c/11 and 4c/11 -- and a column no tree feeds is its base score: the mean
    over no trees adds nothing."""
    c = 0.375
    columns = [0, 1, 2, 1, 2, 0, 1, 2, 2, 1, 0]
    base = np.asarray([0.25, -1.0, 2.0, 0.5], np.float32)
    X = np.asarray([[-1.0], [0.0], [3.0], [np.nan]], np.float32)
    f = _constant_leaf_trees(columns, c, 4, aggregate=wl.AGG_MEAN, base_score=base)
    res = oracle.predict(f, X)
    want = np.asarray([0.25 + c, -1.0 + c, 2.0 + c, 0.5], np.float32)
    assert (res.scores == want[None, :]).all()
    assert res.labels.tolist() == [2, 2, 2, 2]
    # SUM of the same forest: base + (trees feeding the column) * c
    g = _constant_leaf_trees(columns, c, 4, aggregate=wl.AGG_SUM, base_score=base)
    want_sum = np.asarray([0.25 + 3 * c, -1.0 + 4 * c, 2.0 + 4 * c, 0.5], np.float32)
    assert (oracle.predict(g, X).scores == want_sum[None, :]).all()
    # without base scores the unfed column is exactly 0, never 0/0
    h = _constant_leaf_trees(columns, c, 4, aggregate=wl.AGG_MEAN)
    assert (oracle.predict(h, X).scores == np.asarray([c, c, c, 0.0], np.float32)[None, :]).all()


def test_single_output_labels_follow_the_transformed_score():
    """K = 1: the label is taken before the monotone transform (Section 4.3.3) and must agree with
    thresholding the transformed score at one half wherever the score is not within rounding of
    it: sigmoid(raw) > 0.5 iff raw > 0; without transform, raw > 0.5."""
    X = np.random.default_rng(5).standard_normal((4000, 6)).astype(np.float32)
    g = wl.random_forest(34, n_trees=9, n_features=6, max_depth=4, transform=wl.TRANSFORM_SIGMOID)
    centre = np.float32(-np.median(oracle.predict(g, X).raw))      # both classes occur
    g = wl.Forest(**{**g.__dict__, "base_score": np.asarray([centre], np.float32)})
    rs = oracle.predict(g, X)
    off = np.abs(rs.scores[:, 0].astype(np.float64) - 0.5) > 1e-6
    assert off.sum() > 3900 and 0.2 < rs.labels.mean() < 0.8
    assert (rs.labels[off] == (rs.scores[off, 0] > 0.5)).all()
    # a raw value of exactly zero is class 0 under sigmoid, and exactly one half is class 0 without
    for transform, value in ((wl.TRANSFORM_SIGMOID, 0.0), (wl.TRANSFORM_NONE, 0.5)):
        z = _constant_leaf_trees([0], value, 1, transform=transform)
        assert oracle.predict(z, X[:4, :1]).labels.tolist() == [0, 0, 0, 0]
        nxt = float(np.nextafter(np.float32(value), np.float32(1)))
        z = _constant_leaf_trees([0], nxt, 1, transform=transform)
        assert oracle.predict(z, X[:4, :1]).labels.tolist() == [1, 1, 1, 1]


def test_tree_order_and_forest_doubling():
    f = wl.random_forest(21, n_trees=7, n_features=4, max_depth=4, aggregate=wl.AGG_MEAN)
    # dyadic leaf values: fp64 sums are exact, so any tree order gives identical bits
    f.leaf_value = (np.round(f.leaf_value * 64) / 64).astype(np.float32)
    X = np.random.default_rng(1).standard_normal((128, 4)).astype(np.float32)
    base = oracle.predict(f, X).raw
    trees = [wl.Forest(n_features=4, n_outputs=1, leaf_width=1,
                       tree_offset=np.asarray([0, b - a], np.int64), feature=f.feature[a:b],
                       threshold=f.threshold[a:b], left=f.left[a:b], right=f.right[a:b],
                       leaf_value=f.leaf_value[a:b], tree_output=np.zeros(1, np.int32))
             for a, b in zip(f.tree_offset[:-1], f.tree_offset[1:])]
    perm = [3, 0, 6, 2, 5, 1, 4]
    shuffled = _concat([trees[i] for i in perm], aggregate=wl.AGG_MEAN)
    np.testing.assert_array_equal(oracle.predict(shuffled, X).raw, base)
    doubled = _concat(trees + trees, aggregate=wl.AGG_MEAN)
    np.testing.assert_array_equal(oracle.predict(doubled, X).raw, base)


def test_softmax_sigmoid_and_labels():
    f = wl.random_forest(33, n_trees=12, n_features=6, max_depth=4, n_outputs=4,
                         transform=wl.TRANSFORM_SOFTMAX)
    X = np.random.default_rng(2).standard_normal((256, 6)).astype(np.float32)
    res = oracle.predict(f, X)
    np.testing.assert_allclose(res.scores.sum(axis=1), 1.0, atol=1e-6)
    # softmax from its textbook definition on the raw values
    e = np.exp(res.raw - res.raw.max(axis=1, keepdims=True))
    np.testing.assert_allclose(res.scores, e / e.sum(axis=1, keepdims=True), rtol=1e-6)
    # monotone transform in front of argmax changes nothing (Section 4.3.3)
    assert (res.labels == np.argmax(res.raw, axis=1)).all()
    none = wl.Forest(**{**f.__dict__, "transform": wl.TRANSFORM_NONE})
    assert (oracle.predict(none, X).labels == res.labels).all()
    # sigmoid, K = 1
    g = wl.random_forest(34, n_trees=5, n_features=6, max_depth=3, transform=wl.TRANSFORM_SIGMOID)
    rs = oracle.predict(g, X)
    np.testing.assert_allclose(rs.scores[:, 0], 1 / (1 + np.exp(-rs.raw[:, 0])), rtol=1e-6)
    assert (rs.labels == (rs.raw[:, 0] > 0)).all()


def test_first_index_wins_exact_class_ties():
    # three single-leaf trees feeding columns 0,1,2 with values 1, 2, 2 -> label 1, not 2
    T = 3
    f = wl.Forest(n_features=1, n_outputs=3, leaf_width=1,
                  tree_offset=np.arange(T + 1, dtype=np.int64), feature=np.full(T, -1, np.int32),
                  threshold=np.zeros(T, np.float32), left=np.full(T, -1, np.int32),
                  right=np.full(T, -1, np.int32),
                  leaf_value=np.asarray([[1.0], [2.0], [2.0]], np.float32),
                  tree_output=np.asarray([0, 1, 2], np.int32), transform=wl.TRANSFORM_SOFTMAX)
    res = oracle.predict(f, np.zeros((4, 1), np.float32), want_leaves=True)
    assert res.labels.tolist() == [1, 1, 1, 1]
    assert (res.leaf_node_id == 0).all()       # a root that is a leaf is a legal tree


def test_thread_count_does_not_change_results():
    w = wl.make_workload("c4", n_rows=777, n_trees=40)
    X = w.make_x(777)
    a = oracle.predict(w.forest, X, want_leaves=True, n_threads=1)
    b = oracle.predict(w.forest, X, want_leaves=True, n_threads=5)
    np.testing.assert_array_equal(a.scores, b.scores)
    np.testing.assert_array_equal(a.leaf_node_id, b.leaf_node_id)
    np.testing.assert_array_equal(a.labels, b.labels)
