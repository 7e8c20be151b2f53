"""Pins of the linear-model oracle against things other than itself: scikit-learn's own
estimators, closed forms, brute force, and the invariants the paper's redundant elimination
rests on."""
import numpy as np
import pytest

from oracle.linear_oracle import predict_linear
from workloads import OUT_BOTH, TRANSFORM_NONE, TRANSFORM_SIGMOID, TRANSFORM_SOFTMAX
from workloads.linear import LinearModel, make_linear_workload


def _model(w, b, transform, output=OUT_BOTH):
    w = np.asarray(w, np.float32)
    return LinearModel(w.shape[0], w.shape[1], w, np.asarray(b, np.float32), transform, output)


def test_brute_force_on_a_tiny_input():
    rng = np.random.default_rng(1)
    w = rng.standard_normal((5, 3)).astype(np.float32)
    b = rng.standard_normal(3).astype(np.float32)
    X = rng.standard_normal((7, 5)).astype(np.float32)
    got = predict_linear(_model(w, b, TRANSFORM_SOFTMAX), X)
    for r in range(7):
        raw = [float(b[k]) + sum(float(X[r, f]) * float(w[f, k]) for f in range(5)) for k in range(3)]
        np.testing.assert_allclose(got.raw[r], raw, rtol=1e-14, atol=1e-14)
        e = [np.exp(v - max(raw)) for v in raw]
        np.testing.assert_allclose(got.scores[r], np.float32(np.asarray(e) / sum(e)), rtol=1e-6)
        assert got.labels[r] == max(range(3), key=lambda k: (raw[k], -k))


def test_closed_forms():
    X = np.arange(24, dtype=np.float32).reshape(6, 4) - 7
    # unit weights select features; zero weights leave the bias
    eye = np.eye(4, dtype=np.float32)
    np.testing.assert_array_equal(predict_linear(_model(eye, np.zeros(4), TRANSFORM_NONE), X).scores, X)
    out = predict_linear(_model(np.zeros((4, 2)), [1.5, -2.0], TRANSFORM_NONE), X)
    np.testing.assert_array_equal(out.scores, np.tile(np.float32([1.5, -2.0]), (6, 1)))
    assert np.all(out.labels == 0)
    # ties go to the first maximum
    tie = predict_linear(_model(np.zeros((4, 3)), [2.0, 2.0, 1.0], TRANSFORM_SOFTMAX), X)
    assert np.all(tie.labels == 0)
    np.testing.assert_allclose(tie.scores.sum(axis=1), 1.0, rtol=1e-6)
    # two-class softmax is the sigmoid of the difference
    rng = np.random.default_rng(2)
    w = rng.standard_normal((4, 2)).astype(np.float32)
    two = predict_linear(_model(w, [0.25, -0.5], TRANSFORM_SOFTMAX), X)
    one = predict_linear(_model((w[:, 1:] - w[:, :1]), [-0.75], TRANSFORM_SIGMOID), X)
    np.testing.assert_allclose(two.scores[:, 1], one.scores[:, 0], rtol=2e-6, atol=1e-7)
    np.testing.assert_array_equal(two.labels, one.labels)
    # one output without transform: the 0.5 threshold of a probability-valued regressor
    reg = predict_linear(_model(np.ones((4, 1)), [0.0], TRANSFORM_NONE), np.float32([[0, 0, 0, 0.5], [0, 0, 0.25, 0.5]]))
    np.testing.assert_array_equal(reg.labels, [0, 1])


def test_label_is_unchanged_by_the_monotone_transform():
    """Redundant elimination (Section 4.3.3): argmax after softmax == argmax before it."""
    w = make_linear_workload("l3", n_rows=2000)
    X = w.make_x()
    soft = predict_linear(w.model, X)
    none = predict_linear(LinearModel(**{**w.model.__dict__, "transform": TRANSFORM_NONE}), X)
    np.testing.assert_array_equal(soft.labels, none.labels)
    np.testing.assert_array_equal(soft.labels, np.argmax(soft.scores.astype(np.float64), axis=1))


def test_against_scikit_learn_estimators():
    sk = pytest.importorskip("sklearn.linear_model")
    rng = np.random.default_rng(3)
    X = rng.standard_normal((300, 6)).astype(np.float32)
    y3 = (X[:, 0] + 0.5 * X[:, 1] > 0).astype(int) + (X[:, 2] > 0.8).astype(int)
    clf = sk.LogisticRegression(max_iter=500).fit(X, y3)
    m = _model(clf.coef_.T.astype(np.float32), clf.intercept_.astype(np.float32), TRANSFORM_SOFTMAX)
    got = predict_linear(m, X)
    ref = sk.LogisticRegression()
    ref.classes_, ref.coef_, ref.intercept_ = clf.classes_, m.weight.T.astype(np.float64), m.bias.astype(np.float64)
    np.testing.assert_allclose(got.raw, ref.decision_function(X), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(got.scores, ref.predict_proba(X), rtol=2e-6, atol=1e-7)
    np.testing.assert_array_equal(got.labels, ref.predict(X))
    # binary: one weight vector, sigmoid, label = decision > 0
    yb = (X[:, 3] - X[:, 4] > 0.1).astype(int)
    sgd = sk.SGDClassifier(loss="log_loss", random_state=0, max_iter=50, tol=None).fit(X, yb)
    mb = _model(sgd.coef_.T.astype(np.float32), sgd.intercept_.astype(np.float32), TRANSFORM_SIGMOID)
    gb = predict_linear(mb, X)
    refb = sk.SGDClassifier(loss="log_loss")
    refb.classes_, refb.coef_, refb.intercept_ = sgd.classes_, mb.weight.T.astype(np.float64), mb.bias.astype(np.float64)
    np.testing.assert_array_equal(gb.labels, refb.predict(X))
    np.testing.assert_allclose(gb.scores[:, 0], refb.predict_proba(X)[:, 1], rtol=2e-6, atol=1e-7)
    # regression
    lin = sk.LinearRegression().fit(X, X @ np.arange(6) + 2.0)
    mr = _model(lin.coef_.reshape(-1, 1).astype(np.float32), [np.float32(lin.intercept_)], TRANSFORM_NONE)
    refr = sk.LinearRegression()
    refr.coef_, refr.intercept_ = mr.weight[:, 0].astype(np.float64), float(mr.bias[0])
    np.testing.assert_allclose(predict_linear(mr, X).scores[:, 0], refr.predict(X), rtol=2e-6)


def test_workloads_are_reproducible_and_prefix_stable():
    a = make_linear_workload("l1")
    b = make_linear_workload("l1")
    np.testing.assert_array_equal(a.model.weight, b.model.weight)
    np.testing.assert_array_equal(a.make_x(700), b.make_x(1000)[:700])
    big = make_linear_workload("l3", n_rows=70000)
    np.testing.assert_array_equal(big.make_x(70000)[65530:65540], make_linear_workload("l3").make_x(65540)[65530:])
    assert a.model.weight.dtype == np.float32 and a.model.weight.shape == (20, 3)
