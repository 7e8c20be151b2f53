"""CPU oracle for the linear-model family.  TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper's linear classifiers and regressors (Section 3.3, Table 4: LogisticRegression,
SGDClassifier, RidgeClassifier, LinearRegression, LinearSVC, ...) are one matmul plus bias,
optionally followed by a monotone transform and an index operator; redundant elimination
(Section 4.3.3) takes the label from the values before the transform.  This is that definition
written out in float64 with numpy:

    raw    = X . W + b                         float64, X and W widened from float32
    scores = raw | sigmoid(raw) | softmax(raw) rounded to float32 once
    label  = first argmax_k raw[k]             (K >= 2)
             raw > 0 (sigmoid) / raw > 0.5     (K == 1; same convention as the forests)
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

TRANSFORM_NONE, TRANSFORM_SIGMOID, TRANSFORM_SOFTMAX = 0, 1, 2


@dataclass
class LinearResult:
    scores: np.ndarray   # float32 [n_rows, K]
    labels: np.ndarray   # int32 [n_rows]
    raw: np.ndarray      # float64 [n_rows, K]


def predict_linear(model, X: np.ndarray) -> LinearResult:
    X = np.asarray(X, dtype=np.float32)
    assert X.ndim == 2 and X.shape[1] == model.n_features
    w = np.asarray(model.weight, dtype=np.float64).reshape(model.n_features, model.n_outputs)
    # an absent bias is a zero bias (the description's bias pointer may be NULL)
    b = (np.zeros(model.n_outputs) if model.bias is None
         else np.asarray(model.bias, dtype=np.float64).reshape(model.n_outputs))
    with np.errstate(all="ignore"):
        raw = X.astype(np.float64) @ w + b
        if model.transform == TRANSFORM_SOFTMAX:
            z = np.exp(raw - raw.max(axis=1, keepdims=True))
            scores = z / z.sum(axis=1, keepdims=True)
        elif model.transform == TRANSFORM_SIGMOID:
            scores = 1.0 / (1.0 + np.exp(-raw))
        else:
            scores = raw
    if model.n_outputs >= 2:
        labels = np.argmax(raw, axis=1)          # first maximum
    elif model.transform == TRANSFORM_SIGMOID:
        labels = raw[:, 0] > 0.0
    else:
        labels = raw[:, 0] > 0.5
    return LinearResult(scores.astype(np.float32), labels.astype(np.int32), raw)
