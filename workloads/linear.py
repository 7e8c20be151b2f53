"""Seeded synthetic linear models and feature matrices (generators only, no arithmetic of the
method): stand-ins for the linear models of the paper's evaluation (LogisticRegression,
SGDClassifier, LinearRegression, ... of Table 5 on YearPrediction, 515 345 x 90), whose trained
weights the paper does not give.

    l1  1 000 x 20,  3 classes, softmax + label      small case the oracle finishes at once
    l2  4 000 000 x 90, 1 output, no transform       regression at the paper's feature count
    l3  2 000 000 x 128, 10 classes, softmax + label multinomial logistic regression
    l4  8 000 000 x 28, 1 output, sigmoid + label    binary logistic regression

Weights ~ N(0, 1/sqrt(F)), bias ~ N(0, 0.1), X ~ N(0, 1) in chunks of 65 536 rows so that every
row prefix is reproducible from the seed.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Iterator, Optional

import numpy as np

from . import OUT_BOTH, OUT_SCORES, TRANSFORM_NONE, TRANSFORM_SIGMOID, TRANSFORM_SOFTMAX, X_CHUNK_ROWS

LINEAR_SEEDS = {"l1": 13441101, "l2": 13441102, "l3": 13441103, "l4": 13441104}
LINEAR_ROWS = {"l1": 1_000, "l2": 4_000_000, "l3": 2_000_000, "l4": 8_000_000}
_SHAPES = {  # n_features, n_outputs, transform, output
    "l1": (20, 3, TRANSFORM_SOFTMAX, OUT_BOTH),
    "l2": (90, 1, TRANSFORM_NONE, OUT_SCORES),
    "l3": (128, 10, TRANSFORM_SOFTMAX, OUT_BOTH),
    "l4": (28, 1, TRANSFORM_SIGMOID, OUT_BOTH),
}


@dataclass
class LinearModel:
    n_features: int
    n_outputs: int
    weight: np.ndarray      # float32 [n_features, n_outputs]
    bias: np.ndarray        # float32 [n_outputs]
    transform: int = TRANSFORM_NONE
    output: int = OUT_SCORES


@dataclass
class LinearWorkload:
    name: str
    model: LinearModel
    n_rows: int
    seed: int

    def x_chunks(self, n_rows: Optional[int] = None) -> Iterator[np.ndarray]:
        n = self.n_rows if n_rows is None else n_rows
        done = 0
        chunk = 0
        while done < n:
            rng = np.random.default_rng([self.seed, 7, chunk])
            block = rng.standard_normal((X_CHUNK_ROWS, self.model.n_features), dtype=np.float32)
            take = min(X_CHUNK_ROWS, n - done)
            yield block[:take]
            done += take
            chunk += 1

    def make_x(self, n_rows: Optional[int] = None) -> np.ndarray:
        return np.concatenate(list(self.x_chunks(n_rows)), axis=0)


def make_linear_workload(name: str, n_rows: Optional[int] = None) -> LinearWorkload:
    n_features, n_outputs, transform, output = _SHAPES[name]
    seed = LINEAR_SEEDS[name]
    rng = np.random.default_rng(seed)
    weight = (rng.standard_normal((n_features, n_outputs)) / np.sqrt(n_features)).astype(np.float32)
    bias = (rng.standard_normal(n_outputs) * 0.1).astype(np.float32)
    model = LinearModel(n_features, n_outputs, weight, bias, transform, output)
    return LinearWorkload(name, model, LINEAR_ROWS[name] if n_rows is None else n_rows, seed)
