"""Seeded synthetic datasets and initial points (inputs only; no method arithmetic).

Every array is produced once on the host by numpy's PCG64 generator and handed,
as the same float32 / int32 bytes, to whichever implementation consumes it.

Recipes
-------
least squares
    One shared ground truth ``w* ~ N(0, 1)^d``.  Worker ``i`` owns ``n`` rows of
    iid ``N(0, 1)`` features and targets ``y = a . w* + 0.1 N(0, 1)``.
Gaussian mixture
    ``C`` shared class means ``mu_c ~ N(0, I_d)``.  Worker ``i`` draws ``n``
    labels from its own class proportions -- uniform (iid workers) or one
    ``Dirichlet(alpha 1_C)`` draw per worker (the case where the workers'
    distributions D_i differ, Section 1 of the paper) -- and features
    ``mu_c + N(0, I_d)``.
initial point
    Least squares starts at zero.  An MLP draws ``W_l ~ N(0, s / d_{l-1})`` with
    ``s = 1`` (tanh) or ``s = 2`` (ReLU) and zero biases.  Every worker starts
    from this same point (Algorithm 1, input line).

The flat parameter vector of an MLP is ``[W_1, b_1, W_2, b_2, ...]`` with
``W_l`` stored row-major as ``[d_{l-1}][d_l]``.
"""
from __future__ import annotations

from typing import Dict, Optional, Sequence, Tuple

import numpy as np

from .configs import Workload


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(int(seed)))


def param_count(model: str, dims: Sequence[int]) -> int:
    """m: the number of scalar parameters of one replica."""
    if model == "lsq":
        return int(dims[0])
    return int(sum(dims[l] * dims[l + 1] + dims[l + 1] for l in range(len(dims) - 1)))


def make_lsq_data(n_workers: int, rows: int, d: int, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """features [N][n][d] float32, targets [N][n] float32."""
    w_star = _rng(seed).standard_normal(d, dtype=np.float32)
    feats = np.empty((n_workers, rows, d), dtype=np.float32)
    targs = np.empty((n_workers, rows), dtype=np.float32)
    for i in range(n_workers):
        g = _rng(seed + 1 + i)
        feats[i] = g.standard_normal((rows, d), dtype=np.float32)
        noise = g.standard_normal(rows, dtype=np.float32)
        targs[i] = feats[i] @ w_star + np.float32(0.1) * noise
    return feats, targs


def make_gmm_data(n_workers: int, rows: int, d: int, n_classes: int, seed: int,
                  dirichlet_alpha: Optional[float] = None) -> Tuple[np.ndarray, np.ndarray]:
    """features [N][n][d] float32, labels [N][n] int32."""
    means = _rng(seed).standard_normal((n_classes, d), dtype=np.float32)
    feats = np.empty((n_workers, rows, d), dtype=np.float32)
    labels = np.empty((n_workers, rows), dtype=np.int32)
    for i in range(n_workers):
        g = _rng(seed + 1 + i)
        if dirichlet_alpha is None:
            p = np.full(n_classes, 1.0 / n_classes)
        else:
            p = g.dirichlet(np.full(n_classes, float(dirichlet_alpha)))
        c = g.choice(n_classes, size=rows, p=p).astype(np.int32)
        labels[i] = c
        x = g.standard_normal((rows, d), dtype=np.float32)
        x += means[c]
        feats[i] = x
    return feats, labels


def make_x0(model: str, dims: Sequence[int], activation: str, seed: int) -> np.ndarray:
    """The common initial point, flat float32 [m]."""
    if model == "lsq":
        return np.zeros(int(dims[0]), dtype=np.float32)
    g = _rng(seed)
    scale = 2.0 if activation == "relu" else 1.0
    parts = []
    for l in range(len(dims) - 1):
        d_in, d_out = int(dims[l]), int(dims[l + 1])
        w = g.standard_normal((d_in, d_out), dtype=np.float32)
        w *= np.float32(np.sqrt(scale / d_in))
        parts.append(w.ravel())
        parts.append(np.zeros(d_out, dtype=np.float32))
    return np.concatenate(parts)


def make_inputs(w: Workload) -> Dict[str, np.ndarray]:
    """All host inputs of one workload: features, targets (float32 or int32 labels), x0."""
    if w.model == "lsq":
        feats, targs = make_lsq_data(w.n_workers, w.rows_per_worker, w.dims[0], w.data_seed)
    else:
        feats, targs = make_gmm_data(w.n_workers, w.rows_per_worker, w.dims[0], w.n_classes,
                                     w.data_seed, w.dirichlet_alpha)
    x0 = make_x0(w.model, w.dims, w.activation, w.x0_seed)
    return {"features": feats, "targets": targs, "x0": x0}
