"""Parallel Restarted SGD on the CPU, step by step (test infrastructure).

Algorithm 1 of the paper in the *restart* form its prose and Algorithms 2/3 use:
the iterations are cut into epochs of length I; inside an epoch every worker
runs plain SGD on its own objective (eq. 3); after every iteration t with
t mod I == 0 the node average (eq. 2 / eq. 4) overwrites every replica, so the
next gradient is taken at the common point.  Under this reading I = 1 is exactly
parallel mini-batch SGD (Section 1, first footnote) and N = 1 is plain SGD.
``run_prsgd_literal`` keeps the printed line order of Algorithm 1 instead
(gradient observed at the pre-average point, then x_i^t = ybar - gamma G_i^t);
both satisfy the mean recursion eq. (5) and the restart identity eq. (6).

No average is taken at t = 0 (replicas start equal).  When T is not a multiple
of I the run ends un-averaged; the analysed iterate xbar^T (eq. 4) is then read
with ``node_average`` without touching the replicas.

State and arithmetic are float64; inputs are the float32 bytes of the shared
input generators, widened exactly.
"""
from __future__ import annotations

from typing import Callable, Dict, Optional, Sequence

import numpy as np

from .models import loss_grad
from .philox import sample_rows

Recorder = Optional[Callable[[Dict], None]]


def node_average(x: np.ndarray) -> np.ndarray:
    """xbar = (1/N) sum_i x_i  (eq. 4), workers summed in ascending order."""
    n = x.shape[0]
    s = np.zeros(x.shape[1], dtype=np.float64)
    for i in range(n):
        s += x[i]
    return s / n


def _gradients(model, dims, activation, features, targets, x, t, batch, seed, bf16, active=None):
    """G_i^t for every worker at its current x_i (row t of the index stream)."""
    n_workers, m = x.shape
    g = np.zeros((n_workers, m), dtype=np.float64)
    losses = np.full(n_workers, np.nan)
    rows_all = np.zeros((n_workers, batch), dtype=np.int64)
    for i in range(n_workers):
        if active is not None and not active[i]:
            continue
        rows = sample_rows(seed, i, t, batch, features.shape[1])
        rows_all[i] = rows
        losses[i], g[i] = loss_grad(model, x[i], dims, activation,
                                    features[i][rows], targets[i][rows], bf16=bf16)
    return g, losses, rows_all


def _start(x0, n_workers, x_init):
    if x_init is not None:
        return np.array(x_init, dtype=np.float64, copy=True)
    return np.tile(np.asarray(x0, dtype=np.float64), (n_workers, 1))


def momentum_step(x: np.ndarray, v: np.ndarray, g: np.ndarray, lr: float, mu: float) -> None:
    """Momentum form of the local step, in place:  v <- mu v + G,  x <- x - gamma v.

    The paper's experiment (Section 4) runs its local steps with momentum 0.9 in a framework
    whose momentum SGD has exactly this form; Algorithm 1 itself is the case mu = 0."""
    v *= mu
    v += g
    x -= lr * v


def run_prsgd(model: str, dims: Sequence[int], activation: str, features: np.ndarray,
              targets: np.ndarray, x0: np.ndarray, n_workers: int, batch: int, lr: float,
              interval: int, iterations: int, seed: int, bf16: bool = False,
              t_start: int = 0, x_init: Optional[np.ndarray] = None,
              record: Recorder = None, momentum: float = 0.0, momentum_restart: str = "keep",
              v_init: Optional[np.ndarray] = None) -> Dict:
    """Algorithm 1 (restart form).  Returns {'x': [N][m], 'losses': [N], 't': int, 'v': [N][m]}.

    With ``momentum`` > 0 every worker keeps a momentum buffer v_i (zero at the start) and takes
    ``momentum_step`` instead of eq. (3).  The paper does not say what a restart does to the
    buffers; ``momentum_restart`` selects "keep" (they stay local), "average" (their node average
    overwrites them, like the points) or "reset" (zeroed)."""
    if momentum_restart not in ("keep", "average", "reset"):
        raise ValueError(momentum_restart)
    x = _start(x0, n_workers, x_init)
    v = np.zeros_like(x) if v_init is None else np.array(v_init, dtype=np.float64, copy=True)
    losses = np.full(n_workers, np.nan)
    t = t_start
    for _ in range(iterations):
        t += 1
        g, losses, rows = _gradients(model, dims, activation, features, targets, x, t, batch,
                                     seed, bf16)
        x_before = x.copy() if record else None
        if momentum != 0.0:
            momentum_step(x, v, g, lr, momentum)
        else:
            x -= lr * g                                     # eq. (3)
        averaged = (t % interval == 0)
        x_stepped = x.copy() if record else None
        if averaged:                                        # restart from the node average
            x[:] = node_average(x)
            if momentum != 0.0 and momentum_restart == "average":
                v[:] = node_average(v)
            elif momentum != 0.0 and momentum_restart == "reset":
                v[:] = 0.0
        if record:
            record({"t": t, "g": g, "rows": rows, "x_before": x_before,
                    "x_stepped": x_stepped, "x_after": x.copy(), "averaged": averaged,
                    "losses": losses.copy(), "v": v.copy()})
    return {"x": x, "losses": losses, "t": t, "v": v}


def run_prsgd_literal(model: str, dims: Sequence[int], activation: str, features: np.ndarray,
                      targets: np.ndarray, x0: np.ndarray, n_workers: int, batch: int, lr: float,
                      interval: int, iterations: int, seed: int, bf16: bool = False,
                      record: Recorder = None) -> Dict:
    """Algorithm 1 in its printed order: observe G at x^{t-1}; when t mod I == 0 set
    x_i^t = ybar - gamma G_i^t with ybar the average of the x_i^{t-1} (eq. 2)."""
    x = _start(x0, n_workers, None)
    losses = np.full(n_workers, np.nan)
    for t in range(1, iterations + 1):
        g, losses, rows = _gradients(model, dims, activation, features, targets, x, t, batch,
                                     seed, bf16)
        x_before = x.copy() if record else None
        averaged = (t % interval == 0)
        if averaged:
            x[:] = node_average(x)                          # ybar
        ybar = x.copy() if record else None
        x -= lr * g                                         # eq. (2) or eq. (3)
        if record:
            record({"t": t, "g": g, "rows": rows, "x_before": x_before, "ybar": ybar,
                    "x_after": x.copy(), "averaged": averaged})
    return {"x": x, "losses": losses, "t": iterations}


def time_varying_schedule(n_epochs: int, n_workers: int):
    """Theorem 2's choice: K^s = ceil(s^(1/3) / N), gamma^s = N / s^(2/3), s = 1..S."""
    ks, gs = [], []
    for s in range(1, n_epochs + 1):
        ks.append(int(np.ceil(s ** (1.0 / 3.0) / n_workers - 1e-12)))
        gs.append(n_workers / s ** (2.0 / 3.0))
    return ks, gs


def run_time_varying(model: str, dims: Sequence[int], activation: str, features: np.ndarray,
                     targets: np.ndarray, x0: np.ndarray, n_workers: int, batch: int,
                     epoch_lengths: Sequence[int], epoch_rates: Sequence[float], seed: int,
                     bf16: bool = False) -> Dict:
    """Algorithm 2: epoch s starts from the node average of the previous epoch's final
    points and runs K^s local steps at rate gamma^s.  Iterations are numbered
    consecutively across epochs (the paper's re-indexing remark below Algorithm 2)."""
    x = _start(x0, n_workers, None)
    losses = np.full(n_workers, np.nan)
    t = 0
    for k_s, gamma_s in zip(epoch_lengths, epoch_rates):
        x[:] = node_average(x)
        for _ in range(int(k_s)):
            t += 1
            g, losses, _ = _gradients(model, dims, activation, features, targets, x, t, batch,
                                      seed, bf16)
            x -= float(gamma_s) * g
    return {"x": x, "losses": losses, "t": t}


def run_heterogeneous(model: str, dims: Sequence[int], activation: str, features: np.ndarray,
                      targets: np.ndarray, x0: np.ndarray, n_workers: int, batch: int, lr: float,
                      worker_steps: Sequence[int], n_epochs: int, seed: int,
                      bf16: bool = False) -> Dict:
    """Algorithm 3: in every epoch worker i runs I_i local steps from the node average.
    The iteration clock advances by max_i I_i per epoch; a worker that has finished its
    I_i steps keeps its point (the paper's imagined zero-gradient steps)."""
    x = _start(x0, n_workers, None)
    losses = np.full(n_workers, np.nan)
    steps = [int(v) for v in worker_steps]
    i_max = max(steps)
    t = 0
    for _ in range(n_epochs):
        x[:] = node_average(x)
        for k in range(1, i_max + 1):
            t += 1
            active = [k <= s for s in steps]
            g, l_now, _ = _gradients(model, dims, activation, features, targets, x, t, batch,
                                     seed, bf16, active=active)
            for i in range(n_workers):
                if active[i]:
                    losses[i] = l_now[i]
            x -= lr * g                                     # g is zero for finished workers
    return {"x": x, "losses": losses, "t": t}
