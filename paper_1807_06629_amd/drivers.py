"""Host loops of the paper's algorithms on top of the C-ABI calls (no arithmetic here)."""
from __future__ import annotations

from typing import Dict, Sequence

import numpy as np
import torch

from . import prsgd


def open_workload(w, inputs: Dict[str, np.ndarray], device="cuda:0", fused_update: bool = True,
                  stream=None) -> prsgd.Handle:
    """Uploads one workload's inputs and creates a context for it.

    `w` is a hyper-parameter record with the fields of workloads.Workload."""
    cfg = prsgd.make_config(w.n_workers, w.model, w.dims, w.batch, w.rows_per_worker, w.lr,
                            w.index_seed, activation=w.activation, gemm_dtype=w.gemm_dtype,
                            fused_update=fused_update, momentum=getattr(w, "momentum", 0.0),
                            momentum_restart=getattr(w, "momentum_restart", "keep"))
    feats = torch.from_numpy(inputs["features"]).to(device)
    targs = torch.from_numpy(inputs["targets"]).to(device)
    return prsgd.prsgd_init(cfg, inputs["x0"], feats, targs, stream=stream)


def run_algorithm1(h: prsgd.Handle, iterations: int, interval: int) -> None:
    """Algorithm 1: local steps with a restart average after every I-th iteration."""
    prsgd.prsgd_run(h, iterations, interval)


def time_varying_schedule(n_epochs: int, n_workers: int):
    """Theorem 2's epoch lengths K^s and rates gamma^s, s = 1..S, as the library computes them."""
    ks, gs = prsgd.prsgd_time_varying_schedule(n_epochs, n_workers)
    return [int(k) for k in ks], [float(g) for g in gs]


def run_algorithm2(h: prsgd.Handle, epoch_lengths: Sequence[int], epoch_rates: Sequence[float]) -> None:
    """Algorithm 2: every epoch restarts from the node average, then takes K^s local steps
    at rate gamma^s."""
    for k_s, gamma_s in zip(epoch_lengths, epoch_rates):
        prsgd.prsgd_average(h)
        prsgd.prsgd_set_lr(h, float(gamma_s))
        prsgd.prsgd_local_steps(h, int(k_s))


def run_algorithm3(h: prsgd.Handle, worker_steps: Sequence[int], n_epochs: int) -> None:
    """Algorithm 3: every epoch restarts from the node average, then worker i takes I_i steps."""
    for _ in range(n_epochs):
        prsgd.prsgd_average(h)
        prsgd.prsgd_local_steps_hetero(h, worker_steps)


def read_all(h: prsgd.Handle) -> np.ndarray:
    """Every replica as a [N][m] array."""
    return np.stack([prsgd.prsgd_read_params(h, i) for i in range(h.cfg.n_workers)])
