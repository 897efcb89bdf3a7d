"""Named workload configurations (hyper-parameter records only).

Each record fixes the inputs of the paper's Algorithm 1 (N, gamma, I, T) plus the
synthetic objective F_i that stands in for the paper's abstract stochastic
objective (Section 1, eq. 1): a least-squares problem or an MLP classifier on a
Gaussian mixture.  The paper measured ResNet20 on CIFAR10; the 784- and
3072-dimensional mixtures only borrow MNIST-like and CIFAR-like *shapes*.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple


@dataclass(frozen=True)
class Workload:
    name: str
    model: str                      # "lsq" | "mlp"
    n_workers: int                  # N
    dims: Tuple[int, ...]           # lsq: (d,) ; mlp: (d0, ..., dL)
    activation: str                 # "tanh" | "relu" | "none"
    gemm_dtype: str                 # "f32" | "bf16"
    batch: int                      # B rows per worker per iteration
    rows_per_worker: int            # n (power of two)
    lr: float                       # gamma
    interval: int                   # I
    iterations: int                 # T
    n_classes: int = 0
    dirichlet_alpha: Optional[float] = None   # None -> iid uniform classes
    interval_sweep: Tuple[int, ...] = ()
    data_seed: int = 1
    x0_seed: int = 2
    index_seed: int = 3
    momentum: float = 0.0           # mu of the local momentum-SGD step (0: eq. 3 as printed)
    momentum_restart: str = "keep"  # momentum buffers at a restart: "keep" | "average" | "reset"

    def scaled(self, **kw) -> "Workload":
        """A copy with some fields replaced (used for reduced-size test cases)."""
        return replace(self, **kw)


WORKLOADS = {
    # Least squares, N=4, m=64.
    "c1": Workload("c1", "lsq", 4, (64,), "none", "f32", 16, 4096, 0.01, 8, 256),
    # Non-convex tanh MLP, iid data.
    "c2": Workload("c2", "mlp", 8, (784, 256, 10), "tanh", "f32", 32, 8192, 0.05, 16, 2000,
                   n_classes=10),
    # Non-iid (Dirichlet 0.3 class proportions per worker), bf16 GEMM operands.
    "c3": Workload("c3", "mlp", 16, (3072, 1024, 1024, 10), "relu", "bf16", 64, 8192, 0.05, 32,
                   5000, n_classes=10, dirichlet_alpha=0.3),
    # Many small replicas: the averaging-dominated regime.
    "c4": Workload("c4", "mlp", 64, (256, 128, 10), "relu", "f32", 8, 8192, 0.02, 8, 10000,
                   n_classes=10, interval_sweep=(1, 2, 4, 8)),
    # Large replicas, bf16 GEMM operands.
    "c5": Workload("c5", "mlp", 8, (4096, 4096, 4096, 4096, 1000), "relu", "bf16", 128, 8192,
                   0.01, 16, 500, n_classes=1000, interval_sweep=(1, 4, 16, 64)),
}


def get_workload(name: str) -> Workload:
    return WORKLOADS[name.lower()]
