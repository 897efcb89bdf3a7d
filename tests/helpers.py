"""Shared helpers of the GPU parity tests (comparison norms, oracle runs)."""
from __future__ import annotations

import numpy as np

import oracle
from workloads import Workload, make_inputs


def rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max_i ||got_i - want_i||_inf / ||want_i||_inf over replicas (rows)."""
    got = np.atleast_2d(np.asarray(got, dtype=np.float64))
    want = np.atleast_2d(np.asarray(want, dtype=np.float64))
    num = np.abs(got - want).max(axis=1)
    den = np.maximum(np.abs(want).max(axis=1), 1e-30)
    return float((num / den).max())


def oracle_args(w: Workload, inp):
    return dict(model=w.model, dims=w.dims, activation=w.activation, features=inp["features"],
                targets=inp["targets"], x0=inp["x0"], n_workers=w.n_workers, batch=w.batch,
                seed=w.index_seed, bf16=(w.gemm_dtype == "bf16"))


def oracle_run(w: Workload, inp, iterations=None, interval=None, **kw):
    return oracle.run_prsgd(**oracle_args(w, inp), lr=w.lr,
                            interval=w.interval if interval is None else interval,
                            iterations=w.iterations if iterations is None else iterations, **kw)


def small_mlp(**kw) -> Workload:
    base = dict(name="t", model="mlp", n_workers=3, dims=(37, 19, 7), activation="tanh",
                gemm_dtype="f32", batch=5, rows_per_worker=64, lr=0.05, interval=4, iterations=8,
                n_classes=7)
    base.update(kw)
    if "n_classes" not in kw:
        base["n_classes"] = base["dims"][-1]
    return Workload(**base)


def inputs_for(w: Workload):
    return make_inputs(w)


def oracle_full_run(name: str, interval: int):
    """A workload's whole oracle trajectory; meant to run in a spawned process (numpy only) while
    the GPU tests go on.  The small configurations are bound by Python overhead, so one BLAS
    thread is enough and keeps the cores free for the other oracle runs."""
    from threadpoolctl import threadpool_limits
    from workloads import get_workload
    w = get_workload(name)
    inp = make_inputs(w)
    with threadpool_limits(limits=1):
        out = oracle_run(w, inp, interval=interval)
    return interval, out["x"], out["losses"]
