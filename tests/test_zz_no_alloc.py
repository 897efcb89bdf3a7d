"""prsgd_init_static: contexts on the library's static workspace, for callers that cannot allocate.

Each case runs the same seeded problem through prsgd_init (caller-allocated workspace) and through
prsgd_init_static and demands bit-identical replicas, losses and indices; the run is also held to
the oracle at the usual tolerance.  Two static contexts are used in a row, the second smaller, so
that what the first left in the shared array (partial logits, arrival counters, activations) must
not leak into the second.
"""
import ctypes

import numpy as np
import pytest
import torch

from helpers import inputs_for, oracle_run, rel_err, small_mlp
from workloads import get_workload, make_inputs

pytestmark = pytest.mark.gpu


def _run(P, D, w, inp, static):
    cfg = P.make_config(w.n_workers, w.model, w.dims, w.batch, w.rows_per_worker, w.lr, w.index_seed,
                        activation=w.activation, gemm_dtype=w.gemm_dtype)
    feats = torch.from_numpy(inp["features"]).cuda()
    targs = torch.from_numpy(inp["targets"]).cuda()
    h = (P.prsgd_init_static if static else P.prsgd_init)(cfg, inp["x0"], feats, targs)
    assert (h.workspace is None) == static
    P.prsgd_run(h, w.iterations, w.interval)
    out = (D.read_all(h), P.prsgd_read_loss(h), P.prsgd_read_indices(h), P.prsgd_read_params(h, -1))
    P.prsgd_status(h)
    P.prsgd_destroy(h)
    return out


def test_static_workspace_contexts_match_allocated_ones_twice_in_a_row():
    from paper_1807_06629_amd import drivers as D, prsgd as P
    cases = [
        # epoch kernel: partial logits and arrival counters live in the workspace
        small_mlp(dims=(256, 128, 10), batch=8, n_workers=16, rows_per_worker=256, interval=4,
                  iterations=13, activation="relu", lr=0.02),
        # smaller, other kernels: per-layer chain with bf16 shadow, activations and the mean vector
        small_mlp(dims=(100, 72, 40, 10), batch=24, n_workers=3, rows_per_worker=128, interval=3,
                  iterations=7, gemm_dtype="bf16", activation="relu"),
        # smallest: least squares
        get_workload("c1").scaled(rows_per_worker=128, n_workers=3, iterations=9, interval=2),
    ]
    for w in cases:
        inp = make_inputs(w)
        ref = _run(P, D, w, inp, static=False)
        got = _run(P, D, w, inp, static=True)
        for a, b in zip(ref, got):
            assert np.array_equal(a, b)
        want = oracle_run(w, inp)
        tol = 5e-3 if w.gemm_dtype == "bf16" else 1e-4
        assert rel_err(got[0], want["x"]) <= tol


def test_static_workspace_limits_and_single_live_context():
    from paper_1807_06629_amd import prsgd as P
    # a configuration beyond the limit is refused with a message that names it
    big = get_workload("c3").scaled(rows_per_worker=64)
    cfg = P.make_config(big.n_workers, big.model, big.dims, big.batch, big.rows_per_worker, big.lr, 3,
                        activation="relu", gemm_dtype="bf16")
    assert P.prsgd_workspace_bytes(cfg) > (16 << 20)
    feats = torch.zeros((big.n_workers, 64, big.dims[0]), dtype=torch.float32, device="cuda")
    targs = torch.zeros((big.n_workers, 64), dtype=torch.int32, device="cuda")
    x0 = np.zeros(P.prsgd_param_count(cfg), dtype=np.float32)
    with pytest.raises(P.PrsgdError) as err:
        P.prsgd_init_static(cfg, x0, feats, targs)
    assert err.value.code == P.PRSGD_EINVAL and "static workspace" in str(err.value)
    # one live static context per device
    w = small_mlp()
    inp = inputs_for(w)
    cfg = P.make_config(w.n_workers, w.model, w.dims, w.batch, w.rows_per_worker, w.lr, w.index_seed,
                        activation=w.activation)
    feats = torch.from_numpy(inp["features"]).cuda()
    targs = torch.from_numpy(inp["targets"]).cuda()
    h = P.prsgd_init_static(cfg, inp["x0"], feats, targs)
    with pytest.raises(P.PrsgdError) as err:
        P.prsgd_init_static(cfg, inp["x0"], feats, targs)
    assert err.value.code == P.PRSGD_ESTATE
    P.prsgd_local_steps(h, 2)
    P.prsgd_destroy(h)
    h = P.prsgd_init_static(cfg, inp["x0"], feats, targs)      # free again after destroy
    P.prsgd_local_steps(h, 2)
    assert rel_err(np.stack([P.prsgd_read_params(h, i) for i in range(w.n_workers)]),
                   oracle_run(w, inp, iterations=2)["x"]) <= 1e-4
    P.prsgd_destroy(h)
    # an invalid call leaves the slot free
    ctx = ctypes.c_void_p()
    assert P._lib.prsgd_init_static(ctypes.byref(cfg), None, None, None, None, None,
                                    ctypes.byref(ctx)) == P.PRSGD_EINVAL
    h = P.prsgd_init_static(cfg, inp["x0"], feats, targs)
    P.prsgd_destroy(h)
