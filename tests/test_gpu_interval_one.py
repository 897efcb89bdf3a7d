"""GPU parity of the pass that takes an epoch's last local iteration and the restart together,
    (1/N) sum_i (x_i - gamma G_i) = ybar - (gamma / N) sum_i G_i,   ybar = (1/N) sum_i x_i   (eq. 2-3).
With I = 1 every worker already sits at ybar and the pass is one step of parallel mini-batch SGD on
the common point with the gradient averaged over the N B samples of all workers (first footnote of
Section 1)."""
import numpy as np
import pytest
import torch

import oracle
from helpers import inputs_for, oracle_args, oracle_run, rel_err, small_mlp
from workloads import get_workload, make_inputs

pytestmark = pytest.mark.gpu

BF16_LOSS_TOL = 2e-2
LOSS_QUANTUM = 2.0 ** -20


@pytest.fixture(scope="module")
def P():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_1807_06629_amd import prsgd
    return prsgd


@pytest.fixture(scope="module")
def D():
    from paper_1807_06629_amd import drivers
    return drivers


def _names(P, h, k, interval):
    P.prsgd_profile_enable(h, True)
    P.prsgd_run(h, k, interval)
    names = {r["name"] for r in P.prsgd_profile_read(h)}
    P.prsgd_profile_enable(h, False)
    return names


SHAPES = [
    dict(dims=(100, 72, 40, 10), batch=24, n_workers=4),          # ragged everywhere, 32-row panels
    dict(dims=(96, 80, 40, 10), batch=64, n_workers=8),           # 64-row panels, N = 8
    dict(dims=(136, 264, 136, 12), batch=128, n_workers=2),       # 128-row panels, several tiles
    dict(dims=(200, 130, 7), batch=33, n_workers=3),              # odd tile group, one hidden layer
    dict(dims=(64, 10), batch=1, n_workers=5),                    # no hidden layer, one row
]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("activation", ["relu", "tanh"])
def test_interval_one_single_pass_against_the_oracle(P, D, shape, activation):
    w = small_mlp(activation=activation, gemm_dtype="bf16", interval=1, iterations=7,
                  rows_per_worker=256, **shape)
    inp = inputs_for(w)
    h = D.open_workload(w, inp, device="cuda:0")
    names = _names(P, h, w.iterations, 1)
    # first iteration: per-replica step + restart; from then on the single pass
    assert "step_mean" in names and "restart_mean" in names and "broadcast" not in names, names
    want = oracle_run(w, inp)
    got = P.prsgd_read_loss(h)
    assert np.all(np.abs(got - want["losses"]) <= BF16_LOSS_TOL * np.abs(want["losses"]) + LOSS_QUANTUM)
    xs = D.read_all(h)
    assert rel_err(xs, want["x"]) <= 5e-3
    for i in range(1, w.n_workers):                      # every worker reads as the node average
        assert np.array_equal(xs[i], xs[0])
    assert np.array_equal(P.prsgd_read_params(h, -1), xs[0])
    assert P.prsgd_iteration(h) == w.iterations
    P.prsgd_destroy(h)


@pytest.mark.parametrize("shape", SHAPES[:4])
def test_single_pass_against_the_per_replica_kernels(P, D, shape):
    """Same run through step + averaging kernels (broadcast every restart) and through the single
    pass.  The single pass rounds ybar - (gamma / N) sum_i G_i once where the other path rounds every
    x_i = ybar - gamma G_i and then their mean, and the two contract in different kernels: they
    agree to fp32 rounding, not bit for bit."""
    w = small_mlp(activation="relu", gemm_dtype="bf16", interval=1, iterations=2,
                  rows_per_worker=256, **shape)
    inp = inputs_for(w)
    outs = []
    for lazy in (True, False):
        h = D.open_workload(w, inp, device="cuda:0")
        P.prsgd_set_lazy_restart(h, lazy)
        names = _names(P, h, 2, 1)
        assert ("step_mean" in names) == lazy, names
        outs.append((P.prsgd_read_params(h, -1), P.prsgd_read_loss(h)))
        P.prsgd_destroy(h)
    (a, la), (b, lb) = outs
    assert np.array_equal(la, lb)                        # losses are taken before the update
    assert rel_err(a[None], b[None]) <= 1e-5


def test_single_pass_is_deterministic_and_resumes(P, D):
    w = small_mlp(dims=(100, 72, 40, 10), batch=24, n_workers=4, gemm_dtype="bf16", activation="relu",
                  rows_per_worker=128, interval=1, iterations=9)
    inp = inputs_for(w)
    runs = []
    for split in (None, 4):
        h = D.open_workload(w, inp, device="cuda:0")
        if split is None:
            P.prsgd_run(h, w.iterations, 1)
        else:                                            # stop, read, carry on: same bits
            P.prsgd_run(h, split, 1)
            P.prsgd_read_params(h, 1)
            P.prsgd_run(h, w.iterations - split, 1)
        runs.append(D.read_all(h))
        P.prsgd_destroy(h)
    assert np.array_equal(runs[0], runs[1])
    # a longer interval afterwards starts from the averaged point and writes full replicas again:
    # restarts fall on t = 1..5 (I = 1), then on the multiples of 2, and t = 9 ends unaveraged
    h = D.open_workload(w, inp, device="cuda:0")
    P.prsgd_run(h, 5, 1)
    P.prsgd_run(h, 4, 2)
    lengths = [1] * 6 + [2, 1]
    want = oracle.run_time_varying(**oracle_args(w, inp), epoch_lengths=lengths,
                                   epoch_rates=[w.lr] * len(lengths))
    xs = D.read_all(h)
    assert not np.array_equal(xs[0], xs[1])
    assert rel_err(xs, want["x"]) <= 5e-3
    P.prsgd_destroy(h)


def test_single_pass_with_time_varying_rates(P, D):
    # Algorithm 2 with K^s = 1: the rate changes between iterations, the pass reads it per launch
    w = small_mlp(dims=(100, 72, 40, 10), batch=24, n_workers=4, gemm_dtype="bf16", activation="tanh",
                  rows_per_worker=128, interval=1, iterations=6)
    inp = inputs_for(w)
    rates = [0.05, 0.04, 0.03, 0.02, 0.01, 0.005]
    h = D.open_workload(w, inp, device="cuda:0")
    for r in rates:
        P.prsgd_set_lr(h, r)
        P.prsgd_run(h, 1, 1)
    want = oracle.run_time_varying(**oracle_args(w, inp), epoch_lengths=[1] * len(rates), epoch_rates=rates)
    xbar = oracle.node_average(want["x"])               # the GPU run ends on a restart
    assert rel_err(P.prsgd_read_params(h, -1)[None], xbar[None]) <= 5e-3
    P.prsgd_destroy(h)


@pytest.mark.parametrize("shape", SHAPES[:4] + [dict(dims=(256, 128, 64, 10), batch=32, n_workers=4)])
@pytest.mark.parametrize("interval", [2, 3])
def test_last_iteration_of_an_epoch_taken_with_the_restart(P, D, shape, interval):
    """I >= 2: the pass against the separate kernels (local iteration, then the restart kernel) after
    one epoch: fp32 rounding apart; both against the oracle over several epochs; a run that ends inside
    an epoch ends with distinct replicas."""
    w = small_mlp(activation="relu", gemm_dtype="bf16", interval=interval, iterations=2 * interval + 1,
                  rows_per_worker=256, **shape)
    inp = inputs_for(w)
    outs = []
    for fused in (True, False):
        h = D.open_workload(w, inp, device="cuda:0")
        P.prsgd_set_restart_fusion(h, fused)
        names = _names(P, h, interval, interval)             # exactly one epoch
        assert ("step_mean" in names) == fused and "restart_mean" in names, names
        one_epoch = P.prsgd_read_params(h, -1)
        for i in (0, w.n_workers - 1):                       # every worker reads as the average
            assert np.array_equal(P.prsgd_read_params(h, i), one_epoch)
        P.prsgd_run(h, w.iterations - interval, interval)    # one more epoch and one iteration into the next
        outs.append((one_epoch, D.read_all(h), P.prsgd_read_loss(h)))
        P.prsgd_destroy(h)
    assert rel_err(outs[0][0][None], outs[1][0][None]) <= 1e-5
    want = oracle_run(w, inp)
    for _, xs, losses in outs:
        assert not np.array_equal(xs[0], xs[1])              # the run ended inside an epoch
        assert rel_err(xs, want["x"]) <= 5e-3
        assert np.all(np.abs(losses - want["losses"]) <= BF16_LOSS_TOL * np.abs(want["losses"]) + LOSS_QUANTUM)
