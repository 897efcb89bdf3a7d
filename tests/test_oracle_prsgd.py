"""Pins for the oracle's Algorithm 1/2/3 loops (no GPU).

Each test checks the loop against something the paper or plain mathematics
fixes, written out independently in the test: the I = 1 and N = 1 special cases
(Section 1), the mean recursion eq. (5), the restart identity eq. (6), equality
of the replicas after a restart, the reductions of Algorithms 2 and 3 to
Algorithm 1, and full-batch least squares against gradient descent and the
normal equations.
"""
import numpy as np
import pytest

from oracle import (loss_grad, node_average, run_heterogeneous, run_prsgd, run_prsgd_literal,
                    run_time_varying, sample_rows, time_varying_schedule)
from workloads import get_workload, make_inputs


def _small(name, **kw):
    w = get_workload(name).scaled(**kw)
    return w, make_inputs(w)


def _args(w, inp):
    return dict(model=w.model, dims=w.dims, activation=w.activation,
                features=inp["features"], targets=inp["targets"], x0=inp["x0"],
                n_workers=w.n_workers, batch=w.batch, seed=w.index_seed)


LSQ = dict(rows_per_worker=256, iterations=24)
MLP = dict(dims=(20, 12, 5), n_classes=5, rows_per_worker=128, n_workers=3, batch=6,
           iterations=20, interval=4)


@pytest.mark.parametrize("name,kw", [("c1", LSQ), ("c2", MLP)])
def test_interval_one_is_parallel_minibatch_sgd(name, kw):
    # Section 1: with I = 1, step-then-average equals one SGD step on the common point
    # with the gradient averaged over workers.
    w, inp = _small(name, **kw)
    out = run_prsgd(**_args(w, inp), lr=w.lr, interval=1, iterations=w.iterations)
    x = inp["x0"].astype(np.float64)
    for t in range(1, w.iterations + 1):
        gsum = np.zeros_like(x)
        for i in range(w.n_workers):
            rows = sample_rows(w.index_seed, i, t, w.batch, w.rows_per_worker)
            gsum += loss_grad(w.model, x, w.dims, w.activation,
                              inp["features"][i][rows], inp["targets"][i][rows])[1]
        x = x - w.lr * gsum / w.n_workers
    for i in range(w.n_workers):
        assert np.allclose(out["x"][i], x, rtol=1e-12, atol=1e-14)
    assert np.array_equal(out["x"][0], out["x"][-1])


@pytest.mark.parametrize("interval", [1, 3, 7])
def test_single_worker_is_plain_sgd(interval):
    # eq. (1) with N = 1: the average of one replica is the replica itself.
    w, inp = _small("c2", **{**MLP, "n_workers": 1})
    out = run_prsgd(**_args(w, inp), lr=w.lr, interval=interval, iterations=w.iterations)
    x = inp["x0"].astype(np.float64)
    for t in range(1, w.iterations + 1):
        rows = sample_rows(w.index_seed, 0, t, w.batch, w.rows_per_worker)
        x = x - w.lr * loss_grad(w.model, x, w.dims, w.activation,
                                 inp["features"][0][rows], inp["targets"][0][rows])[1]
    assert np.array_equal(out["x"][0], x)


@pytest.mark.parametrize("runner", [run_prsgd, run_prsgd_literal])
@pytest.mark.parametrize("interval", [1, 4, 5])
def test_mean_recursion_eq5_and_sum_preservation(runner, interval):
    w, inp = _small("c2", **MLP)
    log = []
    runner(**_args(w, inp), lr=w.lr, interval=interval, iterations=w.iterations,
           record=log.append)
    xbar = inp["x0"].astype(np.float64)
    for rec in log:
        xbar = xbar - w.lr * rec["g"].mean(axis=0)                  # eq. (5)
        got = rec["x_after"].mean(axis=0)
        assert np.allclose(got, xbar, rtol=1e-12, atol=1e-14)
        if runner is run_prsgd and rec["averaged"]:
            # averaging preserves sum_i x_i
            assert np.allclose(rec["x_stepped"].sum(axis=0), rec["x_after"].sum(axis=0),
                               rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("interval", [3, 4])
def test_restart_identity_eq6_and_equal_replicas_after_restart(interval):
    w, inp = _small("c1", **LSQ)
    log = []
    run_prsgd(**_args(w, inp), lr=w.lr, interval=interval, iterations=w.iterations,
              record=log.append)
    ybar = inp["x0"].astype(np.float64)
    acc = np.zeros((w.n_workers, ybar.size))
    spread_prev = 0.0
    for rec in log:
        acc += rec["g"]
        # eq. (6): x_i^t = ybar - gamma * sum of the gradients since the last restart
        assert np.allclose(rec["x_stepped"], ybar - w.lr * acc, rtol=1e-12, atol=1e-14)
        if rec["averaged"]:
            assert rec["t"] % interval == 0
            for i in range(1, w.n_workers):
                assert np.array_equal(rec["x_after"][i], rec["x_after"][0])
            ybar = rec["x_after"][0].copy()
            acc[:] = 0.0
            spread_prev = 0.0
        else:
            assert rec["t"] % interval != 0
            spread = np.abs(rec["x_after"] - rec["x_after"].mean(axis=0)).max()
            assert spread > 0.0
            spread_prev = spread


def test_literal_line_order_differs_in_phase_but_not_in_mean():
    # Printed order of Algorithm 1: the gradient at t = kI is taken *before* the average.
    w, inp = _small("c1", **LSQ)
    a, b = [], []
    run_prsgd(**_args(w, inp), lr=w.lr, interval=4, iterations=12, record=a.append)
    run_prsgd_literal(**_args(w, inp), lr=w.lr, interval=4, iterations=12, record=b.append)
    # identical until the first restart ...
    for t in range(3):
        assert np.array_equal(a[t]["x_after"], b[t]["x_after"])
    # ... at t = 4 the literal form keeps distinct replicas: x_i = ybar - gamma G_i
    rec = b[3]
    want = node_average(rec["x_before"]) - w.lr * rec["g"]
    assert np.allclose(rec["x_after"], want, rtol=1e-13, atol=1e-15)
    assert not np.array_equal(rec["x_after"][0], rec["x_after"][1])
    # with I = 1 the literal form lags by one average but its mean obeys the same recursion
    assert np.allclose(a[3]["x_after"].mean(axis=0), b[3]["x_after"].mean(axis=0),
                       rtol=1e-12, atol=1e-14)


def test_node_average_definition_and_single_replica_identity():
    x = np.random.default_rng(0).standard_normal((5, 7))
    want = sum(x[i] for i in range(5)) / 5
    assert np.allclose(node_average(x), want, rtol=1e-15)
    assert np.array_equal(node_average(x[:1]), x[0])


def test_run_not_multiple_of_interval_ends_unaveraged():
    w, inp = _small("c1", **LSQ)
    out = run_prsgd(**_args(w, inp), lr=w.lr, interval=5, iterations=12)
    assert not np.array_equal(out["x"][0], out["x"][1])
    out = run_prsgd(**_args(w, inp), lr=w.lr, interval=4, iterations=12)
    assert np.array_equal(out["x"][0], out["x"][1])


def test_resume_from_checkpoint_is_bit_identical():
    w, inp = _small("c2", **MLP)
    full = run_prsgd(**_args(w, inp), lr=w.lr, interval=3, iterations=14)
    first = run_prsgd(**_args(w, inp), lr=w.lr, interval=3, iterations=8)
    rest = run_prsgd(**_args(w, inp), lr=w.lr, interval=3, iterations=6, t_start=8,
                     x_init=first["x"])
    assert np.array_equal(full["x"], rest["x"])


def test_time_varying_with_constant_schedule_is_algorithm1():
    # Remark below Algorithm 2: constant (gamma, K) is Algorithm 1 with I = K.
    w, inp = _small("c2", **MLP)
    a = run_prsgd(**_args(w, inp), lr=w.lr, interval=4, iterations=20)
    b = run_time_varying(**_args(w, inp), epoch_lengths=[4] * 5, epoch_rates=[w.lr] * 5)
    # Algorithm 2 averages at epoch starts, so its last epoch ends un-averaged
    assert np.allclose(node_average(b["x"]), a["x"][0], rtol=1e-12, atol=1e-14)
    assert b["t"] == 20


def test_time_varying_rates_against_an_independent_loop():
    # Algorithm 2 with epochs of different lengths AND different rates, written out here with
    # nothing but the gradient and the row sampler: epoch s starts every worker from the mean of
    # the previous epoch's final points, then takes K^s steps at rate gamma^s; iterations are
    # numbered through.  A loop that kept gamma^1, or K^1, for every epoch fails.
    w, inp = _small("c2", **MLP)
    lengths, rates = [3, 1, 4, 2], [0.08, 0.02, 0.05, 0.11]
    out = run_time_varying(**_args(w, inp), epoch_lengths=lengths, epoch_rates=rates)
    xs = [inp["x0"].astype(np.float64).copy() for _ in range(w.n_workers)]
    t0 = 0
    for k_s, gamma_s in zip(lengths, rates):
        start = sum(xs) / w.n_workers
        for i in range(w.n_workers):
            x = start.copy()
            for t in range(t0 + 1, t0 + k_s + 1):
                rows = sample_rows(w.index_seed, i, t, w.batch, w.rows_per_worker)
                x = x - gamma_s * loss_grad(w.model, x, w.dims, w.activation,
                                            inp["features"][i][rows], inp["targets"][i][rows])[1]
            xs[i] = x
        t0 += k_s
    assert out["t"] == sum(lengths)
    assert np.allclose(out["x"], np.stack(xs), rtol=1e-12, atol=1e-14)
    # and the wrong loops really differ
    flat = run_time_varying(**_args(w, inp), epoch_lengths=lengths, epoch_rates=[rates[0]] * 4)
    assert np.abs(flat["x"] - out["x"]).max() > 1e-4


def test_time_varying_rates_closed_form_on_a_one_row_least_squares_problem():
    # one worker whose shard has a single row a, target y: every minibatch is that row, the
    # residual r = a.x - y obeys r <- r (1 - gamma |a|^2), so after the epochs
    #   r_T = r_0 * prod_s (1 - gamma^s |a|^2)^(K^s)
    rng = np.random.default_rng(3)
    a = rng.standard_normal((1, 1, 5)).astype(np.float32)
    y = rng.standard_normal((1, 1)).astype(np.float32)
    lengths, rates = [2, 5, 1, 3], [0.30, 0.05, 0.21, 0.11]
    out = run_time_varying("lsq", (5,), "none", a, y, np.zeros(5, np.float32), 1, 3,
                           epoch_lengths=lengths, epoch_rates=rates, seed=4)
    a64, y64 = a[0, 0].astype(np.float64), float(y[0, 0])
    want = -y64
    for k_s, g_s in zip(lengths, rates):
        want *= (1.0 - g_s * (a64 @ a64)) ** k_s
    assert a64 @ out["x"][0] - y64 == pytest.approx(want, rel=1e-11)
    assert out["t"] == 11


def test_time_varying_schedule_theorem2():
    ks, gs = time_varying_schedule(30, 2)
    assert ks[0] == 1 and gs[0] == 2.0                      # s=1: ceil(1/2)=1, N/1
    assert ks[7] == 1 and gs[7] == pytest.approx(2 / 4.0)   # s=8: ceil(2/2)=1, 2/8^(2/3)
    assert ks[26] == 2                                      # s=27: ceil(3/2)=2
    assert all(k >= 1 for k in ks)
    assert all(g2 < g1 for g1, g2 in zip(gs, gs[1:]))


def test_heterogeneous_with_equal_steps_is_algorithm1():
    # Section on heterogeneous networks: I_i = I for all i degrades to Algorithm 1.
    w, inp = _small("c2", **MLP)
    a = run_prsgd(**_args(w, inp), lr=w.lr, interval=4, iterations=12)
    b = run_heterogeneous(**_args(w, inp), lr=w.lr, worker_steps=[4, 4, 4], n_epochs=3)
    assert np.allclose(node_average(b["x"]), a["x"][0], rtol=1e-12, atol=1e-14)
    assert b["t"] == 12


def test_heterogeneous_slow_workers_take_zero_gradient_steps():
    w, inp = _small("c2", **MLP)
    steps = [5, 3, 1]
    out = run_heterogeneous(**_args(w, inp), lr=w.lr, worker_steps=steps, n_epochs=1)
    # one epoch from x0: worker i is x0 minus gamma times its first I_i gradients along
    # its own trajectory, with iteration numbers 1..I_i
    for i, k_i in enumerate(steps):
        x = inp["x0"].astype(np.float64)
        for t in range(1, k_i + 1):
            rows = sample_rows(w.index_seed, i, t, w.batch, w.rows_per_worker)
            x = x - w.lr * loss_grad(w.model, x, w.dims, w.activation,
                                     inp["features"][i][rows], inp["targets"][i][rows])[1]
        assert np.array_equal(out["x"][i], x)
    assert out["t"] == 5


def test_full_batch_least_squares_converges_to_normal_equations():
    # B = n with a constant index set makes each local step deterministic gradient descent;
    # checked against a plain numpy GD loop and against the normal-equation solution.
    w, inp = _small("c1", n_workers=1, rows_per_worker=1, batch=1, iterations=1)
    rng = np.random.default_rng(0)
    a = rng.standard_normal((1, 1, 3)).astype(np.float32)   # n = 1 row -> every draw is row 0
    y = rng.standard_normal((1, 1)).astype(np.float32)
    out = run_prsgd("lsq", (3,), "none", a, y, np.zeros(3, np.float32), 1, 4, 0.1, 2, 50, seed=1)
    x = np.zeros(3)
    a64, y64 = a[0, 0].astype(np.float64), float(y[0, 0])
    for _ in range(50):
        x = x - 0.1 * a64 * (a64 @ x - y64)
    assert np.allclose(out["x"][0], x, rtol=1e-12)
    # pooled multi-row problem: small steps approach the least-squares solution
    w, inp = _small("c1", rows_per_worker=64, batch=64, iterations=1)
    big = run_prsgd(**_args(w, inp), lr=0.05, interval=2, iterations=3000)
    pooled_a = inp["features"].reshape(-1, 64).astype(np.float64)
    pooled_y = inp["targets"].reshape(-1).astype(np.float64)
    x_star = np.linalg.lstsq(pooled_a, pooled_y, rcond=None)[0]
    # stochastic sampling noise leaves an O(gamma) neighbourhood
    assert np.linalg.norm(node_average(big["x"]) - x_star) < 0.15 * np.linalg.norm(x_star)


def test_least_squares_loss_decreases_on_c1_shape():
    w, inp = _small("c1", rows_per_worker=512)
    out0 = run_prsgd(**_args(w, inp), lr=w.lr, interval=w.interval, iterations=1)
    out = run_prsgd(**_args(w, inp), lr=w.lr, interval=w.interval, iterations=w.iterations)
    assert out["losses"].mean() < 0.2 * out0["losses"].mean()
