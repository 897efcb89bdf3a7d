"""Pins of the oracle's momentum local step (no GPU).

The paper's experiment (Section 4) runs the local steps with momentum 0.9; Algorithm 1 itself is
the case without momentum, and the paper does not define the buffers' fate at a restart.  The
oracle's form  v <- mu v + G,  x <- x - gamma v  and its three restart options are pinned here
against closed forms and independently written loops.
"""
import numpy as np
import pytest

import oracle
from helpers import oracle_args, small_mlp
from workloads import get_workload, make_inputs


def test_mu_zero_is_the_plain_step_of_eq3():
    rng = np.random.default_rng(0)
    x, g = rng.standard_normal(50), rng.standard_normal(50)
    v = rng.standard_normal(50)
    want = x - 0.3 * g
    oracle.momentum_step(x, v, g, 0.3, 0.0)
    assert np.array_equal(x, want) and np.array_equal(v, g)


def test_constant_gradient_closed_form():
    # v_t = g (1 - mu^t) / (1 - mu),   x_t = x_0 - gamma g sum_{tau <= t} (1 - mu^tau) / (1 - mu)
    rng = np.random.default_rng(1)
    g, x0 = rng.standard_normal(7), rng.standard_normal(7)
    mu, lr, steps = 0.9, 0.05, 40
    x, v = x0.copy(), np.zeros(7)
    for _ in range(steps):
        oracle.momentum_step(x, v, g, lr, mu)
    geo = (1.0 - mu ** np.arange(1, steps + 1)) / (1.0 - mu)
    assert np.allclose(v, g * geo[-1], rtol=1e-13)
    assert np.allclose(x, x0 - lr * g * geo.sum(), rtol=1e-12, atol=1e-13)


def _case():
    w = small_mlp(dims=(12, 9, 4), batch=5, n_workers=3, rows_per_worker=32, iterations=11, interval=3)
    return w, make_inputs(w)


def test_one_worker_is_heavy_ball_sgd():
    w, inp = _case()
    w = w.scaled(n_workers=1)
    inp = make_inputs(w)
    mu = 0.8
    got = oracle.run_prsgd(**oracle_args(w, inp), lr=w.lr, interval=w.interval, iterations=w.iterations,
                           momentum=mu)
    x = inp["x0"].astype(np.float64)
    v = np.zeros_like(x)
    for t in range(1, w.iterations + 1):
        rows = oracle.sample_rows(w.index_seed, 0, t, w.batch, w.rows_per_worker)
        g = oracle.loss_grad(w.model, x, w.dims, w.activation, inp["features"][0][rows],
                             inp["targets"][0][rows])[1]
        v = mu * v + g
        x = x - w.lr * v
    assert np.allclose(got["x"][0], x, rtol=1e-13, atol=1e-15)
    assert np.allclose(got["v"][0], v, rtol=1e-13, atol=1e-15)


def test_interval_one_with_averaged_buffers_is_minibatch_momentum_sgd():
    # averaging points and buffers after every step == one momentum step with the averaged gradient
    w, inp = _case()
    mu = 0.9
    got = oracle.run_prsgd(**oracle_args(w, inp), lr=w.lr, interval=1, iterations=w.iterations,
                           momentum=mu, momentum_restart="average")
    x = inp["x0"].astype(np.float64)
    v = np.zeros_like(x)
    for t in range(1, w.iterations + 1):
        g = np.zeros_like(x)
        for i in range(w.n_workers):
            rows = oracle.sample_rows(w.index_seed, i, t, w.batch, w.rows_per_worker)
            g += oracle.loss_grad(w.model, x, w.dims, w.activation, inp["features"][i][rows],
                                  inp["targets"][i][rows])[1]
        v = mu * v + g / w.n_workers
        x = x - w.lr * v
    for i in range(w.n_workers):
        assert np.allclose(got["x"][i], x, rtol=1e-12, atol=1e-14)
        assert np.allclose(got["v"][i], v, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("mode", ["keep", "average"])
def test_mean_recursion_with_momentum(mode):
    # xbar^t = xbar^{t-1} - gamma vbar^t,  vbar^t = mu vbar^{t-1} + (1/N) sum_i G_i^t  at every t:
    # the momentum analogue of eq. (5); averaging points (and buffers) does not move either mean
    w, inp = _case()
    mu = 0.7
    log = []
    oracle.run_prsgd(**oracle_args(w, inp), lr=w.lr, interval=w.interval, iterations=w.iterations,
                     momentum=mu, momentum_restart=mode, record=log.append)
    xbar = inp["x0"].astype(np.float64)
    vbar = np.zeros_like(xbar)
    for rec in log:
        vbar = mu * vbar + rec["g"].mean(axis=0)
        xbar = xbar - w.lr * vbar
        assert np.allclose(rec["x_after"].mean(axis=0), xbar, rtol=1e-12, atol=1e-14)
        assert np.allclose(rec["v"].mean(axis=0), vbar, rtol=1e-12, atol=1e-14)


def test_buffers_at_a_restart():
    w, inp = _case()
    out = {}
    for mode in ("keep", "average", "reset"):
        log = []
        oracle.run_prsgd(**oracle_args(w, inp), lr=w.lr, interval=w.interval, iterations=6,
                         momentum=0.9, momentum_restart=mode, record=log.append)
        out[mode] = log
    at = 2                                   # record of t = 3, the first restart
    assert out["keep"][at]["averaged"]
    assert not np.array_equal(out["keep"][at]["v"][0], out["keep"][at]["v"][1])
    assert np.array_equal(out["average"][at]["v"][0], out["average"][at]["v"][2])
    assert np.allclose(out["average"][at]["v"][0], out["keep"][at]["v"].mean(axis=0), rtol=1e-13)
    assert not out["reset"][at]["v"].any()
    for mode in out:                          # the points themselves restart from the average in every mode
        assert np.array_equal(out[mode][at]["x_after"][0], out[mode][at]["x_after"][1])
    with pytest.raises(ValueError):
        oracle.run_prsgd(**oracle_args(w, inp), lr=w.lr, interval=2, iterations=2, momentum=0.5,
                         momentum_restart="sometimes")
