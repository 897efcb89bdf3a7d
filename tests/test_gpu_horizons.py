"""GPU parity at the configurations' own sizes and horizons (slow: the fp64 oracle sets the pace).

  c4  256-128-10 fp32, N = 64, n = 8192: the full T = 10,000 iterations at I = 1 and I = 8,
      parameters <= 1e-3 (the T-step gate).
  c3  3072-1024-1024-10 bf16, N = 16, n = 8192: 64 iterations (two restarts at I = 32).
  c5  4096x3-1000 bf16, N = 8, n = 8192: 20 iterations (one restart at I = 16), the launch
      configuration the benchmark times.

The bf16 configurations are gated on the minibatch loss, 2e-2 relative, at EVERY step, in two ways
driven by one oracle run:
  re-synchronised  the GPU takes each step from the oracle's own point (written back after every
                   step), so every step is a one-step comparison along the whole trajectory;
  free-running     the GPU is never corrected.  c5 holds the same 2e-2 gate on every worker's loss.
                   On c3 (gamma = 0.05 on unnormalised 3072-dimensional inputs: the loss explodes to
                   ~18, then collapses to 1e-2 .. 1e-7 per worker) rounding differences are amplified
                   chaotically -- one bf16 unit in the last place of ONE input value moves the loss
                   by ~1e-2 relative within six steps (tests/test_bf16_sensitivity.py, on the oracle
                   alone) and the fp32-accumulating kernels differ from the fp64 oracle in hundreds
                   of roundings per step -- so a single worker's tiny loss is not a stable
                   observable there (deviations of 10 % and more at losses of 1e-4).  What the
                   free-running c3 run is held to instead: its parameters stay within 1e-2 of the
                   oracle's at every step checked, and the loss averaged over the workers within
                   1e-1.
Both carry an absolute floor of 2^-20: the loss head evaluates log(sum exp) in fp32, which
resolves a nearly saturated row (loss below ~1e-6) only to 2^-23..2^-24.
"""
import concurrent.futures
import multiprocessing
import time

import numpy as np
import pytest

import oracle
from helpers import oracle_full_run, oracle_run, rel_err
from workloads import get_workload, make_inputs

pytestmark = [pytest.mark.gpu, pytest.mark.slow]

BF16_LOSS_TOL = 2e-2              # the stated gate for bf16-operand configurations
BF16_FREE_RUN_BAND = 1e-1         # free-running c3, loss averaged over the workers (see above)
LOSS_QUANTUM = 2.0 ** -20         # fp32 resolution of a nearly saturated softmax row, 8 ulps of 1
T_STEP_TOL = 1e-3
# Parameters one step after a common point.  Both sides round the same operands, so most replicas
# agree to ~1e-5; but one bf16 rounding of a layer-1 activation that falls the other way under
# fp32 accumulation shifts every layer-2 pre-activation of that sample by ~2e-4, enough to move one
# that sits that close to zero across the ReLU kink, which switches the sample's whole share
# (1/B) of a column of dW on or off.  With these recipes the first updates are as large as the
# weights themselves, so one such switch is worth up to ~1e-2 of max|x| (observed: 2.4e-3 on one
# worker of c3 at t = 1, 3e-5 on its neighbours).  The stated gate for these configurations is
# the loss; this bound only catches gross errors.
BF16_ONE_STEP_X_TOL = 1e-2


@pytest.fixture(scope="module")
def c4_oracle_runs():
    # the c4 oracle is bound by Python overhead on one core (~4 minutes for 640,000 worker
    # iterations); both intervals run in processes of their own while the other tests go on
    ctx = multiprocessing.get_context("spawn")
    pool = concurrent.futures.ProcessPoolExecutor(max_workers=2, mp_context=ctx)
    futures = {i: pool.submit(oracle_full_run, "c4", i) for i in (1, 8)}
    yield futures
    procs = list((getattr(pool, "_processes", None) or {}).values())
    for f in futures.values():
        f.cancel()
    pool.shutdown(wait=False, cancel_futures=True)
    for p in procs:                                           # a failed run must not leave them behind
        if p.is_alive():
            p.terminate()


@pytest.fixture(scope="module")
def P():
    from paper_1807_06629_amd import prsgd
    return prsgd


@pytest.fixture(scope="module")
def D():
    from paper_1807_06629_amd import drivers
    return drivers


def _loss_ok(got, want, rtol):
    return bool(np.all(np.abs(got - want) <= rtol * np.abs(want) + LOSS_QUANTUM))


def _bf16_horizon(P, D, capsys, name, steps, chaotic):
    w = get_workload(name).scaled(iterations=steps)
    inp = make_inputs(w)
    free = D.open_workload(w, inp, device="cuda:0")
    sync = D.open_workload(w, inp, device="cuda:0")
    t0 = time.time()
    probe = (0, w.n_workers - 1)                              # sampled replicas, every parameter
    worst = {"free": 0.0, "sync": 0.0, "x_sync": 0.0, "x_free": 0.0}

    def step(rec):
        t, want = rec["t"], rec["losses"]
        P.prsgd_run(free, 1, w.interval)
        P.prsgd_run(sync, 1, w.interval)
        lf, ls = P.prsgd_read_loss(free), P.prsgd_read_loss(sync)
        assert _loss_ok(ls, want, BF16_LOSS_TOL), ("re-synchronised", t, ls, want)
        if chaotic:
            assert abs(lf.mean() - want.mean()) <= BF16_FREE_RUN_BAND * want.mean() + LOSS_QUANTUM, \
                ("free-running, worker mean", t, lf, want)
            worst["free"] = max(worst["free"], float(abs(lf.mean() - want.mean()) / want.mean()))
        else:
            assert _loss_ok(lf, want, BF16_LOSS_TOL), ("free-running", t, lf, want)
            worst["free"] = max(worst["free"], float((np.abs(lf - want) / (np.abs(want) + 50 * LOSS_QUANTUM)).max()))
        worst["sync"] = max(worst["sync"], float((np.abs(ls - want) / (np.abs(want) + 50 * LOSS_QUANTUM)).max()))
        for i in probe:
            e = rel_err(P.prsgd_read_params(sync, i), rec["x_after"][i])
            worst["x_sync"] = max(worst["x_sync"], e)
            assert e <= BF16_ONE_STEP_X_TOL, ("re-synchronised parameters", t, i, e)
        if t == 1 or t % 8 == 0 or t == steps:
            for i in probe:
                e = rel_err(P.prsgd_read_params(free, i), rec["x_after"][i])
                worst["x_free"] = max(worst["x_free"], e)
                assert e <= BF16_ONE_STEP_X_TOL, ("free-running parameters", t, i, e)
        # the next step starts from the oracle's point (fp32-rounded, as the GPU holds it)
        if rec["averaged"]:
            P.prsgd_write_params(sync, -1, rec["x_after"][0].astype(np.float32))
        else:
            for i in range(w.n_workers):
                P.prsgd_write_params(sync, i, rec["x_after"][i].astype(np.float32))
        if t % 4 == 0 or t == steps:
            with capsys.disabled():
                print("[%s t=%d/%d %.0fs mean loss %.3e | worst so far: loss free %.1e re-sync %.1e, "
                      "x free %.1e re-sync %.1e]" % (name, t, steps, time.time() - t0, float(want.mean()),
                                                     worst["free"], worst["sync"], worst["x_free"],
                                                     worst["x_sync"]), flush=True)

    oracle_run(w, inp, record=step)
    assert P.prsgd_iteration(free) == steps
    P.prsgd_destroy(free)
    P.prsgd_destroy(sync)


def test_c3_full_size_two_restart_intervals(P, D, capsys, c4_oracle_runs):
    _bf16_horizon(P, D, capsys, "c3", 64, chaotic=True)


def test_c5_full_size_across_a_restart(P, D, capsys, c4_oracle_runs):
    _bf16_horizon(P, D, capsys, "c5", 20, chaotic=False)


@pytest.mark.parametrize("interval", [1, 8])
def test_c4_full_horizon(P, D, capsys, c4_oracle_runs, interval):
    w = get_workload("c4")
    inp = make_inputs(w)
    h = D.open_workload(w, inp, device="cuda:0")
    P.prsgd_run(h, w.iterations, interval)
    got = D.read_all(h)
    losses = P.prsgd_read_loss(h)
    assert P.prsgd_iteration(h) == w.iterations
    P.prsgd_destroy(h)
    fut = c4_oracle_runs[interval]
    t0 = time.time()
    while not fut.done():                                     # the oracle sets the pace
        try:
            fut.result(timeout=30.0)
        except concurrent.futures.TimeoutError:
            with capsys.disabled():
                print("[c4 I=%d: waiting for the oracle, %.0fs]" % (interval, time.time() - t0), flush=True)
    _, want_x, want_losses = fut.result()
    assert rel_err(got, want_x) <= T_STEP_TOL
    for i in range(1, w.n_workers):                           # I | T: the run ends on a restart
        assert np.array_equal(got[i], got[0])
    assert np.allclose(losses, want_losses, rtol=5e-2, atol=1e-5)
