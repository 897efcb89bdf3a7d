"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on identical seeded inputs.

Gates (norm = max over replicas of
||got - want||_inf / ||want||_inf):
    minibatch indices              bit-exact
    fp32 parameters, one step      <= 1e-5
    fp32 parameters, T steps       <= 1e-3
    bf16-operand configs, loss     <= 2e-2 relative
"""
import numpy as np
import pytest
import torch

import oracle
from helpers import inputs_for, oracle_args, oracle_run, rel_err, small_mlp
from workloads import get_workload, make_inputs

pytestmark = pytest.mark.gpu

ONE_STEP_TOL = 1e-5
T_STEP_TOL = 1e-3
BF16_LOSS_TOL = 2e-2
# Absolute floor of every bf16 loss comparison: the loss head evaluates log(sum exp) in fp32,
# which resolves a nearly saturated row (loss below ~1e-6) only to 2^-23..2^-24; 8 ulps of 1.
LOSS_QUANTUM = 2.0 ** -20
# Free-running multi-step trajectories of the c3 recipe (gamma = 0.05, unnormalised 3072-dimensional
# inputs: the loss explodes, then collapses) amplify rounding differences chaotically: one bf16
# unit in the last place of one input value moves the loss ~1e-2 relative within six steps
# (tests/test_bf16_sensitivity.py, on the oracle alone).  Such runs are held to this band; the
# 2e-2 gate is applied to every step taken from the oracle's own point.
BF16_FREE_RUN_BAND = 1e-1


def _bf16_loss_ok(got, want, rtol=BF16_LOSS_TOL):
    return bool(np.all(np.abs(got - want) <= rtol * np.abs(want) + LOSS_QUANTUM))


def _resync(P, h, rec):
    """Puts the GPU on the oracle's point after the recorded iteration (fp32-rounded)."""
    if rec["averaged"]:
        P.prsgd_write_params(h, -1, rec["x_after"][0].astype(np.float32))
    else:
        for i in range(rec["x_after"].shape[0]):
            P.prsgd_write_params(h, i, rec["x_after"][i].astype(np.float32))


@pytest.fixture(scope="module")
def P():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_1807_06629_amd import prsgd
    return prsgd


@pytest.fixture(scope="module")
def D():
    from paper_1807_06629_amd import drivers
    return drivers


def _open(D, w, inp, **kw):
    return D.open_workload(w, inp, device="cuda:0", **kw)


# --------------------------------------------------------------------------- index stream
@pytest.mark.parametrize("seed,n_workers,batch,rows,t_first,n_steps", [
    (3, 16, 256, 8192, 1, 256),                       # 1,048,576 tuples
    ((0xDEADBEEF << 32) | 0x12345678, 5, 33, 1 << 20, (1 << 32) - 7, 40),   # t crosses 2^32
    (7, 3, 7, 1, 1, 5),                               # n = 1: every draw is row 0
    (7, 3, 9, 2, 1, 50),
    (11, 2, 64, 1 << 31, 123456789, 16),              # largest shard
])
def test_index_stream_bit_exact(P, seed, n_workers, batch, rows, t_first, n_steps):
    got = P.prsgd_sample_indices(seed, n_workers, batch, rows, t_first, n_steps).cpu().numpy()
    want = np.empty_like(got, dtype=np.int64)
    for s in range(n_steps):
        for i in range(n_workers):
            want[s, i] = oracle.sample_rows(seed, i, t_first + s, batch, rows)
    assert np.array_equal(got.astype(np.int64), want)


def test_local_step_uses_the_same_rows_as_the_stateless_stream(P, D):
    w = small_mlp(batch=13, rows_per_worker=256)
    inp = inputs_for(w)
    h = _open(D, w, inp)
    P.prsgd_local_steps(h, 3)
    got = P.prsgd_read_indices(h)
    for i in range(w.n_workers):
        assert np.array_equal(got[i], oracle.sample_rows(w.index_seed, i, 3, w.batch, 256))
    P.prsgd_destroy(h)


def test_draw_ahead_follows_the_iteration_counter(P, D):
    """The layer-wise path draws the minibatch of iteration t + 1 during iteration t; a changed
    counter, or a heterogeneous epoch (masked draws) in between, must not let a stale draw through.
    The draw is a pure function of (seed, worker, t, slot): the row indices tell."""
    w = small_mlp(dims=(40, 24, 16, 6), batch=6, n_workers=3, rows_per_worker=128)   # per-layer kernels
    inp = inputs_for(w)
    h = _open(D, w, inp)

    def rows_of(t):
        return np.stack([oracle.sample_rows(w.index_seed, i, t, w.batch, w.rows_per_worker)
                         for i in range(w.n_workers)])

    P.prsgd_local_steps(h, 1)
    assert np.array_equal(P.prsgd_read_indices(h), rows_of(1))
    P.prsgd_local_steps(h, 2)                          # both taken from draws made ahead
    assert np.array_equal(P.prsgd_read_indices(h), rows_of(3))
    P.prsgd_set_iteration(h, 40)                       # the waiting draw (t = 4) is not t = 41
    P.prsgd_local_steps(h, 1)
    assert np.array_equal(P.prsgd_read_indices(h), rows_of(41))
    P.prsgd_set_iteration(h, 41)                       # same counter again: the draw ahead is t = 42
    P.prsgd_local_steps(h, 1)
    assert np.array_equal(P.prsgd_read_indices(h), rows_of(42))
    P.prsgd_local_steps_hetero(h, [2, 0, 1])           # t = 43, 44; worker 1 draws nothing
    got = P.prsgd_read_indices(h)
    assert np.array_equal(got[0], rows_of(44)[0])
    P.prsgd_local_steps(h, 1)                          # t = 45, complete again
    assert np.array_equal(P.prsgd_read_indices(h), rows_of(45))
    P.prsgd_destroy(h)
    # the same sequence of counters gives the same parameters as stepping without any jump
    a, b = _open(D, w, inp), _open(D, w, inp)
    P.prsgd_local_steps(a, 5)
    for _ in range(5):
        P.prsgd_set_iteration(b, P.prsgd_iteration(b))
        P.prsgd_local_steps(b, 1)
    assert np.array_equal(D.read_all(a), D.read_all(b))
    P.prsgd_destroy(a)
    P.prsgd_destroy(b)


# --------------------------------------------------------------------------- least squares
def test_c1_least_squares_full_run(P, D):
    w = get_workload("c1")
    inp = make_inputs(w)
    h = _open(D, w, inp)
    P.prsgd_local_steps(h, 1)
    one = oracle_run(w, inp, iterations=1)
    assert rel_err(D.read_all(h), one["x"]) <= ONE_STEP_TOL
    assert np.allclose(P.prsgd_read_loss(h), one["losses"], rtol=1e-5)
    P.prsgd_run(h, w.iterations - 1, w.interval)
    full = oracle_run(w, inp)
    got = D.read_all(h)
    assert rel_err(got, full["x"]) <= T_STEP_TOL
    assert P.prsgd_iteration(h) == w.iterations
    for i in range(1, w.n_workers):                     # I | T: the run ends on a restart
        assert np.array_equal(got[i], got[0])
    assert np.allclose(P.prsgd_read_loss(h), full["losses"], rtol=1e-3)
    P.prsgd_destroy(h)


# the shapes with d % 4 == 0 and at most 8192 minibatch floats take the LDS-staged kernel in each
# of its four (vectors per thread, prefetch depth) variants; the others the plain kernel
@pytest.mark.parametrize("d,batch", [(1, 1), (7, 3), (300, 70), (1000, 9), (4, 1), (32, 40), (128, 20),
                                     (64, 100), (8, 300), (2048, 4), (16, 512),
                                     (8192, 2), (8192, 600)])   # largest d: > 64 KiB of LDS in the plain kernel
def test_least_squares_ragged_shapes(P, D, d, batch):
    w = get_workload("c1").scaled(dims=(d,), batch=batch, rows_per_worker=128, n_workers=3,
                                  lr=0.01 / max(1, d // 64), interval=3, iterations=10)
    inp = make_inputs(w)
    h = _open(D, w, inp)
    P.prsgd_run(h, w.iterations, w.interval)
    want = oracle_run(w, inp)
    assert rel_err(D.read_all(h), want["x"]) <= 1e-4
    assert np.array_equal(P.prsgd_read_indices(h)[1],
                          oracle.sample_rows(w.index_seed, 1, w.iterations, batch, 128))
    P.prsgd_destroy(h)


# --------------------------------------------------------------------------- MLP, fp32
MLP_SHAPES = [
    dict(dims=(37, 19, 7), batch=5),                             # everything ragged, one tile
    dict(dims=(200, 150, 70, 10), batch=40),                     # several tiles, 64-row variant
    dict(dims=(200, 150, 70, 10), batch=100, n_workers=2),       # 128-row variant
    dict(dims=(130, 260, 10), batch=160, n_workers=2),           # batch spans two M tiles
    dict(dims=(64, 10), batch=8),                                # single layer (softmax regression)
    dict(dims=(33, 1), batch=4),                                 # one class: loss identically 0
    dict(dims=(20, 16, 16, 16, 16, 5), batch=1, n_workers=1),    # B = 1, N = 1, deep
    dict(dims=(48, 40, 300), batch=9, n_workers=2),              # wide loss head: one workgroup per row
    dict(dims=(72, 1000), batch=5, n_workers=2),                 # ... with a split logits contraction
]


@pytest.mark.parametrize("shape", MLP_SHAPES)
@pytest.mark.parametrize("activation", ["tanh", "relu"])
@pytest.mark.parametrize("fused", [True, False])
def test_mlp_fp32_one_step_and_short_run(P, D, shape, activation, fused):
    w = small_mlp(activation=activation, **shape)
    inp = inputs_for(w)
    h = _open(D, w, inp, fused_update=fused)
    P.prsgd_local_steps(h, 1)
    one = oracle_run(w, inp, iterations=1)
    assert rel_err(D.read_all(h), one["x"]) <= ONE_STEP_TOL
    assert np.allclose(P.prsgd_read_loss(h), one["losses"], rtol=2e-5, atol=1e-6)
    P.prsgd_run(h, w.iterations - 1, w.interval)
    want = oracle_run(w, inp)
    assert rel_err(D.read_all(h), want["x"]) <= 1e-4
    P.prsgd_destroy(h)


def test_c2_shape_reduced_horizon(P, D):
    w = get_workload("c2").scaled(iterations=64, rows_per_worker=1024)
    inp = make_inputs(w)
    h = _open(D, w, inp)
    P.prsgd_local_steps(h, 1)
    assert rel_err(D.read_all(h), oracle_run(w, inp, iterations=1)["x"]) <= ONE_STEP_TOL
    P.prsgd_run(h, w.iterations - 1, w.interval)
    want = oracle_run(w, inp)
    got = D.read_all(h)
    assert rel_err(got, want["x"]) <= T_STEP_TOL
    assert np.array_equal(got[0], got[-1])
    assert np.allclose(P.prsgd_read_params(h, -1), want["x"][0], rtol=0, atol=T_STEP_TOL * np.abs(want["x"][0]).max())
    P.prsgd_destroy(h)


def test_c4_shape_interval_sweep_reduced_horizon(P, D):
    base = get_workload("c4").scaled(iterations=48, rows_per_worker=256)
    inp = make_inputs(base)
    for interval in base.interval_sweep:
        h = _open(D, base, inp)
        P.prsgd_run(h, base.iterations, interval)
        want = oracle_run(base, inp, interval=interval)
        assert rel_err(D.read_all(h), want["x"]) <= T_STEP_TOL, interval
        P.prsgd_destroy(h)


# --------------------------------------------------------------------------- epoch kernel (one hidden layer, fp32)
EPOCH_SHAPES = [
    dict(dims=(64, 32, 10), batch=8, n_workers=3),                 # P=2 teams, N not a multiple of 8
    dict(dims=(100, 48, 7), batch=20, n_workers=8),                # ragged d0 (7 row blocks), two batch tiles
    dict(dims=(256, 128, 10), batch=8, n_workers=16),              # C4's shape
    dict(dims=(784, 256, 10), batch=32, n_workers=8),              # C2's shape
    dict(dims=(784, 256, 10), batch=32, n_workers=16),             # one workgroup on every compute unit
    dict(dims=(600, 48, 7), batch=20, n_workers=3),                # ragged last row block of 38
    dict(dims=(900, 32, 33), batch=30, n_workers=2),               # 57 row blocks: eight per wavefront; 33 classes
    dict(dims=(128, 64, 33), batch=50, n_workers=2),               # 33 classes (padded to 48), four batch tiles
    dict(dims=(1024, 16, 3), batch=1, n_workers=1),                # widest input, B = 1, single-member team
]


def _kernel_names(P, h, k, interval):
    P.prsgd_profile_enable(h, True)
    P.prsgd_run(h, k, interval)
    names = {r["name"] for r in P.prsgd_profile_read(h)}
    P.prsgd_profile_enable(h, False)
    return names


@pytest.mark.parametrize("shape", EPOCH_SHAPES)
@pytest.mark.parametrize("activation", ["tanh", "relu"])
def test_epoch_kernel_parity(P, D, shape, activation):
    w = small_mlp(activation=activation, rows_per_worker=128, interval=4, iterations=12, lr=0.02,
                  **shape)
    inp = inputs_for(w)
    h = _open(D, w, inp)
    P.prsgd_local_steps(h, 1)
    one = oracle_run(w, inp, iterations=1)
    assert rel_err(D.read_all(h), one["x"]) <= ONE_STEP_TOL
    assert np.allclose(P.prsgd_read_loss(h), one["losses"], rtol=2e-5, atol=1e-6)
    assert np.array_equal(P.prsgd_read_indices(h)[0],
                          oracle.sample_rows(w.index_seed, 0, 1, w.batch, w.rows_per_worker))
    names = _kernel_names(P, h, w.iterations - 1, w.interval)
    assert "mlp2_epoch" in names and "gemm_fwd" not in names      # the fused path really ran
    want = oracle_run(w, inp)
    assert rel_err(D.read_all(h), want["x"]) <= 1e-4
    assert np.allclose(P.prsgd_read_loss(h), want["losses"], rtol=1e-3, atol=1e-6)
    P.prsgd_destroy(h)


def test_epoch_kernel_matches_layerwise_kernels(P, D):
    # same problem through the fused epoch kernel and through the per-layer kernel chain
    w = small_mlp(dims=(96, 32, 10), batch=16, n_workers=8, rows_per_worker=128, interval=5,
                  iterations=15, activation="tanh")
    inp = inputs_for(w)
    outs = []
    for fused in (True, False):           # the un-fused update path never uses the epoch kernel
        h = _open(D, w, inp, fused_update=fused)
        P.prsgd_run(h, w.iterations, w.interval)
        outs.append(D.read_all(h))
        P.prsgd_destroy(h)
    assert rel_err(outs[0], outs[1]) <= 1e-5


@pytest.mark.parametrize("dims", [(64, 32, 10), (640, 32, 10)])     # with and without minibatch prefetch
def test_epoch_kernel_heterogeneous_steps(P, D, dims):
    w = small_mlp(dims=dims, batch=8, n_workers=4, rows_per_worker=128)
    inp = inputs_for(w)
    steps = [5, 3, 0, 1]
    h = _open(D, w, inp)
    D.run_algorithm3(h, steps, 3)
    args = oracle_args(w, inp)
    args.pop("bf16")
    want = oracle.run_heterogeneous(**args, lr=w.lr, worker_steps=steps, n_epochs=3)
    assert P.prsgd_iteration(h) == want["t"]
    assert rel_err(D.read_all(h), want["x"]) <= 1e-4
    P.prsgd_destroy(h)


# --------------------------------------------------------------------------- MLP, bf16 operands
@pytest.mark.parametrize("shape", [
    dict(dims=(96, 80, 40, 10), batch=64, n_workers=4),
    dict(dims=(100, 72, 10), batch=24, n_workers=3),
    dict(dims=(136, 264, 136, 12), batch=128, n_workers=2),
    dict(dims=(96, 80, 520), batch=40, n_workers=3),              # wide loss head, padded to whole tiles
])
@pytest.mark.parametrize("fused", [True, False])
def test_mlp_bf16_loss_and_parameters(P, D, shape, fused):
    w = small_mlp(activation="relu", gemm_dtype="bf16", interval=4, iterations=8, **shape)
    inp = inputs_for(w)
    h = _open(D, w, inp, fused_update=fused)
    P.prsgd_local_steps(h, 1)
    one = oracle_run(w, inp, iterations=1)
    assert np.allclose(P.prsgd_read_loss(h), one["losses"], rtol=BF16_LOSS_TOL)
    # the oracle applies the same operand roundings, so one step agrees far inside the loss gate
    assert rel_err(D.read_all(h), one["x"]) <= 1e-4
    P.prsgd_run(h, w.iterations - 1, w.interval)
    want = oracle_run(w, inp)
    assert np.allclose(P.prsgd_read_loss(h), want["losses"], rtol=BF16_LOSS_TOL)
    assert rel_err(D.read_all(h), want["x"]) <= 5e-3
    P.prsgd_destroy(h)


def test_c3_shape_noniid_reduced(P, D):
    w = get_workload("c3").scaled(n_workers=4, rows_per_worker=512, iterations=6, interval=3)
    inp = make_inputs(w)
    free, sync = _open(D, w, inp), _open(D, w, inp)
    log = []
    want = oracle_run(w, inp, record=log.append)
    for rec in log:
        # every step from the oracle's own point: the stated gate; free-running: the band
        P.prsgd_run(sync, 1, w.interval)
        got = P.prsgd_read_loss(sync)
        assert _bf16_loss_ok(got, rec["losses"]), (rec["t"], got, rec["losses"])
        assert rel_err(D.read_all(sync), rec["x_after"]) <= 1e-3
        _resync(P, sync, rec)
        P.prsgd_run(free, 1, w.interval)
        got = P.prsgd_read_loss(free)
        assert _bf16_loss_ok(got, rec["losses"], BF16_FREE_RUN_BAND), (rec["t"], got, rec["losses"])
    assert rel_err(D.read_all(free), want["x"]) <= 5e-3
    P.prsgd_destroy(free)
    P.prsgd_destroy(sync)


@pytest.mark.parametrize("shape", [
    dict(dims=(256, 128, 64, 10), batch=32, n_workers=3),
    dict(dims=(384, 192, 10), batch=64, n_workers=8),
    dict(dims=(512, 64, 72, 12), batch=128, n_workers=2),
])
@pytest.mark.parametrize("activation,momentum", [("relu", 0.0), ("tanh", 0.0), ("relu", 0.9)])
def test_first_layer_backward_runs_the_next_forward_product(P, D, shape, activation, momentum):
    """Layers made of whole tiles: the backward kernel of layer 1 also computes H_1 of the next
    iteration from the weights it writes.  Same bits as the two separate launches, through restarts,
    a rewritten replica, a moved iteration counter and an Algorithm 3 epoch in between."""
    w = small_mlp(gemm_dtype="bf16", activation=activation, rows_per_worker=256, interval=3, iterations=8,
                  momentum=momentum, **shape)
    inp = inputs_for(w)
    outs = []
    for on in (True, False):
        h = _open(D, w, inp)
        P.prsgd_set_first_layer_fusion(h, on)
        names = _kernel_names(P, h, w.iterations, w.interval)
        assert ("gemm_bwd_first" in names) == on, names
        first = (D.read_all(h), P.prsgd_read_loss(h), P.prsgd_read_indices(h))
        # the activation computed ahead must be dropped when the points or the counter change
        x1 = P.prsgd_read_params(h, 1)
        P.prsgd_write_params(h, 1, (x1 * np.float32(0.5)).astype(np.float32))
        P.prsgd_local_steps(h, 2)
        P.prsgd_set_iteration(h, 100)
        P.prsgd_local_steps(h, 2)
        if momentum == 0.0:                           # Algorithm 3 is not defined with momentum
            P.prsgd_local_steps_hetero(h, [1] + [2] * (w.n_workers - 1))
        P.prsgd_run(h, 4, 2)
        outs.append(first + (D.read_all(h), P.prsgd_read_loss(h)))
        P.prsgd_destroy(h)
    for a, b in zip(outs[0], outs[1]):
        assert np.array_equal(a, b)
    want = oracle_run(w, inp, **(dict(momentum=momentum) if momentum else {}))
    assert _bf16_loss_ok(outs[0][1], want["losses"])
    assert rel_err(outs[0][0], want["x"]) <= (5e-3 if momentum == 0.0 else 2e-2)
    for i in range(w.n_workers):
        assert np.array_equal(outs[0][2][i], oracle.sample_rows(w.index_seed, i, w.iterations, w.batch, 256))


def test_bf16_fused_backward_kernel_runs_and_falls_back_above_128_rows(P, D):
    # B <= 128: one fused backward kernel per layer; B > 128: the separate products
    for batch, expect in ((48, "gemm_bwd"), (160, "gemm_dw")):
        w = small_mlp(dims=(72, 136, 40, 10), batch=batch, n_workers=2, gemm_dtype="bf16",
                      activation="relu", rows_per_worker=256, interval=3, iterations=6)
        inp = inputs_for(w)
        h = _open(D, w, inp)
        P.prsgd_set_restart_fusion(h, False)     # the pass that closes an epoch has products of its own
        names = _kernel_names(P, h, w.iterations, w.interval)
        assert expect in names, names
        assert ("gemm_dx" in names) == (expect == "gemm_dw")
        want = oracle_run(w, inp)
        assert np.allclose(P.prsgd_read_loss(h), want["losses"], rtol=BF16_LOSS_TOL)
        assert rel_err(D.read_all(h), want["x"]) <= 5e-3
        P.prsgd_destroy(h)


def test_bf16_heterogeneous_steps_mask_the_fused_backward_kernel(P, D):
    w = small_mlp(dims=(100, 72, 40, 10), batch=24, n_workers=4, gemm_dtype="bf16", activation="tanh")
    inp = inputs_for(w)
    steps = [4, 0, 2, 1]
    h = _open(D, w, inp)
    D.run_algorithm3(h, steps, 2)
    args = oracle_args(w, inp)
    want = oracle.run_heterogeneous(**args, lr=w.lr, worker_steps=steps, n_epochs=2)
    assert P.prsgd_iteration(h) == want["t"]
    assert rel_err(D.read_all(h), want["x"]) <= 5e-3
    P.prsgd_destroy(h)


@pytest.mark.parametrize("shape", [
    dict(dims=(72, 96, 256, 10), batch=32, n_workers=3),          # layer 2: three 32-row bands
    dict(dims=(64, 160, 384, 12), batch=64, n_workers=2),         # five bands, six column tiles
    dict(dims=(80, 64, 256, 256, 10), batch=128, n_workers=2),    # layers 2 and 3
])
@pytest.mark.parametrize("activation,momentum", [("relu", 0.0), ("tanh", 0.0), ("relu", 0.9)])
def test_backward_kernel_on_whole_tile_layers_with_few_row_bands(P, D, shape, activation, momentum):
    """Hidden layers made of whole 32 x 64 tiles, too small to give every compute unit two 64-row
    bands: the backward kernel walks them in 32-row bands.  One step, a run with restarts and an
    Algorithm 3 epoch against the oracle."""
    w = small_mlp(gemm_dtype="bf16", activation=activation, rows_per_worker=256, interval=3, iterations=7,
                  momentum=momentum, **shape)
    inp = inputs_for(w)
    kw = dict(momentum=momentum) if momentum else {}
    h = _open(D, w, inp)
    P.prsgd_set_restart_fusion(h, False)
    P.prsgd_local_steps(h, 1)
    one = oracle_run(w, inp, iterations=1, **kw)
    assert np.allclose(P.prsgd_read_loss(h), one["losses"], rtol=BF16_LOSS_TOL)
    assert rel_err(D.read_all(h), one["x"]) <= 1e-4
    P.prsgd_run(h, w.iterations - 1, w.interval)
    want = oracle_run(w, inp, **kw)
    assert _bf16_loss_ok(P.prsgd_read_loss(h), want["losses"])
    assert rel_err(D.read_all(h), want["x"]) <= (5e-3 if momentum == 0.0 else 2e-2)
    P.prsgd_destroy(h)
    if momentum == 0.0:
        steps = [2, 0, 1][:w.n_workers]
        h = _open(D, w, inp)
        D.run_algorithm3(h, steps, 2)
        args = oracle_args(w, inp)
        want = oracle.run_heterogeneous(**args, lr=w.lr, worker_steps=steps, n_epochs=2)
        assert P.prsgd_iteration(h) == want["t"]
        assert rel_err(D.read_all(h), want["x"]) <= 5e-3
        P.prsgd_destroy(h)


# --------------------------------------------------------------------------- full-size shapes, as benchmarked
def test_c2_full_horizon(P, D):
    # the benchmark's default workload at its full T = 2000, I = 16 (epoch kernel, 125 restarts)
    w = get_workload("c2")
    inp = make_inputs(w)
    h = _open(D, w, inp)
    P.prsgd_run(h, w.iterations, w.interval)
    want = oracle_run(w, inp)
    got = D.read_all(h)
    assert rel_err(got, want["x"]) <= T_STEP_TOL
    assert np.array_equal(got[0], got[-1])              # I | T: the run ends on a restart
    assert np.allclose(P.prsgd_read_loss(h), want["losses"], rtol=5e-2, atol=1e-5)
    P.prsgd_destroy(h)


@pytest.mark.parametrize("interval", [1, 8])
def test_c4_full_shape_long_run(P, D, interval):
    w = get_workload("c4").scaled(iterations=1000, rows_per_worker=1024)
    inp = make_inputs(w)
    h = _open(D, w, inp)
    P.prsgd_run(h, w.iterations, interval)
    want = oracle_run(w, inp, interval=interval)
    assert rel_err(D.read_all(h), want["x"]) <= T_STEP_TOL
    P.prsgd_destroy(h)


@pytest.mark.parametrize("name,iters,interval", [("c3", 4, 2), ("c5", 2, 2), ("c3", 4, 1), ("c5", 3, 1)])
def test_bf16_full_size_replicas(P, D, name, iters, interval):
    # full layer sizes, worker count and batch (the launch shapes the benchmark times) with a
    # restart every second step, or every step (I = 1: the one-pass form); a short horizon and a smaller shard keep the fp64 oracle to
    # seconds (the configurations' own intervals and shards: tests/test_gpu_horizons.py)
    w = get_workload(name).scaled(rows_per_worker=512, iterations=iters, interval=interval)
    inp = make_inputs(w)
    h = _open(D, w, inp)
    log = []
    want = oracle_run(w, inp, record=log.append)
    for rec in log:
        P.prsgd_run(h, 1, w.interval)
        got = P.prsgd_read_loss(h)
        assert _bf16_loss_ok(got, rec["losses"]), (rec["t"], got, rec["losses"])
    # sampled replicas, every parameter
    for i in (0, w.n_workers - 1):
        assert rel_err(P.prsgd_read_params(h, i), want["x"][i]) <= 5e-3
    xbar = P.prsgd_read_params(h, -1)
    assert rel_err(xbar, oracle.node_average(want["x"])) <= 5e-3
    P.prsgd_destroy(h)


@pytest.mark.parametrize("name", ["c3", "c5"])
def test_first_layer_pass_at_full_size_matches_the_separate_launches(P, D, name):
    # the launch shapes the benchmark times (c5: non-temporal weight traffic, 128-row minibatches;
    # c3: 64-row minibatches, 16 replicas): fused and separate forms agree bit for bit
    w = get_workload(name).scaled(rows_per_worker=256, iterations=5, interval=3)
    inp = make_inputs(w)
    outs = []
    for on in (True, False):
        h = _open(D, w, inp)
        P.prsgd_set_first_layer_fusion(h, on)
        names = _kernel_names(P, h, w.iterations, w.interval)
        assert ("gemm_bwd_first" in names) == on, names
        outs.append((P.prsgd_read_params(h, 0), P.prsgd_read_params(h, w.n_workers - 1), P.prsgd_read_loss(h)))
        P.prsgd_destroy(h)
    for a, b in zip(outs[0], outs[1]):
        assert np.array_equal(a, b)


# --------------------------------------------------------------------------- restart average
@pytest.mark.parametrize("n_workers", [1, 2, 3, 8, 19, 64])
def test_restart_average_properties(P, D, n_workers):
    w = small_mlp(n_workers=n_workers, dims=(50, 30, 10), batch=4)
    inp = inputs_for(w)
    h = _open(D, w, inp)
    rng = np.random.default_rng(n_workers)
    xs = rng.standard_normal((n_workers, h.m)).astype(np.float32)
    for i in range(n_workers):
        P.prsgd_write_params(h, i, xs[i])
    assert np.array_equal(D.read_all(h), xs)
    want = oracle.node_average(xs.astype(np.float64))
    xbar = P.prsgd_read_params(h, -1)                  # eq. (4), replicas untouched
    assert np.array_equal(D.read_all(h), xs)
    P.prsgd_average(h)
    got = D.read_all(h)
    for i in range(n_workers):
        assert np.array_equal(got[i], got[0])          # replicas bit-equal after a restart
    assert np.array_equal(got[0], xbar)
    assert np.abs(got[0] - want).max() <= 2e-7 * n_workers * np.abs(xs).max()
    # sum_i x_i is preserved (to fp32 rounding of the mean)
    assert np.abs(got.astype(np.float64).sum(0) - xs.astype(np.float64).sum(0)).max() <= \
        4e-7 * n_workers * np.abs(xs).max() * max(1, n_workers)
    if n_workers == 1:
        assert np.array_equal(got[0], xs[0])           # N = 1: identity
    P.prsgd_destroy(h)


@pytest.mark.parametrize("name", ["c3", "c5"])
def test_eager_average_at_full_replica_sets(P, D, name):
    # the replica sets of the two bf16 configurations (269 MB / 1.74 GB of fp32 masters) select the
    # two-column averaging kernel, cached (c3) and streaming (c5); random replicas, the stand-alone
    # average + broadcast kernel, against the oracle's node average
    w = get_workload(name).scaled(rows_per_worker=64, batch=8)
    inp = make_inputs(w)
    h = _open(D, w, inp)
    P.prsgd_set_lazy_restart(h, False)
    rng = np.random.default_rng(5)
    xs = rng.standard_normal((w.n_workers, h.m), dtype=np.float32)
    for i in range(w.n_workers):
        P.prsgd_write_params(h, i, xs[i])
    P.prsgd_profile_enable(h, True)
    P.prsgd_average(h)
    names = {r["name"] for r in P.prsgd_profile_read(h)}
    P.prsgd_profile_enable(h, False)
    assert names == {"average"}
    want = oracle.node_average(xs.astype(np.float64))
    bound = 2e-7 * w.n_workers * np.abs(xs).max()
    for i in (0, w.n_workers // 2, w.n_workers - 1):
        got = P.prsgd_read_params(h, i)
        assert np.abs(got - want).max() <= bound
        if i == 0:
            first = got
        else:
            assert np.array_equal(got, first)                # replicas bit-equal after a restart
    # the bf16 image every replica carries is the rounded mean: one more local step from it equals
    # a step of a context initialised at the mean
    P.prsgd_local_steps(h, 1)
    after = P.prsgd_read_params(h, w.n_workers - 1)
    P.prsgd_destroy(h)
    w2 = w
    h2 = D.open_workload(w2, dict(inp, x0=first), device="cuda:0")
    P.prsgd_local_steps(h2, 1)
    assert np.array_equal(P.prsgd_read_params(h2, w.n_workers - 1), after)
    P.prsgd_destroy(h2)


LAZY_CASES = [
    ("lsq", dict()),
    ("epoch", dict(dims=(64, 32, 10), batch=8, n_workers=3)),
    ("epoch-wide", dict(dims=(784, 32, 10), batch=16, n_workers=3)),     # seven row blocks per wavefront
    ("bf16", dict(dims=(100, 72, 40, 10), batch=24, n_workers=4, gemm_dtype="bf16", activation="relu")),
    ("fp32-layers", dict(dims=(40, 24, 16, 6), batch=6, n_workers=3)),   # no deferred broadcast: falls back
]


def _lazy_workload(kind, kw):
    if kind == "lsq":
        return get_workload("c1").scaled(rows_per_worker=128, n_workers=3, iterations=9, interval=2)
    return small_mlp(rows_per_worker=128, iterations=9, interval=2, **kw)


@pytest.mark.parametrize("kind,kw", LAZY_CASES)
@pytest.mark.parametrize("interval", [1, 2])
def test_deferred_broadcast_gives_the_same_run_as_the_averaging_kernel(P, D, kind, kw, interval):
    w = _lazy_workload(kind, kw)
    inp = make_inputs(w)
    outs = []
    for lazy in (True, False):
        h = _open(D, w, inp)
        P.prsgd_set_lazy_restart(h, lazy)
        names = _kernel_names(P, h, w.iterations, interval)
        if kind != "fp32-layers":
            assert ("restart_mean" in names) == lazy and ("average" in names) == (not lazy), names
            if lazy and interval == 1:
                assert "broadcast" not in names          # the replicas are never broadcast
        xs, xbar = D.read_all(h), P.prsgd_read_params(h, -1)
        outs.append((xs, xbar, P.prsgd_read_loss(h)))
        P.prsgd_destroy(h)
    if kind == "bf16":
        # With the broadcast deferred prsgd_run takes an epoch's last iteration and the restart as one
        # pass over the node average (fewer roundings, another contraction order).  The masters differ
        # by fp32 rounding after one such pass (tests/test_gpu_interval_one.py holds that to 1e-5);
        # their bf16 images then differ by whole bf16 units here and there, so nine iterations later
        # the two runs are as far apart as each is from the oracle: the bf16 gates
        assert rel_err(outs[0][0], outs[1][0]) <= 5e-3 and rel_err(outs[0][1][None], outs[1][1][None]) <= 5e-3
        assert _bf16_loss_ok(outs[0][2], outs[1][2])
    else:
        for a, b in zip(outs[0], outs[1]):
            assert np.array_equal(a, b)
    want = oracle_run(w, inp, interval=interval)
    if kind == "bf16":
        assert _bf16_loss_ok(outs[0][2], want["losses"])
        assert rel_err(outs[0][0], want["x"]) <= 5e-3
    else:
        assert rel_err(outs[0][0], want["x"]) <= 1e-4


def test_deferred_broadcast_is_bit_identical_when_stepped_by_hand_with_bf16_operands(P, D):
    # prsgd_local_steps + prsgd_average never take the one-pass form: with or without the broadcast
    # deferred the same kernels update the replicas, and the results agree bit for bit
    w = small_mlp(dims=(256, 128, 64, 10), batch=32, n_workers=4, gemm_dtype="bf16", activation="relu",
                  rows_per_worker=128)
    inp = inputs_for(w)
    outs = []
    for lazy in (True, False):
        h = _open(D, w, inp)
        P.prsgd_set_lazy_restart(h, lazy)
        for k in (2, 1, 3):
            P.prsgd_local_steps(h, k)
            P.prsgd_average(h)
        P.prsgd_local_steps(h, 1)
        outs.append((D.read_all(h), P.prsgd_read_params(h, -1), P.prsgd_read_loss(h)))
        P.prsgd_destroy(h)
    for a, b in zip(outs[0], outs[1]):
        assert np.array_equal(a, b)


def test_state_right_after_a_deferred_restart(P, D):
    w = small_mlp(dims=(100, 72, 40, 10), batch=24, n_workers=4, gemm_dtype="bf16", activation="relu",
                  rows_per_worker=128)
    inp = inputs_for(w)
    h = _open(D, w, inp)
    P.prsgd_local_steps(h, 3)
    xbar = P.prsgd_read_params(h, -1)
    P.prsgd_average(h)
    P.prsgd_average(h)                                   # second call: nothing to do
    for i in range(w.n_workers):                         # every worker sits at the average
        assert np.array_equal(P.prsgd_read_params(h, i), xbar)
    assert np.array_equal(P.prsgd_read_params(h, -1), xbar)
    # overwriting one replica keeps the others at the restart point
    other = (xbar * np.float32(0.5)).astype(np.float32)
    P.prsgd_write_params(h, 1, other)
    got = D.read_all(h)
    assert np.array_equal(got[1], other) and np.array_equal(got[0], xbar) and np.array_equal(got[3], xbar)
    P.prsgd_destroy(h)
    # Algorithm 3 right after a deferred restart: a worker with zero steps keeps the average
    h = _open(D, w, inp)
    P.prsgd_local_steps(h, 2)
    P.prsgd_average(h)
    xbar = P.prsgd_read_params(h, -1)
    P.prsgd_local_steps_hetero(h, [2, 0, 1, 0])
    got = D.read_all(h)
    assert np.array_equal(got[1], xbar) and np.array_equal(got[3], xbar)
    assert not np.array_equal(got[0], xbar)
    P.prsgd_destroy(h)


def test_interval_one_is_minibatch_sgd_on_the_gpu(P, D):
    w = small_mlp(dims=(40, 24, 6), batch=6, n_workers=4, iterations=12, interval=1)
    inp = inputs_for(w)
    h = _open(D, w, inp)
    P.prsgd_run(h, w.iterations, 1)
    # independent loop: one SGD step on the common point with the averaged gradient
    x = inp["x0"].astype(np.float64)
    for t in range(1, w.iterations + 1):
        g = np.zeros_like(x)
        for i in range(w.n_workers):
            rows = oracle.sample_rows(w.index_seed, i, t, w.batch, w.rows_per_worker)
            g += oracle.loss_grad(w.model, x, w.dims, w.activation, inp["features"][i][rows],
                                  inp["targets"][i][rows])[1]
        x -= w.lr * g / w.n_workers
    assert rel_err(D.read_all(h), np.tile(x, (w.n_workers, 1))) <= 1e-4
    P.prsgd_destroy(h)


def test_run_not_multiple_of_interval_ends_unaveraged(P, D):
    w = small_mlp(iterations=10, interval=4)
    inp = inputs_for(w)
    h = _open(D, w, inp)
    P.prsgd_run(h, 10, 4)
    got = D.read_all(h)
    want = oracle_run(w, inp)
    assert not np.array_equal(got[0], got[1])
    assert rel_err(got, want["x"]) <= 1e-4
    assert rel_err(P.prsgd_read_params(h, -1), oracle.node_average(want["x"])) <= 1e-4
    P.prsgd_destroy(h)


# --------------------------------------------------------------------------- determinism, resume
@pytest.mark.parametrize("gemm_dtype", ["f32", "bf16"])
def test_same_seed_twice_is_bit_identical(P, D, gemm_dtype):
    w = small_mlp(dims=(200, 150, 70, 10), batch=40, gemm_dtype=gemm_dtype, activation="relu",
                  iterations=9, interval=3)
    inp = inputs_for(w)
    outs = []
    for _ in range(2):
        h = _open(D, w, inp)
        P.prsgd_run(h, w.iterations, w.interval)
        outs.append((D.read_all(h), P.prsgd_read_loss(h)))
        P.prsgd_destroy(h)
    assert np.array_equal(outs[0][0], outs[1][0])
    assert np.array_equal(outs[0][1], outs[1][1])


def test_checkpoint_resume_is_bit_identical(P, D):
    w = small_mlp(dims=(60, 40, 10), batch=8, iterations=14, interval=3)
    inp = inputs_for(w)
    h = _open(D, w, inp)
    P.prsgd_run(h, 14, 3)
    full = D.read_all(h)
    P.prsgd_destroy(h)
    h = _open(D, w, inp)
    P.prsgd_run(h, 8, 3)
    ckpt, t = D.read_all(h), P.prsgd_iteration(h)
    P.prsgd_destroy(h)
    h = _open(D, w, inp)
    for i in range(w.n_workers):
        P.prsgd_write_params(h, i, ckpt[i])
    P.prsgd_set_iteration(h, t)
    P.prsgd_run(h, 6, 3)
    assert np.array_equal(D.read_all(h), full)
    P.prsgd_destroy(h)


# --------------------------------------------------------------------------- Algorithms 2 and 3
def test_algorithm2_time_varying_rates(P, D):
    w = small_mlp(dims=(40, 24, 6), batch=6, n_workers=2)
    inp = inputs_for(w)
    ks, gs = D.time_varying_schedule(12, w.n_workers)
    gs = [0.05 * g for g in gs]                        # keep the tiny problem stable
    h = _open(D, w, inp)
    D.run_algorithm2(h, ks, gs)
    args = oracle_args(w, inp)
    args.pop("bf16")
    want = oracle.run_time_varying(**args, epoch_lengths=ks, epoch_rates=gs)
    assert P.prsgd_iteration(h) == want["t"]
    assert rel_err(D.read_all(h), want["x"]) <= 1e-4
    P.prsgd_destroy(h)


@pytest.mark.parametrize("model", ["mlp", "lsq"])
@pytest.mark.parametrize("fused", [True, False])
def test_algorithm3_heterogeneous_steps(P, D, model, fused):
    if model == "lsq":
        w = get_workload("c1").scaled(rows_per_worker=128, n_workers=4)
        steps = [6, 4, 4, 1]
    else:
        w = small_mlp(dims=(40, 24, 6), batch=6, n_workers=3)
        steps = [5, 3, 0]
    inp = make_inputs(w)
    h = _open(D, w, inp, fused_update=fused)
    D.run_algorithm3(h, steps, 3)
    args = oracle_args(w, inp)
    args.pop("bf16")
    want = oracle.run_heterogeneous(**args, lr=w.lr, worker_steps=steps, n_epochs=3)
    assert P.prsgd_iteration(h) == want["t"]
    assert rel_err(D.read_all(h), want["x"]) <= 1e-4
    P.prsgd_destroy(h)


# --------------------------------------------------------------------------- momentum local steps
MOMENTUM_CASES = [
    ("lsq", dict()),
    ("one-hidden", dict(dims=(64, 32, 10), batch=8, n_workers=3)),          # epoch kernel, prefetching variant
    ("one-hidden-wide", dict(dims=(784, 64, 10), batch=32, n_workers=2, activation="tanh")),  # no prefetch
    ("one-hidden-unfit", dict(dims=(64, 40, 10), batch=8, n_workers=3)),    # d_1 % 16 != 0: per-layer chain
    ("fp32-layers", dict(dims=(40, 24, 16, 6), batch=6, n_workers=3)),
    ("bf16", dict(dims=(100, 72, 40, 10), batch=24, n_workers=4, gemm_dtype="bf16", activation="relu")),
    ("bf16-wide", dict(dims=(200, 136, 10), batch=100, n_workers=2, gemm_dtype="bf16", activation="relu")),
    ("bf16-unfit", dict(dims=(60, 40, 10), batch=160, n_workers=2, gemm_dtype="bf16", activation="relu")),
]
# which kernel applies the momentum update
MOMENTUM_KERNEL = {"one-hidden": "mlp2_epoch", "one-hidden-wide": "mlp2_epoch", "one-hidden-unfit": "sgd_update",
                   "fp32-layers": "sgd_update", "bf16": "gemm_bwd", "bf16-wide": "gemm_bwd",
                   "bf16-unfit": "sgd_update"}


@pytest.mark.parametrize("kind,kw", MOMENTUM_CASES)
@pytest.mark.parametrize("mode", ["keep", "average", "reset"])
def test_momentum_local_steps(P, D, kind, kw, mode):
    if kind == "lsq":
        w = get_workload("c1").scaled(rows_per_worker=128, n_workers=3, iterations=9, interval=2,
                                      momentum=0.9, momentum_restart=mode)
    else:
        w = small_mlp(rows_per_worker=128, iterations=9, interval=2, lr=0.01, **kw)
        w = w.scaled(momentum=0.9, momentum_restart=mode)
    inp = make_inputs(w)
    h = _open(D, w, inp)
    names = _kernel_names(P, h, w.iterations, w.interval)
    if kind != "lsq":
        others = {"sgd_update", "mlp2_epoch", "gemm_bwd"} - {MOMENTUM_KERNEL[kind]}
        if mode == "reset":
            others.discard("sgd_update")                # the velocity reset is booked under this label
        assert MOMENTUM_KERNEL[kind] in names and not (others & set(names)), names
    want = oracle.run_prsgd(**oracle_args(w, inp), lr=w.lr, interval=w.interval, iterations=w.iterations,
                            momentum=w.momentum, momentum_restart=mode)
    got_x = D.read_all(h)
    got_v = np.stack([P.prsgd_read_velocity(h, i) for i in range(w.n_workers)])
    if kind.startswith("bf16"):
        assert _bf16_loss_ok(P.prsgd_read_loss(h), want["losses"])
        assert rel_err(got_x, want["x"]) <= 5e-3
        # right after a reset the velocity is one or two raw gradients: a hidden pre-activation
        # that fp32 accumulation puts on the other side of zero switches one sample's share of a
        # dW column on or off (ReLU'), up to 1/B of that column (B = 100 in the widest case)
        assert rel_err(got_v, want["v"]) <= 2e-2
    else:
        assert rel_err(got_x, want["x"]) <= 1e-4
        assert rel_err(got_v, want["v"]) <= 1e-4
    P.prsgd_destroy(h)


@pytest.mark.parametrize("kind,kw", [c for c in MOMENTUM_CASES if c[0] in ("lsq", "one-hidden", "bf16")])
def test_momentum_deferred_broadcast_is_bit_identical(P, D, kind, kw):
    if kind == "lsq":
        w = get_workload("c1").scaled(rows_per_worker=128, n_workers=3, iterations=9, interval=2)
    else:
        w = small_mlp(rows_per_worker=128, iterations=9, interval=2, lr=0.01, **kw)
    w = w.scaled(momentum=0.9, momentum_restart="average")
    inp = make_inputs(w)
    outs = []
    for lazy in (True, False):
        h = _open(D, w, inp)
        P.prsgd_set_lazy_restart(h, lazy)
        names = _kernel_names(P, h, w.iterations, w.interval)
        assert ("restart_mean" in names) == lazy, names
        outs.append((D.read_all(h), np.stack([P.prsgd_read_velocity(h, i) for i in range(w.n_workers)])))
        P.prsgd_destroy(h)
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])


def test_momentum_checkpoint_resume_and_errors(P, D):
    w = small_mlp(dims=(40, 24, 16, 6), batch=6, n_workers=3, iterations=14, interval=3)
    w = w.scaled(momentum=0.9)
    inp = inputs_for(w)
    h = _open(D, w, inp)
    P.prsgd_run(h, 14, 3)
    full_x = D.read_all(h)
    full_v = np.stack([P.prsgd_read_velocity(h, i) for i in range(w.n_workers)])
    with pytest.raises(P.PrsgdError):                   # Algorithm 3 is not defined with momentum
        P.prsgd_local_steps_hetero(h, [1, 1, 1])
    P.prsgd_destroy(h)
    h = _open(D, w, inp)
    P.prsgd_run(h, 8, 3)
    ck_x, t = D.read_all(h), P.prsgd_iteration(h)
    ck_v = [P.prsgd_read_velocity(h, i) for i in range(w.n_workers)]
    P.prsgd_destroy(h)
    h = _open(D, w, inp)
    for i in range(w.n_workers):
        P.prsgd_write_params(h, i, ck_x[i])
        P.prsgd_write_velocity(h, i, ck_v[i])
    P.prsgd_set_iteration(h, t)
    P.prsgd_run(h, 6, 3)
    assert np.array_equal(D.read_all(h), full_x)
    assert np.array_equal(np.stack([P.prsgd_read_velocity(h, i) for i in range(w.n_workers)]), full_v)
    P.prsgd_destroy(h)
    # no momentum buffers without momentum
    w0 = small_mlp()
    h = _open(D, w0, inputs_for(w0))
    with pytest.raises(P.PrsgdError):
        P.prsgd_read_velocity(h, 0)
    P.prsgd_destroy(h)


# --------------------------------------------------------------------------- stand-alone update
# 2^26 and 2^28 elements select the streaming (non-temporal) variant of the kernel
@pytest.mark.parametrize("count", [4, 1000, 4099, 1 << 20, (1 << 26) + 3, 1 << 28])
def test_standalone_sgd_update(P, count):
    rng = np.random.default_rng(count % 1000003)
    x = rng.standard_normal(count, dtype=np.float32)
    g = rng.standard_normal(count, dtype=np.float32)
    xd, gd = torch.from_numpy(x).cuda(), torch.from_numpy(g).cuda()
    sh = torch.zeros(count, dtype=torch.bfloat16, device="cuda")
    P.prsgd_sgd_update(xd, gd, 0.05, shadow=sh)
    torch.cuda.synchronize()
    got = xd.cpu().numpy()
    got_sh = sh.float().cpu().numpy()
    del xd, gd, sh
    # eq. (3) in float64 on the same float32 inputs; the kernel rounds once (fused multiply-add)
    lr = np.float64(np.float32(0.05))
    block = 1 << 24                                     # bounded host memory at the large counts
    for lo in range(0, count, block):
        hi = min(count, lo + block)
        want = x[lo:hi].astype(np.float64) - lr * g[lo:hi].astype(np.float64)
        assert np.abs(got[lo:hi] - want).max() <= 1e-7 * max(1.0, np.abs(want).max())
        assert np.array_equal(got_sh[lo:hi], oracle.round_bf16(got[lo:hi]).astype(np.float32))


def test_bf16_shadow_keeps_nan_and_infinity(P):
    # a diverged master must not read as a finite weight in its bf16 image
    pats = np.array([0x7F800001, 0x7FFFFFFF, 0xFFFFFFFF, 0x7FC00000, 0x7F800000, 0xFF800000,
                     0x7F7FFFFF, 0x3F808000], dtype=np.uint32).view(np.float32)
    xd = torch.from_numpy(pats.copy()).cuda()
    gd = torch.zeros(pats.size, dtype=torch.float32, device="cuda")
    sh = torch.zeros(pats.size, dtype=torch.bfloat16, device="cuda")
    P.prsgd_sgd_update(xd, gd, 0.0, shadow=sh)
    torch.cuda.synchronize()
    got = sh.float().cpu().numpy()
    want = oracle.round_bf16(pats).astype(np.float32)
    assert np.all(np.isnan(got[:4])) and np.all(np.isnan(want[:4]))
    assert np.array_equal(got[4:], want[4:])
    assert got[6] == np.inf                              # the largest float rounds up to infinity


# --------------------------------------------------------------------------- errors with a live context
def test_argument_errors_leave_the_context_usable(P, D):
    w = small_mlp()
    inp = inputs_for(w)
    h = _open(D, w, inp)
    with pytest.raises(P.PrsgdError):
        P.prsgd_local_steps(h, -1)
    with pytest.raises(P.PrsgdError):
        P.prsgd_read_params(h, w.n_workers)
    with pytest.raises(P.PrsgdError):
        P.prsgd_run(h, 4, 0)
    assert "interval" in P.prsgd_last_error(h)
    P.prsgd_local_steps(h, 0)
    assert P.prsgd_iteration(h) == 0
    assert np.array_equal(P.prsgd_read_params(h, 0), inp["x0"])
    P.prsgd_destroy(h)


# --------------------------------------------------------------------------- epoch kernel: the give-up path
def test_epoch_kernel_give_up_is_reported_and_the_context_falls_back(P, D):
    # Driven from the host: with a wait limit of zero polls the first team member to reach the
    # team barrier gives up at once (eight members per team: they never all arrive before the first
    # one's first poll).  Every kernel still runs to its end.
    w = small_mlp(dims=(64, 128, 10), batch=8, n_workers=8, rows_per_worker=128, interval=4, iterations=10,
                  activation="tanh")
    inp = inputs_for(w)
    h = _open(D, w, inp)
    P.prsgd_local_steps(h, 2)
    P.prsgd_status(h)                                     # nothing gave up
    good = D.read_all(h)
    P.prsgd_set_epoch_wait_limit(h, 0)
    P.prsgd_local_steps(h, 4)                             # asynchronous: returns before the kernel ends
    with pytest.raises(P.PrsgdError) as err:
        P.prsgd_status(h)
    assert err.value.code == P.PRSGD_ESTATE and "gave up" in str(err.value)
    for call in (lambda: P.prsgd_local_steps(h, 1), lambda: P.prsgd_average(h), lambda: P.prsgd_run(h, 2, 2),
                 lambda: P.prsgd_read_params(h, 0), lambda: P.prsgd_read_loss(h), lambda: P.prsgd_status(h)):
        with pytest.raises(P.PrsgdError) as err:
            call()
        assert err.value.code == P.PRSGD_ESTATE
    # restore the last good state; the context is usable again and runs the per-layer chain
    for i in range(w.n_workers):
        P.prsgd_write_params(h, i, good[i])
    P.prsgd_set_iteration(h, 2)
    P.prsgd_status(h)
    names = _kernel_names(P, h, w.iterations - 2, w.interval)
    assert "gemm_fwd" in names and "mlp2_epoch" not in names, names
    want = oracle_run(w, inp)
    assert rel_err(D.read_all(h), want["x"]) <= 1e-4
    P.prsgd_destroy(h)
