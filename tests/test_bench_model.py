"""bench.py's accounting of algorithmic work, pinned to closed forms of the workload shapes
(no GPU needed)."""
from __future__ import annotations

import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from workloads import get_workload  # noqa: E402


def _pw(dims):
    return sum(a * b for a, b in zip(dims[:-1], dims[1:]))


def _m(dims):
    return _pw(dims) + sum(dims[1:])


def test_flops_per_iteration_are_2B_times_3Pw_minus_first_layer():
    # forward 2 B P_w, weight gradient 2 B P_w, backward data 2 B (P_w - d0 d1), per worker
    for name, giga in (("c2", 0.209), ("c3", 19.39), ("c4", 0.071), ("c5", 300.0)):
        w = get_workload(name)
        want = 2 * w.n_workers * w.batch * (3 * _pw(w.dims) - w.dims[0] * w.dims[1])
        work = bench.algorithmic_work(w)
        got = work["gemm_fwd"]["flops"] + work["gemm_dx"]["flops"] + work["gemm_dw"]["flops"]
        assert got == want
        assert abs(got / 1e9 - giga) <= 0.01 * giga + 0.001
        assert work["gemm_bwd"]["flops"] == work["gemm_dx"]["flops"] + work["gemm_dw"]["flops"]
        assert work["mlp2_epoch"]["flops"] == want


def test_restart_average_bytes():
    for name in ("c2", "c3", "c4", "c5"):
        w = get_workload(name)
        n, m, pw = w.n_workers, _m(w.dims), _pw(w.dims)
        shadow = 2 if w.gemm_dtype == "bf16" else 0
        work = bench.algorithmic_work(w)
        assert work["average"]["bytes"] == 8 * n * m + shadow * n * pw
        assert work["restart_mean"]["bytes"] == 4 * n * m + 4 * m + shadow * pw
        assert work["sgd_update"]["bytes"] == (12 + shadow) * n * m
    c5 = bench.algorithmic_work(get_workload("c5"))
    assert abs(c5["average"]["bytes"] / 1e9 - 4.355) < 0.01        # 8 N m + 2 N P_w
    c1 = bench.algorithmic_work(get_workload("c1"))
    assert c1["average"]["bytes"] == 8 * 4 * 64


def test_fused_backward_moves_ten_bytes_per_weight_element_and_eighteen_with_momentum():
    w = get_workload("c5")
    n, b = w.n_workers, w.batch
    layers = list(zip(w.dims[:-1], w.dims[1:]))
    panels = sum(n * b * (di + do) * 2 for di, do in layers) + sum(n * b * di * 2 for di, _ in layers[1:])
    assert bench.algorithmic_work(w)["gemm_bwd"]["bytes"] == 10 * n * _pw(w.dims) + panels
    wm = w.scaled(momentum=0.9)
    assert bench.algorithmic_work(wm)["gemm_bwd"]["bytes"] == 18 * n * _pw(w.dims) + panels


def test_more_than_one_gpu_is_refused_with_a_message():
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert out.returncode != 0
    assert "one GPU" in out.stderr and out.stdout.strip() == ""


def test_traffic_table_is_keyed_by_the_kernel_sources():
    # a reading taken on other sources must not be reported
    digest = bench.kernel_source_digest()
    assert len(digest) == 64
    assert bench.measured_traffic("no-such-workload", "gemm_bwd") is None


def test_first_layer_pass_moves_eight_bytes_per_weight_element_and_takes_its_layer_out_of_the_others():
    w = get_workload("c5")
    n, b = w.n_workers, w.batch
    d0, d1 = w.dims[0], w.dims[1]
    plain, fused = bench.algorithmic_work(w), bench.algorithmic_work(w, first_fused=True)
    first = fused["gemm_bwd_first"]
    # master read + write; minibatches of both iterations, delta panel, next activation (bf16)
    assert first["bytes"] == n * (8 * d0 * d1 + 2 * b * (2 * d0 + 2 * d1))
    assert first["flops"] == 2 * (2 * n * b * d0 * d1)                 # weight gradient + next forward
    # the other labels lose exactly layer 1
    assert plain["gemm_fwd"]["flops"] - fused["gemm_fwd"]["flops"] == 2 * n * b * d0 * d1
    assert plain["gemm_bwd"]["flops"] - fused["gemm_bwd"]["flops"] == 2 * n * b * d0 * d1
    assert plain["gemm_bwd"]["bytes"] - fused["gemm_bwd"]["bytes"] == n * (10 * d0 * d1 + 2 * b * (d0 + d1))
    # per weight element and iteration: 12 B for layers 2..L, 8 B for layer 1 (weights only)
    pw_rest = _pw(w.dims) - d0 * d1
    weights_only = 8 * n * d0 * d1 + 12 * n * pw_rest
    assert abs(weights_only / 1e9 - 4.688) < 0.005


def test_stacked_product_of_the_epoch_closing_pass():
    w = get_workload("c5")
    n, b = w.n_workers, w.batch
    work = bench.algorithmic_work(w, shared_weights=True)
    panels = sum(n * b * (di + do) * 2 for di, do in zip(w.dims[:-1], w.dims[1:]))
    # the node average read and written once, its bf16 image written once, every panel read once
    assert work["step_mean"]["bytes"] == 8 * _m(w.dims) + 2 * _pw(w.dims) + panels
    assert work["step_mean"]["flops"] == 2 * n * b * _pw(w.dims)
    # shared weights: the forward products read one weight matrix per layer, not one per worker
    assert bench.algorithmic_work(w)["gemm_fwd"]["bytes"] - work["gemm_fwd"]["bytes"] == 2 * (n - 1) * _pw(w.dims)
