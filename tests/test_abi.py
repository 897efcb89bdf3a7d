"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, sizes its buffers as documented and rejects bad configurations."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def P():
    lib = os.path.join(ROOT, "paper_1807_06629_amd", "libprsgd.so")
    if not os.path.exists(lib):
        from paper_1807_06629_amd.build import build
        build()
    from paper_1807_06629_amd import prsgd
    return prsgd


def _declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for header in sorted(os.listdir(inc)):
        if not header.endswith(".h"):
            continue
        text = open(os.path.join(inc, header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(prsgd_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol(P):
    names = _declared_functions()
    assert {"prsgd_init", "prsgd_local_steps", "prsgd_average", "prsgd_read_params"} <= set(names)
    lib = ctypes.CDLL(P.LIB_PATH)
    for name in names:
        assert hasattr(lib, name), name
    # and the binding mirrors each of them under the same name
    for name in names:
        assert hasattr(P, name), name


def test_parameter_counts_match_the_closed_form(P):
    c2 = P.make_config(8, "mlp", (784, 256, 10), 32, 8192, 0.05, 3, "tanh")
    assert P.prsgd_param_count(c2) == 784 * 256 + 256 + 256 * 10 + 10 == 203530
    c5 = P.make_config(8, "mlp", (4096, 4096, 4096, 4096, 1000), 128, 8192, 0.01, 3, "relu", "bf16")
    assert P.prsgd_param_count(c5) == 54440936
    c1 = P.make_config(4, "lsq", (64,), 16, 4096, 0.01, 3)
    assert P.prsgd_param_count(c1) == 64
    for c in (c1, c2, c5):
        stride = P.prsgd_param_stride(c)
        assert stride >= P.prsgd_param_count(c) and stride % 64 == 0
        assert P.prsgd_workspace_bytes(c) % 256 == 0 and P.prsgd_workspace_bytes(c) > 0


def test_workspace_grows_with_shadow_and_gradient_buffers(P):
    # two hidden layers: no epoch-kernel buffers, so the only differences are the ones named
    dims = (64, 32, 24, 10)
    f32 = P.make_config(2, "mlp", dims, 8, 64, 0.1, 1, "relu", "f32", True)
    bf = P.make_config(2, "mlp", dims, 8, 64, 0.1, 1, "relu", "bf16", True)
    unf = P.make_config(2, "mlp", dims, 8, 64, 0.1, 1, "relu", "f32", False)
    stride = P.prsgd_param_stride(f32)
    assert P.prsgd_workspace_bytes(unf) - P.prsgd_workspace_bytes(f32) >= 2 * stride * 4
    assert P.prsgd_workspace_bytes(bf) > 0


@pytest.mark.parametrize("kw", [
    dict(n_workers=0), dict(batch=0), dict(batch=5000), dict(rows_per_worker=100),
    dict(rows_per_worker=0), dict(dims=(5,)), dict(dims=(0, 4)), dict(lr=float("nan")),
    dict(momentum=1.0), dict(momentum=-0.1),
])
def test_invalid_configurations_are_rejected_without_touching_the_gpu(P, kw):
    base = dict(n_workers=2, model="mlp", dims=(8, 4), batch=4, rows_per_worker=16, lr=0.1, seed=1)
    base.update(kw)
    cfg = P.make_config(**base)
    assert P.prsgd_param_count(cfg) == 0
    assert P.prsgd_workspace_bytes(cfg) == 0
    ctx = ctypes.c_void_p()
    rc = P._lib.prsgd_init(ctypes.byref(cfg), None, None, None, None, None, None, ctypes.byref(ctx))
    assert rc == P.PRSGD_EINVAL and not ctx
    assert P.prsgd_last_error(None) != ""


def test_null_context_calls_return_einval(P):
    assert P._lib.prsgd_local_steps(None, 1) == P.PRSGD_EINVAL
    assert P._lib.prsgd_average(None) == P.PRSGD_EINVAL
    assert P._lib.prsgd_run(None, 1, 1) == P.PRSGD_EINVAL
    assert P._lib.prsgd_read_params(None, 0, None, 0) == P.PRSGD_EINVAL
    assert P._lib.prsgd_iteration(None) == -1
    assert P._lib.prsgd_destroy(None) == P.PRSGD_EINVAL


def test_theorem2_schedule_of_the_library(P):
    ks, gs = P.prsgd_time_varying_schedule(27, 2)
    assert ks[0] == 1 and ks[7] == 1 and ks[26] == 2
    assert gs[0] == 2.0 and gs[7] == pytest.approx(0.5)
    assert P._lib.prsgd_time_varying_schedule(3, 0, None, None) == P.PRSGD_EINVAL
    assert P._lib.prsgd_time_varying_schedule(3, 1, None, None) == P.PRSGD_EINVAL
    assert len(P.prsgd_time_varying_schedule(0, 4)[0]) == 0


@pytest.mark.parametrize("n_workers", [1, 2, 8])
def test_theorem2_schedule_matches_the_oracle_and_the_integer_definition(P, n_workers):
    # K^s = ceil(s^(1/3) / N): the smallest integer k with (k N)^3 >= s, checked in exact integer
    # arithmetic, against the oracle's floating-point form and against the library
    import numpy as np
    import oracle
    S = 10000
    ks, gs = P.prsgd_time_varying_schedule(S, n_workers)
    oks, ogs = oracle.time_varying_schedule(S, n_workers)
    for s in range(1, S + 1):
        k = int(ks[s - 1])
        assert (k * n_workers) ** 3 >= s and (k == 1 or ((k - 1) * n_workers) ** 3 < s), s
        assert oks[s - 1] == k, s
    assert np.allclose(gs, np.asarray(ogs), rtol=2e-7, atol=0)
    # perfect cubes are where a rounded cube root would be off by one
    for r in (2, 3, 5, 10, 21):
        s = (r * n_workers) ** 3
        if s <= S:
            assert ks[s - 1] == r and (s == S or ks[s] == r + 1)
