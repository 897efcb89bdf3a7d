"""Thin ctypes binding of libprsgd (argument marshalling only).

Every function mirrors one entry point of include/prsgd.h (or include/prsgd_aux.h, the
measurement and test aids) under the same name.  PyTorch is
used for device memory (the replica buffer and the workspace are torch tensors) and for the
HIP stream; all arithmetic of the method runs in the library's kernels.  There is no CPU
fallback: importing this module without a built libprsgd.so raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libprsgd.so")

PRSGD_OK, PRSGD_EINVAL, PRSGD_ESTATE, PRSGD_EHIP, PRSGD_ENOMEM = 0, -1, -2, -3, -4
PRSGD_LSQ, PRSGD_MLP = 0, 1
PRSGD_TANH, PRSGD_RELU = 0, 1
PRSGD_F32, PRSGD_BF16 = 0, 1
PRSGD_MOM_KEEP, PRSGD_MOM_AVERAGE, PRSGD_MOM_RESET = 0, 1, 2
PRSGD_MAX_DIMS = 16


class PrsgdError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__("prsgd error %d: %s" % (code, message))
        self.code = code


class prsgd_config(ctypes.Structure):
    _fields_ = [
        ("n_workers", ctypes.c_int32),
        ("model", ctypes.c_int32),
        ("n_dims", ctypes.c_int32),
        ("dims", ctypes.c_int32 * PRSGD_MAX_DIMS),
        ("activation", ctypes.c_int32),
        ("gemm_dtype", ctypes.c_int32),
        ("batch", ctypes.c_int32),
        ("fused_update", ctypes.c_int32),
        ("rows_per_worker", ctypes.c_int64),
        ("lr", ctypes.c_float),
        ("seed", ctypes.c_uint64),
        ("momentum", ctypes.c_float),
        ("momentum_restart", ctypes.c_int32),
    ]


class prsgd_kernel_stat(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 48), ("launches", ctypes.c_int64),
                ("total_ms", ctypes.c_double)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError("libprsgd.so is not built; run `python -m paper_1807_06629_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    cfgp = ctypes.POINTER(prsgd_config)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    sigs = {
        "prsgd_param_count": (sz, [cfgp]),
        "prsgd_param_stride": (sz, [cfgp]),
        "prsgd_workspace_bytes": (sz, [cfgp]),
        "prsgd_init": (ctypes.c_int, [cfgp, vp, vp, vp, vp, vp, vp, ctypes.POINTER(vp)]),
        "prsgd_init_static": (ctypes.c_int, [cfgp, vp, vp, vp, vp, vp, ctypes.POINTER(vp)]),
        "prsgd_local_steps": (ctypes.c_int, [vp, i32]),
        "prsgd_local_steps_hetero": (ctypes.c_int, [vp, vp]),
        "prsgd_average": (ctypes.c_int, [vp]),
        "prsgd_set_lazy_restart": (ctypes.c_int, [vp, i32]),
        "prsgd_run": (ctypes.c_int, [vp, i64, i32]),
        "prsgd_read_params": (ctypes.c_int, [vp, i32, vp, sz]),
        "prsgd_write_params": (ctypes.c_int, [vp, i32, vp, sz]),
        "prsgd_read_velocity": (ctypes.c_int, [vp, i32, vp, sz]),
        "prsgd_write_velocity": (ctypes.c_int, [vp, i32, vp, sz]),
        "prsgd_read_loss": (ctypes.c_int, [vp, vp]),
        "prsgd_read_indices": (ctypes.c_int, [vp, vp]),
        "prsgd_sample_indices": (ctypes.c_int, [ctypes.c_uint64, i32, i32, i64, i64, i32, vp, vp]),
        "prsgd_sgd_update": (ctypes.c_int, [vp, vp, vp, sz, ctypes.c_float, vp]),
        "prsgd_copy_bytes": (ctypes.c_int, [vp, vp, sz, vp]),
        "prsgd_time_varying_schedule": (ctypes.c_int, [i32, i32, vp, vp]),
        "prsgd_status": (ctypes.c_int, [vp]),
        "prsgd_set_epoch_wait_limit": (ctypes.c_int, [vp, ctypes.c_uint32]),
        "prsgd_set_first_layer_fusion": (ctypes.c_int, [vp, i32]),
        "prsgd_set_restart_fusion": (ctypes.c_int, [vp, i32]),
        "prsgd_set_lr": (ctypes.c_int, [vp, ctypes.c_float]),
        "prsgd_set_iteration": (ctypes.c_int, [vp, i64]),
        "prsgd_iteration": (i64, [vp]),
        "prsgd_profile_enable": (ctypes.c_int, [vp, i32]),
        "prsgd_profile_read": (ctypes.c_int, [vp, ctypes.POINTER(prsgd_kernel_stat), i32]),
        "prsgd_destroy": (ctypes.c_int, [vp]),
        "prsgd_last_error": (ctypes.c_char_p, [vp]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


_lib = _load()


def make_config(n_workers: int, model: str, dims: Sequence[int], batch: int, rows_per_worker: int,
                lr: float, seed: int, activation: str = "relu", gemm_dtype: str = "f32",
                fused_update: bool = True, momentum: float = 0.0,
                momentum_restart: str = "keep") -> prsgd_config:
    c = prsgd_config()
    c.n_workers = int(n_workers)
    c.model = {"lsq": PRSGD_LSQ, "mlp": PRSGD_MLP}[model]
    c.n_dims = len(dims)
    if len(dims) > PRSGD_MAX_DIMS:
        raise ValueError("too many dims")
    for k, d in enumerate(dims):
        c.dims[k] = int(d)
    c.activation = {"tanh": PRSGD_TANH, "relu": PRSGD_RELU, "none": PRSGD_RELU}[activation]
    c.gemm_dtype = {"f32": PRSGD_F32, "bf16": PRSGD_BF16}[gemm_dtype]
    c.batch = int(batch)
    c.fused_update = 1 if fused_update else 0
    c.rows_per_worker = int(rows_per_worker)
    c.lr = float(lr)
    c.seed = int(seed)
    c.momentum = float(momentum)
    c.momentum_restart = {"keep": PRSGD_MOM_KEEP, "average": PRSGD_MOM_AVERAGE,
                          "reset": PRSGD_MOM_RESET}[momentum_restart]
    return c


@dataclass
class Handle:
    """A live context plus the torch tensors it borrows (kept alive here)."""
    ctx: ctypes.c_void_p
    cfg: prsgd_config
    m: int
    stride: int
    params: torch.Tensor
    workspace: Optional[torch.Tensor]
    features: torch.Tensor
    targets: torch.Tensor
    stream: torch.cuda.Stream


def _check(rc: int, ctx=None):
    if rc != PRSGD_OK:
        msg = _lib.prsgd_last_error(ctx)
        raise PrsgdError(rc, msg.decode() if msg else "")


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    return 0 if stream is None else int(stream.cuda_stream)


def prsgd_param_count(cfg: prsgd_config) -> int:
    return int(_lib.prsgd_param_count(ctypes.byref(cfg)))


def prsgd_param_stride(cfg: prsgd_config) -> int:
    return int(_lib.prsgd_param_stride(ctypes.byref(cfg)))


def prsgd_workspace_bytes(cfg: prsgd_config) -> int:
    return int(_lib.prsgd_workspace_bytes(ctypes.byref(cfg)))


def _init(cfg: prsgd_config, x0: np.ndarray, features: torch.Tensor, targets: torch.Tensor,
          stream: Optional[torch.cuda.Stream], static: bool) -> Handle:
    m = prsgd_param_count(cfg)
    if m == 0:
        _lib.prsgd_init(ctypes.byref(cfg), None, None, None, None, None, None,
                        ctypes.byref(ctypes.c_void_p()))
        raise PrsgdError(PRSGD_EINVAL, _lib.prsgd_last_error(None).decode())
    if not (features.is_cuda and targets.is_cuda):
        raise ValueError("features and targets must be device tensors")
    if features.dtype != torch.float32 or not features.is_contiguous() or not targets.is_contiguous():
        raise ValueError("features must be contiguous float32; targets contiguous")
    want_t = torch.float32 if cfg.model == PRSGD_LSQ else torch.int32
    if targets.dtype != want_t:
        raise ValueError("targets must be %s" % want_t)
    n = cfg.n_workers
    if tuple(features.shape) != (n, cfg.rows_per_worker, cfg.dims[0]) or \
            tuple(targets.shape) != (n, cfg.rows_per_worker):
        raise ValueError("features must be [N][n][d0] and targets [N][n]")
    x0 = np.ascontiguousarray(x0, dtype=np.float32)
    if x0.shape != (m,):
        raise ValueError("x0 must have %d elements" % m)
    dev = features.device
    if stream is None:
        stream = torch.cuda.current_stream(dev)
    stride = prsgd_param_stride(cfg)
    params = torch.empty(n * stride, dtype=torch.float32, device=dev)
    ctx = ctypes.c_void_p()
    with torch.cuda.device(dev):
        if static:
            workspace = None
            rc = _lib.prsgd_init_static(ctypes.byref(cfg), x0.ctypes.data, features.data_ptr(),
                                        targets.data_ptr(), params.data_ptr(), _stream_ptr(stream),
                                        ctypes.byref(ctx))
        else:
            workspace = torch.empty(max(prsgd_workspace_bytes(cfg), 256), dtype=torch.uint8, device=dev)
            rc = _lib.prsgd_init(ctypes.byref(cfg), x0.ctypes.data, features.data_ptr(), targets.data_ptr(),
                                 params.data_ptr(), workspace.data_ptr(), _stream_ptr(stream),
                                 ctypes.byref(ctx))
    _check(rc, None)
    return Handle(ctx, cfg, m, stride, params, workspace, features, targets, stream)


def prsgd_init(cfg: prsgd_config, x0: np.ndarray, features: torch.Tensor, targets: torch.Tensor,
               stream: Optional[torch.cuda.Stream] = None) -> Handle:
    return _init(cfg, x0, features, targets, stream, static=False)


def prsgd_init_static(cfg: prsgd_config, x0: np.ndarray, features: torch.Tensor, targets: torch.Tensor,
                      stream: Optional[torch.cuda.Stream] = None) -> Handle:
    """prsgd_init on the library's static workspace (the replica buffer is still the caller's)."""
    return _init(cfg, x0, features, targets, stream, static=True)


def prsgd_local_steps(h: Handle, k: int) -> None:
    _check(_lib.prsgd_local_steps(h.ctx, int(k)), h.ctx)


def prsgd_local_steps_hetero(h: Handle, steps: Sequence[int]) -> None:
    arr = np.ascontiguousarray(steps, dtype=np.int32)
    if arr.shape != (h.cfg.n_workers,):
        raise ValueError("one step count per worker")
    _check(_lib.prsgd_local_steps_hetero(h.ctx, arr.ctypes.data), h.ctx)


def prsgd_average(h: Handle) -> None:
    _check(_lib.prsgd_average(h.ctx), h.ctx)


def prsgd_set_lazy_restart(h: Handle, on: bool) -> None:
    _check(_lib.prsgd_set_lazy_restart(h.ctx, 1 if on else 0), h.ctx)


def prsgd_run(h: Handle, iterations: int, interval: int) -> None:
    _check(_lib.prsgd_run(h.ctx, int(iterations), int(interval)), h.ctx)


def prsgd_read_params(h: Handle, worker: int) -> np.ndarray:
    out = np.empty(h.m, dtype=np.float32)
    _check(_lib.prsgd_read_params(h.ctx, int(worker), out.ctypes.data, h.m), h.ctx)
    return out


def prsgd_write_params(h: Handle, worker: int, x: np.ndarray) -> None:
    x = np.ascontiguousarray(x, dtype=np.float32)
    _check(_lib.prsgd_write_params(h.ctx, int(worker), x.ctypes.data, x.size), h.ctx)


def prsgd_read_velocity(h: Handle, worker: int) -> np.ndarray:
    out = np.empty(h.m, dtype=np.float32)
    _check(_lib.prsgd_read_velocity(h.ctx, int(worker), out.ctypes.data, out.size), h.ctx)
    return out


def prsgd_write_velocity(h: Handle, worker: int, v: np.ndarray) -> None:
    v = np.ascontiguousarray(v, dtype=np.float32)
    _check(_lib.prsgd_write_velocity(h.ctx, int(worker), v.ctypes.data, v.size), h.ctx)


def prsgd_read_loss(h: Handle) -> np.ndarray:
    out = np.empty(h.cfg.n_workers, dtype=np.float32)
    _check(_lib.prsgd_read_loss(h.ctx, out.ctypes.data), h.ctx)
    return out


def prsgd_read_indices(h: Handle) -> np.ndarray:
    out = np.empty((h.cfg.n_workers, h.cfg.batch), dtype=np.int32)
    _check(_lib.prsgd_read_indices(h.ctx, out.ctypes.data), h.ctx)
    return out


def prsgd_sample_indices(seed: int, n_workers: int, batch: int, rows_per_worker: int, t_first: int,
                         n_steps: int, device="cuda:0") -> torch.Tensor:
    out = torch.empty((n_steps, n_workers, batch), dtype=torch.int32, device=device)
    with torch.cuda.device(out.device):
        s = torch.cuda.current_stream(out.device)
        _check(_lib.prsgd_sample_indices(int(seed), int(n_workers), int(batch), int(rows_per_worker),
                                         int(t_first), int(n_steps), out.data_ptr(), _stream_ptr(s)))
    return out


def prsgd_sgd_update(x: torch.Tensor, g: torch.Tensor, lr: float,
                     shadow: Optional[torch.Tensor] = None) -> None:
    if x.dtype != torch.float32 or g.dtype != torch.float32 or x.numel() != g.numel():
        raise ValueError("x and g must be float32 tensors of equal size")
    if not (x.is_cuda and g.is_cuda and x.is_contiguous() and g.is_contiguous()):
        raise ValueError("x and g must be contiguous device tensors")
    sp = 0
    if shadow is not None:
        if shadow.dtype != torch.bfloat16 or shadow.numel() != x.numel() or not shadow.is_cuda:
            raise ValueError("shadow must be a bfloat16 device tensor of the same size")
        sp = shadow.data_ptr()
    with torch.cuda.device(x.device):
        s = torch.cuda.current_stream(x.device)
        _check(_lib.prsgd_sgd_update(x.data_ptr(), g.data_ptr(), sp, x.numel(), float(lr),
                                     _stream_ptr(s)))


def prsgd_copy_bytes(dst: torch.Tensor, src: torch.Tensor) -> None:
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes or not (dst.is_cuda and src.is_cuda):
        raise ValueError("dst and src must be device tensors of equal byte size")
    with torch.cuda.device(src.device):
        s = torch.cuda.current_stream(src.device)
        _check(_lib.prsgd_copy_bytes(dst.data_ptr(), src.data_ptr(), nbytes, _stream_ptr(s)))


def prsgd_time_varying_schedule(n_epochs: int, n_workers: int):
    """(K^s, gamma^s) for s = 1..n_epochs as int32 / float32 arrays."""
    ks = np.empty(max(n_epochs, 0), dtype=np.int32)
    gs = np.empty(max(n_epochs, 0), dtype=np.float32)
    _check(_lib.prsgd_time_varying_schedule(int(n_epochs), int(n_workers), ks.ctypes.data, gs.ctypes.data))
    return ks, gs


def prsgd_status(h: Handle) -> None:
    _check(_lib.prsgd_status(h.ctx), h.ctx)


def prsgd_set_epoch_wait_limit(h: Handle, polls: int) -> None:
    _check(_lib.prsgd_set_epoch_wait_limit(h.ctx, int(polls)), h.ctx)


def prsgd_set_restart_fusion(h: Handle, on: bool) -> None:
    _check(_lib.prsgd_set_restart_fusion(h.ctx, 1 if on else 0), h.ctx)


def prsgd_set_first_layer_fusion(h: Handle, on: bool) -> None:
    _check(_lib.prsgd_set_first_layer_fusion(h.ctx, 1 if on else 0), h.ctx)


def prsgd_set_lr(h: Handle, lr: float) -> None:
    _check(_lib.prsgd_set_lr(h.ctx, float(lr)), h.ctx)


def prsgd_set_iteration(h: Handle, t: int) -> None:
    _check(_lib.prsgd_set_iteration(h.ctx, int(t)), h.ctx)


def prsgd_iteration(h: Handle) -> int:
    return int(_lib.prsgd_iteration(h.ctx))


def prsgd_profile_enable(h: Handle, on: bool) -> None:
    _check(_lib.prsgd_profile_enable(h.ctx, 1 if on else 0), h.ctx)


def prsgd_profile_read(h: Handle) -> List[dict]:
    buf = (prsgd_kernel_stat * 16)()
    n = _lib.prsgd_profile_read(h.ctx, buf, 16)
    if n < 0:
        _check(n, h.ctx)
    return [{"name": buf[k].name.decode(), "launches": int(buf[k].launches),
             "total_ms": float(buf[k].total_ms)} for k in range(min(n, 16))]


def prsgd_destroy(h: Handle) -> None:
    if h.ctx:
        rc = _lib.prsgd_destroy(h.ctx)
        h.ctx = None
        if rc != PRSGD_OK:
            raise PrsgdError(rc, "prsgd_destroy failed")


def prsgd_last_error(h: Optional[Handle]) -> str:
    msg = _lib.prsgd_last_error(h.ctx if h is not None else None)
    return msg.decode() if msg else ""
