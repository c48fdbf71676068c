"""ctypes binding of libpowergossip.so: the same names as ``include/powergossip.h``,
argument marshalling only.  Every step of a round runs in the library's HIP kernels;
there is no CPU fallback -- a missing library is an ImportError."""
from __future__ import annotations

import ctypes
import os
from typing import Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpowergossip.so")

PG_OK, PG_ERR_ARG, PG_ERR_TOPOLOGY, PG_ERR_SHAPE, PG_ERR_NOMEM, PG_ERR_DEVICE, PG_ERR_TOO_LARGE = 0, -1, -2, -3, -4, -5, -6
PG_STATIC_WORKSPACE_BYTES = 32 << 20

EXPORTS = [
    "pg_strerror", "pg_init", "pg_destroy", "pg_param_floats", "pg_layer_offset", "pg_layer_stride", "pg_layer_rank",
    "pg_qstate_floats", "pg_q_offset", "pg_workspace_bytes", "pg_ws_phat_offset",
    "pg_ws_flag_offset", "pg_message_floats", "pg_round_bytes", "pg_upload", "pg_round", "pg_round_static", "pg_round_sgd",
    "pg_run", "pg_iterate", "pg_pstate_floats", "pg_p_offset",
    "pg_profile_enable", "pg_profile_collect",
]


class pg_kernel_time(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 32), ("launches", ctypes.c_int),
                ("ms", ctypes.c_double), ("bytes", ctypes.c_double)]


def _share_hip_runtime_with_torch():
    """One HIP runtime per process.  PyTorch wheels bundle their own libamdhip64 (same soname
    as the system copy this library is linked against).  Loaded after torch, the library binds
    to the copy torch already mapped; loaded first, it would map the system copy, torch would
    later map its own, and whichever runtime initialises second finds no device.  Mapping
    torch's copy first (without importing torch) makes the order irrelevant."""
    import importlib.util
    try:
        spec = importlib.util.find_spec("torch")
    except (ImportError, ValueError):
        spec = None
    if spec is None or not spec.submodule_search_locations:
        return
    bundled = os.path.join(list(spec.submodule_search_locations)[0], "lib", "libamdhip64.so")
    if os.path.exists(bundled):
        ctypes.CDLL(bundled, mode=ctypes.RTLD_GLOBAL)


def _load():
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build(force=True)
    _share_hip_runtime_with_torch()
    lib = ctypes.CDLL(LIB_PATH)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.pg_strerror.restype = ctypes.c_char_p
    lib.pg_strerror.argtypes = [ci]
    lib.pg_init.restype = ci
    lib.pg_init.argtypes = [ctypes.POINTER(vp), ci, ci, vp, vp, ci, vp, vp, ci, ci]
    lib.pg_destroy.restype = ci
    lib.pg_destroy.argtypes = [vp]
    for name, args in [("pg_param_floats", [vp]), ("pg_layer_offset", [vp, ci]), ("pg_layer_stride", [vp, ci]),
                       ("pg_qstate_floats", [vp]), ("pg_q_offset", [vp, ci, ci]),
                       ("pg_workspace_bytes", [vp]), ("pg_ws_phat_offset", [vp, ci, ci]),
                       ("pg_ws_flag_offset", [vp, ci, ci]), ("pg_message_floats", [vp])]:
        getattr(lib, name).restype = sz
        getattr(lib, name).argtypes = args
    lib.pg_layer_rank.restype = ci
    lib.pg_layer_rank.argtypes = [vp, ci]
    lib.pg_round_bytes.restype = ctypes.c_double
    lib.pg_round_bytes.argtypes = [vp, ci]
    lib.pg_upload.restype = ci
    lib.pg_upload.argtypes = [vp]
    lib.pg_round.restype = ci
    lib.pg_round.argtypes = [vp, vp, vp, vp, vp]
    lib.pg_round_static.restype = ci
    lib.pg_round_static.argtypes = [vp, vp, vp, vp]
    lib.pg_round_sgd.restype = ci
    lib.pg_round_sgd.argtypes = [vp, vp, vp, ctypes.c_float, vp, vp, vp]
    lib.pg_pstate_floats.restype = sz
    lib.pg_pstate_floats.argtypes = [vp]
    lib.pg_p_offset.restype = sz
    lib.pg_p_offset.argtypes = [vp, ci, ci]
    lib.pg_iterate.restype = ci
    lib.pg_iterate.argtypes = [vp, vp, vp, vp, ctypes.c_longlong, ci, vp, ctypes.c_float, vp, vp]
    lib.pg_run.restype = ci
    lib.pg_run.argtypes = [vp, vp, vp, vp, vp, ci]
    lib.pg_profile_enable.restype = ci
    lib.pg_profile_enable.argtypes = [vp, ci]
    lib.pg_profile_collect.restype = ci
    lib.pg_profile_collect.argtypes = [vp, ctypes.POINTER(pg_kernel_time), ci, ctypes.POINTER(ci)]
    return lib


lib = _load()


class PGError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"powergossip: {pg_strerror(status)} ({status})")


def _check(status: int) -> None:
    if status != PG_OK:
        raise PGError(status)


def pg_strerror(status: int) -> str:
    return lib.pg_strerror(status).decode()


def pg_init(n_workers: int, edges, edge_w, rows, cols, rank: int, power_steps: int) -> int:
    """Returns the context handle (an integer address); raises PGError on a bad problem."""
    edges = np.ascontiguousarray(edges, dtype=np.int32).reshape(-1)
    edge_w = np.ascontiguousarray(edge_w, dtype=np.float32).reshape(-1)
    rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1)
    cols = np.ascontiguousarray(cols, dtype=np.int32).reshape(-1)
    if edges.size != 2 * edge_w.size or rows.size != cols.size:
        raise PGError(PG_ERR_ARG)
    out = ctypes.c_void_p()
    _check(lib.pg_init(ctypes.byref(out), n_workers, edge_w.size,
                       edges.ctypes.data if edges.size else None,
                       edge_w.ctypes.data if edge_w.size else None,
                       rows.size, rows.ctypes.data, cols.ctypes.data, rank, power_steps))
    return out.value


def pg_destroy(ctx: int) -> None:
    _check(lib.pg_destroy(ctx))


def pg_param_floats(ctx): return lib.pg_param_floats(ctx)
def pg_layer_offset(ctx, layer): return lib.pg_layer_offset(ctx, layer)
def pg_layer_stride(ctx, layer): return lib.pg_layer_stride(ctx, layer)
def pg_layer_rank(ctx, layer): return lib.pg_layer_rank(ctx, layer)
def pg_qstate_floats(ctx): return lib.pg_qstate_floats(ctx)
def pg_q_offset(ctx, edge, layer): return lib.pg_q_offset(ctx, edge, layer)
def pg_workspace_bytes(ctx): return lib.pg_workspace_bytes(ctx)
def pg_ws_phat_offset(ctx, edge, layer): return lib.pg_ws_phat_offset(ctx, edge, layer)
def pg_ws_flag_offset(ctx, edge, layer): return lib.pg_ws_flag_offset(ctx, edge, layer)
def pg_message_floats(ctx): return lib.pg_message_floats(ctx)
def pg_round_bytes(ctx, fused: bool): return lib.pg_round_bytes(ctx, 1 if fused else 0)


def pg_upload(ctx) -> None:
    _check(lib.pg_upload(ctx))


def _ptr_table(worker_ptrs: Sequence[int]):
    return (ctypes.c_void_p * len(worker_ptrs))(*worker_ptrs)


def pg_round(ctx, worker_ptrs: Sequence[int], q_ptr: int, ws_ptr: int, stream: int = 0) -> None:
    """worker_ptrs: device addresses of the n parameter buffers; q_ptr / ws_ptr: device addresses."""
    _check(lib.pg_round(ctx, _ptr_table(worker_ptrs), q_ptr, ws_ptr, stream))


def pg_round_static(ctx, worker_ptrs: Sequence[int], q_ptr: int, stream: int = 0) -> None:
    """pg_round on the library's static workspace: no allocation of any kind inside the call."""
    _check(lib.pg_round_static(ctx, _ptr_table(worker_ptrs), q_ptr, stream))


def pg_round_sgd(ctx, worker_ptrs: Sequence[int], grad_ptrs: Sequence[int], eta: float, q_ptr: int,
                 ws_ptr: int, stream: int = 0) -> None:
    """grad_ptrs: device addresses of the n gradient buffers (laid out like the parameters)."""
    _check(lib.pg_round_sgd(ctx, _ptr_table(worker_ptrs), _ptr_table(grad_ptrs), eta, q_ptr, ws_ptr, stream))


def pg_pstate_floats(ctx): return lib.pg_pstate_floats(ctx)
def pg_p_offset(ctx, edge, layer): return lib.pg_p_offset(ctx, edge, layer)


def pg_iterate(ctx, worker_ptrs: Sequence[int], q_ptr: int, p_ptr: int, k_done: int, iterations: int,
               grad_ptrs, eta: float, ws_ptr: int, stream: int = 0) -> None:
    """`iterations` of Algorithm 2's single iterations, numbered from k_done + 1; grad_ptrs None = no gradient."""
    _check(lib.pg_iterate(ctx, _ptr_table(worker_ptrs), q_ptr, p_ptr, k_done, iterations,
                          None if grad_ptrs is None else _ptr_table(grad_ptrs), eta, ws_ptr, stream))


def pg_run(ctx, worker_ptrs: Sequence[int], q_ptr: int, ws_ptr: int, stream: int, rounds: int) -> None:
    _check(lib.pg_run(ctx, _ptr_table(worker_ptrs), q_ptr, ws_ptr, stream, rounds))


def pg_profile_enable(ctx, on: bool) -> None:
    _check(lib.pg_profile_enable(ctx, 1 if on else 0))


def pg_profile_collect(ctx):
    """Returns [{name, launches, ms, bytes}] summed per kernel kind since the last collect."""
    buf = (pg_kernel_time * 16)()
    n = ctypes.c_int(0)
    _check(lib.pg_profile_collect(ctx, buf, 16, ctypes.byref(n)))
    return [dict(name=buf[i].name.decode(), launches=buf[i].launches, ms=buf[i].ms, bytes=buf[i].bytes)
            for i in range(n.value)]
