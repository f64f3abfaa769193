"""ctypes binding of the DES-LOC step library: argument marshalling only.

The functions here carry the names of the C ABI in include/desloc.h and do nothing
but convert Python values to C arguments and raise on a negative status.  All of the
method (clip, replica averages, moment and parameter updates) runs in the gfx950
kernels of libdesloc.so.  There is no CPU fallback: a missing library is an error.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIBRARY = os.path.join(_PKG, "libdesloc.so")

# enums of include/desloc.h
ADAM, ADOPT, SGDM = 0, 1, 2
F32, BF16 = 0, 1
FLAG_ADAM_LITERAL, FLAG_ADOPT_AVG_NORMALISER, FLAG_ADOPT_INIT_G0SQ, FLAG_NORM_CLIP = 1, 2, 4, 8
FLAG_POST_AVERAGE, FLAG_AMSGRAD = 16, 32
INIT_AS_IS, INIT_ZERO_STATES, INIT_BROADCAST_REPLICA0 = 0, 1, 2
X, U, V, G, VMAX = 0, 1, 2, 3, 4
REPLICA_MEAN = -1
ALL_TENSORS = -1
SYNC_X, SYNC_U, SYNC_V = 1, 2, 4
OK, ERR_NULL, ERR_BAD_ARG, ERR_ALIGN, ERR_OOM, ERR_HIP, ERR_VARIANT, ERR_TOO_LARGE = 0, -1, -2, -3, -4, -5, -6, -7
STATIC_SCRATCH_BYTES = 4 << 20


class desloc_config(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("variant", ctypes.c_uint32),
        ("M", ctypes.c_uint32),
        ("grad_dtype", ctypes.c_uint32),
        ("n_tensors", ctypes.c_uint64),
        ("numel", ctypes.POINTER(ctypes.c_uint64)),
        ("Kx", ctypes.c_uint64),
        ("Ku", ctypes.c_uint64),
        ("Kv", ctypes.c_uint64),
        ("lr", ctypes.c_float),
        ("beta1", ctypes.c_float),
        ("beta2", ctypes.c_float),
        ("eps", ctypes.c_float),
        ("rho", ctypes.c_float),
        ("flags", ctypes.c_uint32),
        ("init_mode", ctypes.c_uint32),
        ("x", ctypes.POINTER(ctypes.c_void_p)),
        ("u", ctypes.POINTER(ctypes.c_void_p)),
        ("v", ctypes.POINTER(ctypes.c_void_p)),
        ("g", ctypes.POINTER(ctypes.c_void_p)),
        ("vmax", ctypes.POINTER(ctypes.c_void_p)),
        ("stream", ctypes.c_void_p),
        ("chunk_elems", ctypes.c_uint32),
        ("reserved", ctypes.c_uint32),
    ]


class desloc_plan_info(ctypes.Structure):
    _fields_ = [
        ("n_segments", ctypes.c_uint64),
        ("n_chunks", ctypes.c_uint64),
        ("total_numel", ctypes.c_uint64),
        ("chunk_elems", ctypes.c_uint32),
        ("strided", ctypes.c_uint32),
        ("paired_numel", ctypes.c_uint64),
        ("lds_limiter_bytes", ctypes.c_uint32 * 2),
        ("intended_workgroups", ctypes.c_uint32 * 2),
        ("resident_workgroups", ctypes.c_uint32 * 2),
        ("gated_chunk_elems", ctypes.c_uint32),
        ("reserved", ctypes.c_uint32),
    ]


class DeslocError(RuntimeError):
    def __init__(self, status: int, where: str, hip_error: int = 0):
        self.status = status
        self.hip_error = hip_error
        msg = f"{where}: {desloc_strerror(status)} (status {status}"
        msg += f", hipError {hip_error})" if hip_error else ")"
        super().__init__(msg)


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """Loads libdesloc.so (built by `python -m paper_2505_22549_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIBRARY):
            raise FileNotFoundError(
                f"{LIBRARY} is not built; run `python -m paper_2505_22549_amd.build` "
                "(there is no CPU fallback)")
        # PyTorch ships its own HIP runtime; load it first so that this library binds to the
        # same runtime instance that owns the caller's device memory and streams.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIBRARY)
        vp, u64, u32, i32 = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int
        L.desloc_version.restype = u32
        L.desloc_version.argtypes = []
        L.desloc_strerror.restype = ctypes.c_char_p
        L.desloc_strerror.argtypes = [i32]
        L.desloc_last_hip_error.restype = i32
        L.desloc_last_hip_error.argtypes = [vp]
        L.desloc_sync_mask_k.restype = u32
        L.desloc_sync_mask_k.argtypes = [u64, u64, u64, u64]
        L.desloc_plan.restype = i32
        L.desloc_plan.argtypes = [ctypes.POINTER(desloc_config), ctypes.POINTER(desloc_plan_info)]
        L.desloc_init.restype = i32
        L.desloc_init.argtypes = [ctypes.POINTER(desloc_config), ctypes.POINTER(vp)]
        L.desloc_sync_mask.restype = u32
        L.desloc_sync_mask.argtypes = [vp, u64]
        L.desloc_set_lr.restype = i32
        L.desloc_set_lr.argtypes = [vp, ctypes.c_float]
        L.desloc_step.restype = i32
        L.desloc_step.argtypes = [vp, u64]
        L.desloc_read_state.restype = i32
        L.desloc_read_state.argtypes = [vp, i32, i32, ctypes.c_int64, vp, ctypes.c_size_t]
        L.desloc_read_grad_norms.restype = i32
        L.desloc_read_grad_norms.argtypes = [vp, vp, ctypes.c_size_t]
        L.desloc_state_change.restype = i32
        L.desloc_state_change.argtypes = [vp, i32, ctypes.c_int64, vp, vp, vp, ctypes.c_size_t]
        L.desloc_state_change_static.restype = i32
        L.desloc_state_change_static.argtypes = [vp, i32, ctypes.c_int64, vp, vp, vp, ctypes.c_size_t]
        L.desloc_bind_reference.restype = i32
        L.desloc_bind_reference.argtypes = [vp, vp]
        L.desloc_state_change_tensors.restype = i32
        L.desloc_state_change_tensors.argtypes = [vp, i32, vp, vp]
        L.desloc_snapshot_state.restype = i32
        L.desloc_snapshot_state.argtypes = [vp, i32, vp]
        L.desloc_get_plan.restype = i32
        L.desloc_get_plan.argtypes = [vp, ctypes.POINTER(desloc_plan_info)]
        L.desloc_synchronize.restype = i32
        L.desloc_synchronize.argtypes = [vp]
        L.desloc_destroy.restype = i32
        L.desloc_destroy.argtypes = [vp]
        _lib = L
    return _lib


def _check(status: int, where: str, ctx=None) -> None:
    if status < 0:
        hip = lib().desloc_last_hip_error(ctx) if status == ERR_HIP else 0
        raise DeslocError(status, where, hip)


def desloc_version() -> int:
    return int(lib().desloc_version())


def desloc_strerror(status: int) -> str:
    return lib().desloc_strerror(status).decode()


def desloc_sync_mask_k(t: int, Kx: int, Ku: int, Kv: int) -> int:
    return int(lib().desloc_sync_mask_k(t, Kx, Ku, Kv))


class _Marshalled:
    """Keeps the ctypes arrays referenced by a desloc_config alive."""

    def __init__(self, *, variant, M, numel, Kx, Ku, Kv, lr, beta1, beta2, eps, rho, x, u, v, g,
                 vmax=None, grad_dtype=F32, flags=0, init_mode=INIT_AS_IS, stream=0, chunk_elems=0):
        numel = np.ascontiguousarray(numel, dtype=np.uint64)
        nt = int(numel.size)
        self.numel = numel

        def table(t):
            if t is None:
                return None, None
            a = np.ascontiguousarray(t, dtype=np.uint64).reshape(-1)
            if a.size != M * nt:
                raise ValueError(f"pointer table needs M*n_tensors = {M * nt} entries, got {a.size}")
            return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_void_p))

        self.tx, px = table(x)
        self.tu, pu = table(u)
        self.tv, pv = table(v)
        self.tg, pg = table(g)
        self.tvm, pvm = table(vmax)
        self.cfg = desloc_config(
            ctypes.sizeof(desloc_config), variant, M, grad_dtype, nt,
            numel.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)), Kx, Ku, Kv, lr, beta1, beta2, eps,
            rho, flags, init_mode, px, pu, pv, pg, pvm, ctypes.c_void_p(stream or None), chunk_elems, 0)


def desloc_plan(**kw) -> desloc_plan_info:
    """desloc_plan: the segment / chunk decomposition for a config (host only)."""
    m = _Marshalled(**kw)
    info = desloc_plan_info()
    _check(lib().desloc_plan(ctypes.byref(m.cfg), ctypes.byref(info)), "desloc_plan")
    return info


def desloc_init(**kw) -> ctypes.c_void_p:
    """desloc_init: returns the opaque context handle.

    Keyword arguments mirror struct desloc_config; x/u/v/g are integer arrays of
    M*n_tensors device addresses (index m*n_tensors + k)."""
    m = _Marshalled(**kw)
    ctx = ctypes.c_void_p()
    _check(lib().desloc_init(ctypes.byref(m.cfg), ctypes.byref(ctx)), "desloc_init")
    return ctx


def desloc_sync_mask(ctx, t: int) -> int:
    return int(lib().desloc_sync_mask(ctx, t))


def desloc_set_lr(ctx, lr: float) -> None:
    _check(lib().desloc_set_lr(ctx, lr), "desloc_set_lr", ctx)


def desloc_step(ctx, t: int) -> None:
    _check(lib().desloc_step(ctx, t), "desloc_step", ctx)


def desloc_get_plan(ctx) -> desloc_plan_info:
    info = desloc_plan_info()
    _check(lib().desloc_get_plan(ctx, ctypes.byref(info)), "desloc_get_plan", ctx)
    return info


def desloc_read_state(ctx, which: int, replica: int, tensor: int, count: int) -> np.ndarray:
    """desloc_read_state into a fresh float32 array of `count` elements."""
    out = np.empty(count, dtype=np.float32)
    _check(lib().desloc_read_state(ctx, which, replica, tensor, out.ctypes.data_as(ctypes.c_void_p),
                                   out.nbytes), "desloc_read_state", ctx)
    return out


def desloc_read_grad_norms(ctx, M: int) -> np.ndarray:
    """desloc_read_grad_norms: ||g^m||_2 of the most recent step (norm-clip contexts only)."""
    out = np.empty(M, dtype=np.float32)
    _check(lib().desloc_read_grad_norms(ctx, out.ctypes.data_as(ctypes.c_void_p), M),
           "desloc_read_grad_norms", ctx)
    return out


def desloc_snapshot_state(ctx, which: int, dst_table) -> None:
    """desloc_snapshot_state: dst_table is an integer array of M*n_tensors device addresses."""
    t = np.ascontiguousarray(dst_table, dtype=np.uint64).reshape(-1)
    _check(lib().desloc_snapshot_state(ctx, which, t.ctypes.data_as(ctypes.c_void_p)),
           "desloc_snapshot_state", ctx)


def desloc_state_change(ctx, which: int, tensor: int, ref_table, M: int):
    """desloc_state_change: (||s^m - ref^m||_2, ||ref^m||_2) per replica as float32 arrays."""
    t = np.ascontiguousarray(ref_table, dtype=np.uint64).reshape(-1)
    change = np.empty(M, dtype=np.float32)
    base = np.empty(M, dtype=np.float32)
    _check(lib().desloc_state_change(ctx, which, tensor, t.ctypes.data_as(ctypes.c_void_p),
                                     change.ctypes.data_as(ctypes.c_void_p),
                                     base.ctypes.data_as(ctypes.c_void_p), M),
           "desloc_state_change", ctx)
    return change, base


def desloc_bind_reference(ctx, ref_table) -> None:
    """desloc_bind_reference: ref_table is an integer array of M*n_tensors device addresses."""
    t = np.ascontiguousarray(ref_table, dtype=np.uint64).reshape(-1)
    _check(lib().desloc_bind_reference(ctx, t.ctypes.data_as(ctypes.c_void_p)), "desloc_bind_reference", ctx)


def desloc_state_change_tensors(ctx, which: int, change_dev_ptr: int, base_dev_ptr: int) -> None:
    """desloc_state_change_tensors: asynchronous; the two arguments are device addresses of
    n_tensors*M floats each."""
    _check(lib().desloc_state_change_tensors(ctx, which, ctypes.c_void_p(change_dev_ptr),
                                             ctypes.c_void_p(base_dev_ptr)),
           "desloc_state_change_tensors", ctx)


def desloc_state_change_static(ctx, which: int, tensor: int, ref_table, M: int):
    """desloc_state_change_static: as desloc_state_change, from the library's fixed scratch array
    (the entry point itself allocates nothing; the result arrays here are the caller's)."""
    t = np.ascontiguousarray(ref_table, dtype=np.uint64).reshape(-1)
    change = np.empty(M, dtype=np.float32)
    base = np.empty(M, dtype=np.float32)
    _check(lib().desloc_state_change_static(ctx, which, tensor, t.ctypes.data_as(ctypes.c_void_p),
                                            change.ctypes.data_as(ctypes.c_void_p),
                                            base.ctypes.data_as(ctypes.c_void_p), M),
           "desloc_state_change_static", ctx)
    return change, base


def desloc_synchronize(ctx) -> None:
    _check(lib().desloc_synchronize(ctx), "desloc_synchronize", ctx)


def desloc_destroy(ctx) -> None:
    _check(lib().desloc_destroy(ctx), "desloc_destroy")


def packed_pointer_table(base_addr: int, replica_stride_bytes: int, numel: Sequence[int], M: int,
                         elem_size: int) -> np.ndarray:
    """Device addresses of tensor k of replica m when each replica is one packed buffer
    (tensors back to back, no padding) and replicas are `replica_stride_bytes` apart."""
    numel = np.asarray(numel, dtype=np.uint64)
    starts = np.concatenate(([0], np.cumsum(numel)[:-1])).astype(np.uint64) * np.uint64(elem_size)
    rep = (np.arange(M, dtype=np.uint64) * np.uint64(replica_stride_bytes))[:, None]
    return (np.uint64(base_addr) + rep + starts[None, :]).reshape(-1)
