"""Binding of the GPU input generator plus a numpy reference of its integer stream.
INPUT GENERATOR ONLY: no optimizer arithmetic lives here."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIBRARY = os.path.join(_HERE, "libdesloc_inputs.so")

PURPOSE_GRAD, PURPOSE_X0 = 0, 1

_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIBRARY):
            raise FileNotFoundError(f"{LIBRARY} is not built; run `python -m paper_2505_22549_amd.build`")
        import torch  # noqa: F401  (same HIP runtime instance as the tensors' owner)
        L = ctypes.CDLL(LIBRARY)
        vp, u64, u32, i32, f32 = (ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int,
                                  ctypes.c_float)
        L.desloc_inputs_fill.restype = i32
        L.desloc_inputs_fill.argtypes = [vp, i32, u64, vp, vp, u64, i32, f32, f32, u64, u32, u32, u32, vp]
        L.desloc_inputs_philox_raw.restype = i32
        L.desloc_inputs_philox_raw.argtypes = [vp, vp, vp, u64, vp]
        L.desloc_inputs_calibration_copy.restype = i32
        L.desloc_inputs_calibration_copy.argtypes = [vp, vp, u64, vp]
        L.desloc_inputs_stream.restype = i32
        L.desloc_inputs_stream.argtypes = [vp, u64, u64, i32, i32, i32, i32, u32, vp]
        L.desloc_inputs_philox_host.restype = None
        L.desloc_inputs_philox_host.argtypes = [vp, vp, vp]
        _lib = L
    return _lib


def fill(dst_ptr: int, bf16: bool, total: int, d_starts_ptr: int, d_scale_ptr: int, n_tensors: int,
         dist: int, mean0: float, mean_per_replica: float, seed: int, step: int, replica: int,
         purpose: int = PURPOSE_GRAD, stream: int = 0) -> None:
    rc = lib().desloc_inputs_fill(dst_ptr, int(bf16), total, d_starts_ptr, d_scale_ptr, n_tensors,
                                  dist, mean0, mean_per_replica, seed, step, replica, purpose,
                                  ctypes.c_void_p(stream or None))
    if rc != 0:
        raise RuntimeError(f"desloc_inputs_fill failed: hipError {rc}")


def calibration_copy(dst_ptr: int, src_ptr: int, nbytes: int, stream: int = 0) -> None:
    """Plain device copy of exactly nbytes (read nbytes, write nbytes)."""
    rc = lib().desloc_inputs_calibration_copy(dst_ptr, src_ptr, nbytes, ctypes.c_void_p(stream or None))
    if rc != 0:
        raise RuntimeError(f"desloc_inputs_calibration_copy failed: {rc}")


def stream(base_ptr: int, stride_bytes: int, stream_bytes: int, n_read: int, n_write: int, inplace: bool,
           paired: bool, lds_bytes: int, stream: int = 0) -> None:
    """One launch of a streaming yardstick kernel (see desloc_inputs_stream)."""
    rc = lib().desloc_inputs_stream(base_ptr, stride_bytes, stream_bytes, n_read, n_write, int(inplace),
                                    int(paired), lds_bytes, ctypes.c_void_p(stream or None))
    if rc != 0:
        raise RuntimeError(f"desloc_inputs_stream failed: {rc}")


def philox_host(counter, key) -> np.ndarray:
    c = np.ascontiguousarray(counter, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    lib().desloc_inputs_philox_host(c.ctypes.data, k.ctypes.data, out.ctypes.data)
    return out


def philox4x32_10_numpy(counter: np.ndarray, key: np.ndarray) -> np.ndarray:
    """Reference Philox4x32-10 in numpy, written from the published description
    (Salmon et al., SC'11).  counter: [n, 4] uint32, key: [n, 2] uint32 -> [n, 4]."""
    c = np.array(counter, dtype=np.uint64).reshape(-1, 4)
    k = np.array(key, dtype=np.uint64).reshape(-1, 2).copy()
    M0, M1 = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57)
    W0, W1 = np.uint64(0x9E3779B9), np.uint64(0xBB67AE85)
    mask = np.uint64(0xFFFFFFFF)
    s32 = np.uint64(32)
    for _ in range(10):
        p0 = M0 * c[:, 0]
        p1 = M1 * c[:, 2]
        n0 = (p1 >> s32) ^ c[:, 1] ^ k[:, 0]
        n1 = p1 & mask
        n2 = (p0 >> s32) ^ c[:, 3] ^ k[:, 1]
        n3 = p0 & mask
        c = np.stack([n0, n1, n2, n3], axis=1)
        k[:, 0] = (k[:, 0] + W0) & mask
        k[:, 1] = (k[:, 1] + W1) & mask
    return c.astype(np.uint32)


def reference_values(seed: int, purpose: int, step: int, replica: int, tensor: int, idx: np.ndarray,
                     dist: int, scale: float, mean0: float, mean_per_replica: float) -> np.ndarray:
    """float64 reference of the generator's values for elements idx of one tensor."""
    idx = np.asarray(idx, dtype=np.uint64)
    n = idx.size
    ctr = np.empty((n, 4), dtype=np.uint32)
    ctr[:, 0] = (idx & np.uint64(0xFFFFFFFF)).astype(np.uint32)
    ctr[:, 1] = tensor
    ctr[:, 2] = step
    ctr[:, 3] = replica | (purpose << 16)
    key = np.empty((n, 2), dtype=np.uint32)
    key[:, 0] = seed & 0xFFFFFFFF
    key[:, 1] = (idx >> np.uint64(32)).astype(np.uint32)
    r = philox4x32_10_numpy(ctr, key).astype(np.uint64)
    two24 = 2.0 ** -24

    def bm(a, b):
        u1 = ((a >> np.uint64(8)).astype(np.float64) + 1.0) * two24
        u2 = (b >> np.uint64(8)).astype(np.float64) * two24
        rad = np.sqrt(-2.0 * np.log(u1))
        return rad * np.cos(2 * np.pi * u2), rad * np.sin(2 * np.pi * u2)

    z0, z1 = bm(r[:, 0], r[:, 1])
    if dist == 0:
        return mean0 + mean_per_replica * replica + scale * z0
    z2, z3 = bm(r[:, 2], r[:, 3])
    return scale * z0 / np.sqrt((z1 * z1 + z2 * z2 + z3 * z3) / 3.0)
