"""Device-memory plumbing around the C ABI: PyTorch allocates the replica buffers, this
module turns them into the pointer tables desloc_init wants.  No arithmetic of the
method happens here; every step runs in libdesloc.so's kernels.
"""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as B
from .inputs import generator as gen
from .inputs.recipes import Workload


def _round_up(n: int, k: int) -> int:
    return (n + k - 1) // k * k


class PackedReplicas:
    """x, u, v, g for M replicas, each replica one packed buffer (tensors back to back).

    Layout in HBM: one allocation per array of shape [M, stride]; stride is the total
    element count rounded up to a multiple of 16384 elements (64 KiB of fp32).  Large
    PyTorch allocations start on 2 MiB boundaries, so every fp32 stream then starts at the
    same offset modulo 64 KiB: the condition for the library's fastest (paired) mapping."""

    def __init__(self, numel, M: int, has_v: bool, grad_bf16: bool, device="cuda:0",
                 stride_pad_elems: int = 0, has_vmax: bool = False):
        self.numel = np.ascontiguousarray(numel, dtype=np.uint64)
        self.M = M
        self.total = int(self.numel.sum())
        self.stride = _round_up(max(self.total, 1), 16384) + stride_pad_elems
        self.device = torch.device(device)
        f32 = dict(dtype=torch.float32, device=self.device)
        self.x = torch.zeros((M, self.stride), **f32)
        self.u = torch.zeros((M, self.stride), **f32)
        self.v = torch.zeros((M, self.stride), **f32) if has_v else None
        self.vmax = torch.zeros((M, self.stride), **f32) if has_vmax else None
        self.g = torch.zeros((M, self.stride), device=self.device,
                             dtype=torch.bfloat16 if grad_bf16 else torch.float32)
        self.grad_bf16 = grad_bf16

    def table(self, t: Optional[torch.Tensor]):
        if t is None:
            return None
        es = t.element_size()
        return B.packed_pointer_table(t.data_ptr(), self.stride * es, self.numel, self.M, es)

    def starts(self) -> np.ndarray:
        return np.concatenate(([0], np.cumsum(self.numel))).astype(np.uint64)


class DeslocSession:
    """A workload resident on the GPU plus its library context."""

    def __init__(self, w: Workload, device="cuda:0", chunk_elems: int = 0,
                 init_mode: int = B.INIT_BROADCAST_REPLICA0, stream: Optional[torch.cuda.Stream] = None):
        self.w = w
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.stream = stream
        self.mem = PackedReplicas(w.numel, w.M, w.variant != B.SGDM, w.grad_bf16, device,
                                  has_vmax=bool(w.flags & B.FLAG_AMSGRAD))
        self.d_starts = torch.from_numpy(self.mem.starts().astype(np.int64)).to(self.device)
        self.d_scale = torch.from_numpy(np.ascontiguousarray(w.grad_scale, dtype=np.float32)).to(self.device)
        self.d_x0scale = torch.full((w.n_tensors,), w.x0_std, dtype=torch.float32, device=self.device)
        torch.cuda.synchronize(self.device)  # allocations ran on torch's stream, not necessarily ours
        self.fill_x0()
        torch.cuda.synchronize(self.device)
        self.ctx = B.desloc_init(
            variant=w.variant, M=w.M, numel=w.numel, Kx=w.Kx, Ku=w.Ku, Kv=w.Kv, lr=w.lr,
            beta1=w.beta1, beta2=w.beta2, eps=w.eps, rho=w.rho, x=self.mem.table(self.mem.x),
            u=self.mem.table(self.mem.u), v=self.mem.table(self.mem.v), g=self.mem.table(self.mem.g),
            vmax=self.mem.table(self.mem.vmax), grad_dtype=B.BF16 if w.grad_bf16 else B.F32, flags=w.flags, init_mode=init_mode,
            stream=stream.cuda_stream if stream is not None else 0, chunk_elems=chunk_elems)
        B.desloc_synchronize(self.ctx)

    # -- synthetic inputs (outside any timed region) ---------------------------
    def _stream_ptr(self) -> int:
        return self.stream.cuda_stream if self.stream is not None else 0

    def fill_x0(self) -> None:
        """x_0 ~ N(0, x0_std^2) into replica 0 (init broadcasts it: same start on every worker)."""
        w = self.w
        gen.fill(self.mem.x[0].data_ptr(), False, self.mem.total, self.d_starts.data_ptr(),
                 self.d_x0scale.data_ptr(), w.n_tensors, 0, 0.0, 0.0, w.seed, 0, 0,
                 gen.PURPOSE_X0, self._stream_ptr())

    def fill_gradients(self, t: int) -> None:
        """g_t^m for every replica m from the counter-based generator."""
        w = self.w
        for m in range(w.M):
            gen.fill(self.mem.g[m].data_ptr(), w.grad_bf16, self.mem.total, self.d_starts.data_ptr(),
                     self.d_scale.data_ptr(), w.n_tensors, w.dist, w.grad_mean0,
                     w.grad_mean_per_replica, w.seed, t, m, gen.PURPOSE_GRAD, self._stream_ptr())

    # -- the hot path -----------------------------------------------------------
    def step(self, t: int) -> None:
        B.desloc_step(self.ctx, t)

    def sync_mask(self, t: int) -> int:
        return B.desloc_sync_mask(self.ctx, t)

    def synchronize(self) -> None:
        B.desloc_synchronize(self.ctx)

    def read(self, which: int, replica: int, tensor: int = B.ALL_TENSORS) -> np.ndarray:
        n = self.mem.total if tensor == B.ALL_TENSORS else int(self.w.numel[tensor])
        return B.desloc_read_state(self.ctx, which, replica, tensor, n)

    def close(self) -> None:
        if self.ctx is not None:
            B.desloc_destroy(self.ctx)
            self.ctx = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
