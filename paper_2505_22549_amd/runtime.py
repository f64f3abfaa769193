"""Device-memory plumbing around the C ABI: PyTorch allocates the replica buffers, this
module turns them into the pointer tables desloc_init wants.  No arithmetic of the
method happens here; every step runs in libdesloc.so's kernels.
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np
import torch

from . import binding as B
from .inputs import generator as gen
from .inputs.recipes import Workload


def _round_up(n: int, k: int) -> int:
    return (n + k - 1) // k * k


def _esize(dt) -> int:
    return 2 if dt == torch.bfloat16 else 4


class PackedReplicas:
    """x, u, v, g for M replicas, each replica one packed buffer per array (tensors back to back).

    Layout in HBM: ONE allocation of M records; record m holds replica m's x, u, v (vmax) and g
    one after the other, each `stride` elements long; stride is the total element count rounded
    up to a multiple of 16384 elements (64 KiB of fp32) and the record is rounded up to 64 KiB,
    so every fp32 stream starts at the same offset modulo 64 KiB: the condition for the
    library's fastest (paired) mapping.  To the library this is a strided layout like any other:
    array a of replica m at base[a] + m * record.

    Why replica-major records and not one [M][stride] block per array: a step without a gate
    sweeps one replica's g, x, u, v at a time, and on MI355X streams that are swept together run
    3-5 % faster when they lie in the same physically contiguous block of device memory than
    when they are tens of GiB apart (measured; with per-array blocks the step time of the
    1.7B-parameter workload moved between 6.43 and 6.72 TB/s with the position of the arrays,
    with records it is 6.68-6.76 TB/s everywhere).  Gated steps sweep all replicas at once and
    gain nothing from it."""

    ALIGN = 2 << 20   # placements inside a pool start on 2 MiB boundaries
    RECORD_ALIGN = 65536

    @staticmethod
    def _spec(has_v: bool, grad_bf16: bool, has_vmax: bool):
        gdt = torch.bfloat16 if grad_bf16 else torch.float32
        spec = [("x", torch.float32, True), ("u", torch.float32, True), ("v", torch.float32, has_v),
                ("vmax", torch.float32, has_vmax), ("g", gdt, True)]  # g last: a bf16 g is half as long
        return spec

    def __init__(self, numel, M: int, has_v: bool, grad_bf16: bool, device="cuda:0",
                 stride_pad_elems: int = 0, has_vmax: bool = False,
                 pool: Optional[torch.Tensor] = None, pool_offset: int = 0):
        """pool / pool_offset: carve the records out of an existing zero-filled uint8 tensor,
        starting pool_offset bytes past its first 2 MiB boundary, instead of allocating them."""
        self.numel = np.ascontiguousarray(numel, dtype=np.uint64)
        self.M = M
        self.total = int(self.numel.sum())
        self.stride = _round_up(max(self.total, 1), 16384) + stride_pad_elems
        self.device = torch.device(device)
        self.grad_bf16 = grad_bf16
        spec = self._spec(has_v, grad_bf16, has_vmax)
        self.record_bytes = _round_up(sum(self.stride * _esize(dt) for _, dt, present in spec if present),
                                      self.RECORD_ALIGN)
        need = M * self.record_bytes
        if pool is None:
            pool = torch.zeros(need, dtype=torch.uint8, device=self.device)
            off = 0
        else:
            off = (-pool.data_ptr()) % self.ALIGN + pool_offset
            assert pool_offset % self.ALIGN == 0, "pool_offset must be a multiple of 2 MiB"
            assert off + need <= pool.numel(), "the pool is too small for this placement"
        self.pool = pool
        for name, dt, present in spec:
            if not present:
                setattr(self, name, None)
                continue
            es = _esize(dt)
            flat = pool[:pool.numel() // es * es].view(dt)  # a pool of any byte length
            setattr(self, name, torch.as_strided(flat, (M, self.stride), (self.record_bytes // es, 1),
                                                 flat.storage_offset() + off // es))
            off += self.stride * es

    @classmethod
    def bytes_needed(cls, numel, M: int, has_v: bool, grad_bf16: bool, has_vmax: bool = False) -> int:
        """Bytes a placement occupies."""
        stride = _round_up(max(int(np.asarray(numel, dtype=np.uint64).sum()), 1), 16384)
        rec = sum(stride * _esize(dt) for _, dt, present in cls._spec(has_v, grad_bf16, has_vmax) if present)
        return M * _round_up(rec, cls.RECORD_ALIGN)

    def table(self, t: Optional[torch.Tensor]):
        if t is None:
            return None
        es = t.element_size()
        return B.packed_pointer_table(t.data_ptr(), t.stride(0) * es, self.numel, self.M, es)

    def starts(self) -> np.ndarray:
        return np.concatenate(([0], np.cumsum(self.numel))).astype(np.uint64)

    def snapshot_buffer(self, name: str):
        """(tensor, pointer table) of a zero-filled buffer a state array can be snapshotted into."""
        buf = torch.zeros((self.M, self.stride), dtype=getattr(self, name).dtype, device=self.device)
        return buf, self.table(buf)

    # uniform access for tests and benchmarks, whatever the layout
    def array(self, name: str) -> Optional[torch.Tensor]:
        return getattr(self, name, None)

    def grad_destination(self, m: int) -> torch.Tensor:
        """Where the generator writes replica m's gradients (here: straight into g)."""
        return self.g[m]

    def grads_written(self, m: int) -> None:
        pass

    def packed_view(self, name: str) -> torch.Tensor:
        """[M, >= total] tensor holding array `name` with the tensors back to back."""
        return getattr(self, name)

    def x0_destination(self) -> torch.Tensor:
        return self.x[0]

    def x0_written(self) -> None:
        pass


class SeparateReplicas:
    """x, u, v, g with every tensor of every replica allocated on its own (one torch tensor per
    array, replica and tensor): what a framework holding ordinary per-parameter tensors hands
    over.  The library sees one segment per tensor (or per run of tensors the allocator happens
    to place back to back) and takes its chunk-record / pointer-table path.

    Generated inputs are written into a packed staging buffer and scattered with multi-tensor
    copies; packed_view gathers an array back the same way (tests sample from it)."""

    def __init__(self, numel, M: int, has_v: bool, grad_bf16: bool, device="cuda:0", has_vmax: bool = False):
        self.numel = np.ascontiguousarray(numel, dtype=np.uint64)
        self.M = M
        self.total = int(self.numel.sum())
        self.stride = self.total
        self.device = torch.device(device)
        self.grad_bf16 = grad_bf16
        gdt = torch.bfloat16 if grad_bf16 else torch.float32
        sizes = [int(n) for n in self.numel]

        def alloc(dt):
            return [torch.zeros(n, dtype=dt, device=self.device) for n in sizes]

        # worker by worker, as M separately built model instances would allocate: parameters,
        # gradients, then the optimizer's states
        self.x, self.g, self.u = [], [], []
        self.v = [] if has_v else None
        self.vmax = [] if has_vmax else None
        for _ in range(M):
            self.x.append(alloc(torch.float32))
            self.g.append(alloc(gdt))
            self.u.append(alloc(torch.float32))
            if has_v:
                self.v.append(alloc(torch.float32))
            if has_vmax:
                self.vmax.append(alloc(torch.float32))
        self._sizes = sizes
        self._stage_g = torch.zeros(max(self.total, 1), dtype=gdt, device=self.device)
        self._stage_f = None

    def table(self, t):
        if t is None:
            return None
        # empty tensors have no storage: any non-null, aligned value will do, it is never used
        return np.array([[a.data_ptr() if a.numel() else 0x10 for a in row] for row in t],
                        dtype=np.uint64).reshape(-1)

    def starts(self) -> np.ndarray:
        return np.concatenate(([0], np.cumsum(self.numel))).astype(np.uint64)

    def array(self, name: str):
        return getattr(self, name, None)

    def snapshot_buffer(self, name: str):
        """(tensor, pointer table): one dense [M, total] buffer, tensors back to back."""
        dt = getattr(self, name)[0][0].dtype
        buf = torch.zeros((self.M, _round_up(max(self.total, 1), 4)), dtype=dt, device=self.device)
        es = buf.element_size()
        return buf, B.packed_pointer_table(buf.data_ptr(), buf.stride(0) * es, self.numel, self.M, es)

    # Copies between a packed staging buffer and the layout run piece by piece: a piece is a run of
    # elements that is contiguous both in packed order and in this layout (here: one tensor).
    def _split(self, flat: torch.Tensor):
        return [p for p in torch.split(flat[:self.total], self._sizes) if p.numel()]

    def _pieces(self, name: str, m: int):
        return [t for t in getattr(self, name)[m] if t.numel()]

    def grad_destination(self, m: int) -> torch.Tensor:
        return self._stage_g

    def grads_written(self, m: int) -> None:
        torch._foreach_copy_(self._pieces("g", m), self._split(self._stage_g))

    def x0_destination(self) -> torch.Tensor:
        if self._stage_f is None:
            self._stage_f = torch.zeros(max(self.total, 1), dtype=torch.float32, device=self.device)
        return self._stage_f

    def x0_written(self) -> None:
        torch._foreach_copy_(self._pieces("x", 0), self._split(self._stage_f))

    def packed_view(self, name: str) -> torch.Tensor:
        arr = getattr(self, name)
        out = torch.empty((self.M, max(self.total, 1)), dtype=arr[0][0].dtype, device=self.device)
        for m in range(self.M):
            torch._foreach_copy_(self._split(out[m]), self._pieces(name, m))
        return out


class GroupedReplicas(SeparateReplicas):
    """x, u, v, g in ONE allocation, arranged by groups of consecutive tensors: a group is a run of
    whole tensors of at most `group_bytes` per array and replica (a larger tensor is a group of
    its own), and inside a group lie replica 0's x, u, v, g, then replica 1's, ...  Every tensor
    is contiguous, a group's tensors lie back to back (the library merges them into one segment
    per group) and every array of every group and replica starts on a 64 KiB boundary.

    Why: on MI355X streams that are swept together run fastest when they lie close together
    (within one physically contiguous piece of device memory; which virtual ranges share a piece
    cannot be asked).  With groups, everything a launch touches at any instant, with or without
    a gate, lies within M * 4 * group_bytes: the step time no longer depends on where in HBM the
    allocation landed (records of whole replicas: the gated launches of the 1.7B-parameter workload
    move between 6.25 and 6.5 TB/s with the position; groups: 6.6 TB/s everywhere), and no pool has
    to be held for choosing a placement."""

    GROUP_BYTES = 128 << 20
    ALIGN = 65536

    def __init__(self, numel, M: int, has_v: bool, grad_bf16: bool, device="cuda:0", has_vmax: bool = False,
                 group_bytes: int = 0, pool: Optional[torch.Tensor] = None, pool_offset: int = 0,
                 snapshots: Tuple[str, ...] = ()):
        """pool / pool_offset: carve the groups out of an existing zero-filled uint8 tensor, starting
        pool_offset bytes past its first 64 KiB boundary, instead of allocating (measurements).
        snapshots: states ("x", "u", "v", "vmax") that get a snapshot array of their own inside every
        group, after the replica's g: the rate-of-change diagnostic then reads a state and its
        snapshot from the same neighbourhood (snapshot_buffer returns these arrays)."""
        self.numel = np.ascontiguousarray(numel, dtype=np.uint64)
        self.M = M
        self.total = int(self.numel.sum())
        self.stride = self.total
        self.device = torch.device(device)
        self.grad_bf16 = grad_bf16
        gdt = torch.bfloat16 if grad_bf16 else torch.float32
        sizes = [int(n) for n in self.numel]
        self._sizes = sizes
        group_bytes = group_bytes or self.GROUP_BYTES
        # runs of consecutive tensors
        self.groups, cur, cur_n = [], [], 0
        for k, n in enumerate(sizes):
            if cur and (cur_n + n) * 4 > group_bytes:
                self.groups.append(cur)
                cur, cur_n = [], 0
            cur.append(k)
            cur_n += n
        if cur:
            self.groups.append(cur)
        arrays = [("x", torch.float32), ("u", torch.float32)] + ([("v", torch.float32)] if has_v else []) + \
                 ([("vmax", torch.float32)] if has_vmax else []) + [("g", gdt)]
        state_names = [name for name, _ in arrays if name != "g"]
        assert all(name in state_names for name in snapshots), "snapshots name states of this workload"
        arrays += [("snap_" + name, torch.float32) for name in snapshots]
        slots = []   # per group: (elements rounded up to 64 KiB of fp32, bytes of one replica's arrays)
        need = 0
        for grp in self.groups:
            s_j = _round_up(max(sum(sizes[k] for k in grp), 1), 16384)
            rec = _round_up(sum(s_j * _esize(dt) for _, dt in arrays), self.ALIGN)
            slots.append((s_j, rec))
            need += M * rec
        self.bytes = need
        if pool is None:
            self.pool = torch.zeros(max(need, 1) + self.ALIGN, dtype=torch.uint8, device=self.device)
            off0 = (-self.pool.data_ptr()) % self.ALIGN
        else:
            self.pool = pool
            off0 = (-pool.data_ptr()) % self.ALIGN + pool_offset
            assert pool_offset % self.ALIGN == 0 and off0 + need <= pool.numel(), "the pool is too small for this placement"
        for name in ("x", "u", "v", "vmax", "g"):
            setattr(self, name, None)
        for name, _ in arrays:
            setattr(self, name, [[None] * len(sizes) for _ in range(M)])
        off = off0
        for grp, (s_j, rec) in zip(self.groups, slots):
            for m in range(M):
                a_off = off + m * rec
                for name, dt in arrays:
                    es = _esize(dt)
                    flat = self.pool[:self.pool.numel() // es * es].view(dt)
                    e = a_off // es
                    for k in grp:
                        getattr(self, name)[m][k] = flat[e:e + sizes[k]]
                        e += sizes[k]
                    a_off += s_j * es
            off += M * rec
        self._stage_g = torch.zeros(max(self.total, 1), dtype=gdt, device=self.device)
        self._stage_f = None
        self._slots = slots
        # a group's tensors lie back to back: copies run group by group
        self._group_sizes = [sum(sizes[k] for k in grp) for grp in self.groups]
        self._runs = {}
        for name, dt in arrays:
            es = _esize(dt)
            flat = self.pool[:self.pool.numel() // es * es].view(dt)
            rows = []
            for m in range(M):
                row = []
                for grp, n_j in zip(self.groups, self._group_sizes):
                    first = next((k for k in grp if sizes[k]), None)
                    if first is None:
                        continue
                    e = (getattr(self, name)[m][first].data_ptr() - self.pool.data_ptr()) // es
                    row.append(flat[e:e + n_j])
                rows.append(row)
            self._runs[name] = rows

    def _split(self, flat: torch.Tensor):
        return [p for p in torch.split(flat[:self.total], self._group_sizes) if p.numel()]

    def _pieces(self, name: str, m: int):
        return self._runs[name][m]

    def snapshot_buffer(self, name: str):
        """(tensor, pointer table): the snapshot arrays reserved inside the groups (`snapshots` of the
        constructor; the tensor returned is then the pool), else one allocation arranged like the
        state array itself (per group the M replicas' runs of tensors, each starting on a 64 KiB
        boundary)."""
        inside = getattr(self, "snap_" + name, None)
        if inside is not None:
            return self.pool, self.table(inside)
        dt = getattr(self, name)[0][0].dtype
        es = _esize(dt)
        need = sum(self.M * s_j * es for s_j, _ in self._slots)
        buf = torch.zeros(need + self.ALIGN, dtype=torch.uint8, device=self.device)
        off = buf.data_ptr() + (-buf.data_ptr()) % self.ALIGN
        tab = np.zeros((self.M, len(self._sizes)), dtype=np.uint64)
        for grp, (s_j, _) in zip(self.groups, self._slots):
            for m in range(self.M):
                e = 0
                for k in grp:
                    tab[m, k] = off + (m * s_j + e) * es if self._sizes[k] else 0x10
                    e += self._sizes[k]
            off += self.M * s_j * es
        return buf, tab.reshape(-1)


def search_placement(w: Workload, stream: Optional[torch.cuda.Stream], pool_bytes: int, candidates: int):
    """Where in HBM the records lie changes the time of gated steps by a few percent (streams that
    are swept together are slower when they lie in different physically contiguous blocks of
    device memory, and a gated step sweeps all M records at once; which virtual addresses share
    a block cannot be asked, and differs from device to device and run to run), so measure
    instead of guessing: allocate one zero-filled pool, place the workload's records at evenly
    spaced offsets inside it, time a few steps of the library at each placement (states all zero:
    realistic values run under 1 % slower, everywhere alike), and return (pool, best offset in
    bytes, list of probes).  Setup work, outside any timed region."""
    import math
    has_v, has_vmax = w.variant != B.SGDM, bool(w.flags & B.FLAG_AMSGRAD)
    need = PackedReplicas.bytes_needed(w.numel, w.M, has_v, w.grad_bf16, has_vmax)
    free, _ = torch.cuda.mem_get_info()
    pool_bytes = min(pool_bytes, free - (8 << 30))
    if pool_bytes < need + PackedReplicas.ALIGN:
        raise ValueError(f"placement pool of {pool_bytes} bytes cannot hold the {need}-byte workload")
    pool = torch.zeros(pool_bytes // PackedReplicas.ALIGN * PackedReplicas.ALIGN, dtype=torch.uint8, device="cuda:0")
    room = (pool.numel() - (-pool.data_ptr()) % PackedReplicas.ALIGN - need) // PackedReplicas.ALIGN
    n = max(1, min(candidates, room + 1))
    offsets = sorted({(room * j // max(n - 1, 1)) * PackedReplicas.ALIGN for j in range(n)})
    sptr = stream.cuda_stream if stream is not None else 0
    periods = [k for k in (w.Kx, w.Ku, w.Kv if has_v else 0) if k]
    t_gated = math.lcm(*periods) if periods and w.M > 1 else 0     # every gate of the schedule fires
    if t_gated >= 1 << 63:
        t_gated = periods[0]
    t_plain = 10_000_019
    while any(t_plain % k == 0 for k in periods):
        t_plain += 1
    torch.cuda.synchronize()
    probes = []
    s = stream if stream is not None else torch.cuda.current_stream()
    for off in offsets:
        mem = PackedReplicas(w.numel, w.M, has_v, w.grad_bf16, has_vmax=has_vmax, pool=pool, pool_offset=off)
        ctx = B.desloc_init(variant=w.variant, M=w.M, numel=w.numel, Kx=w.Kx, Ku=w.Ku, Kv=w.Kv, lr=w.lr,
                            beta1=w.beta1, beta2=w.beta2, eps=w.eps, rho=w.rho, x=mem.table(mem.x),
                            u=mem.table(mem.u), v=mem.table(mem.v), g=mem.table(mem.g), vmax=mem.table(mem.vmax),
                            grad_dtype=B.BF16 if w.grad_bf16 else B.F32, flags=w.flags, init_mode=B.INIT_AS_IS,
                            stream=sptr)
        probe = {"offset_gib": off / (1 << 30)}
        for name, t in (("ungated_ms", t_plain), ("gated_ms", t_gated)):
            if not t:
                continue
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            B.desloc_step(ctx, t)
            ev[0].record(s)
            for _ in range(2):
                B.desloc_step(ctx, t)
            ev[1].record(s)
            B.desloc_synchronize(ctx)
            probe[name] = ev[0].elapsed_time(ev[1]) / 2
        B.desloc_destroy(ctx)
        probes.append(probe)
        del mem
    pool.zero_()  # the probes wrote into it
    torch.cuda.synchronize()
    best = min(range(len(probes)), key=lambda i: probes[i]["ungated_ms"] + probes[i].get("gated_ms", 0.0))
    return pool, offsets[best], probes


class DeslocSession:
    """A workload resident on the GPU plus its library context."""

    def __init__(self, w: Workload, device="cuda:0", chunk_elems: int = 0,
                 init_mode: int = B.INIT_BROADCAST_REPLICA0, stream: Optional[torch.cuda.Stream] = None,
                 layout: str = "grouped", placement_pool_gib: float = 0.0, placement_candidates: int = 12,
                 group_bytes: int = 0, snapshots: Tuple[str, ...] = ()):
        """layout: "grouped" (GroupedReplicas, the fastest), "packed" (PackedReplicas: one record of
        whole arrays per replica) or "separate" (SeparateReplicas: every tensor its own allocation).
        placement_pool_gib > 0 (packed layout only): allocate one pool of that size, time the step
        with the records placed at `placement_candidates` offsets inside it and keep the fastest
        placement (see search_placement); the rest of the pool stays allocated but unused.
        group_bytes (grouped layout only): bytes per array and replica of a group of tensors, 0 = default.
        snapshots (grouped layout only): states that get a snapshot array inside every group."""
        self.w = w
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.stream = stream
        self.placement = None
        has_v, has_vmax = w.variant != B.SGDM, bool(w.flags & B.FLAG_AMSGRAD)
        if layout == "packed" and placement_pool_gib > 0:
            pool, offset, probes = search_placement(w, stream, int(placement_pool_gib * (1 << 30)),
                                                    placement_candidates)
            self.mem = PackedReplicas(w.numel, w.M, has_v, w.grad_bf16, device, has_vmax=has_vmax,
                                      pool=pool, pool_offset=offset)
            self.placement = {"pool_gib": pool.numel() / (1 << 30), "offset_gib": offset / (1 << 30),
                              "probes": probes}
        else:
            cls = {"packed": PackedReplicas, "separate": SeparateReplicas, "grouped": GroupedReplicas}[layout]
            extra = {"group_bytes": group_bytes, "snapshots": tuple(snapshots)} if layout == "grouped" else {}
            self.mem = cls(w.numel, w.M, has_v, w.grad_bf16, device, has_vmax=has_vmax, **extra)
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
        gen.fill(self.mem.x0_destination().data_ptr(), False, self.mem.total, self.d_starts.data_ptr(),
                 self.d_x0scale.data_ptr(), w.n_tensors, 0, 0.0, 0.0, w.seed, 0, 0,
                 gen.PURPOSE_X0, self._stream_ptr())
        self._after_generator(self.mem.x0_written)

    def fill_gradients(self, t: int) -> None:
        """g_t^m for every replica m from the counter-based generator."""
        w = self.w
        for m in range(w.M):
            gen.fill(self.mem.grad_destination(m).data_ptr(), w.grad_bf16, self.mem.total, self.d_starts.data_ptr(),
                     self.d_scale.data_ptr(), w.n_tensors, w.dist, w.grad_mean0,
                     w.grad_mean_per_replica, w.seed, t, m, gen.PURPOSE_GRAD, self._stream_ptr())
            self._after_generator(lambda m=m: self.mem.grads_written(m))

    def _after_generator(self, scatter) -> None:
        """Runs a layout's scatter copies (torch work) after the generator kernel on our stream."""
        if isinstance(self.mem, PackedReplicas):
            return
        if self.stream is not None:
            with torch.cuda.stream(self.stream):
                scatter()
        else:
            scatter()

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
