"""The packed layout of the runtime (CPU: torch only allocates here, nothing of the method runs)."""
import numpy as np
import pytest
import torch

from paper_2505_22549_amd.runtime import PackedReplicas

NUMEL = np.array([1000, 70000, 0, 3], dtype=np.uint64)


@pytest.mark.parametrize("grad_bf16", [False, True])
@pytest.mark.parametrize("has_v,has_vmax", [(True, False), (True, True), (False, False)])
def test_replica_records_hold_the_arrays_back_to_back(grad_bf16, has_v, has_vmax):
    M = 3
    mem = PackedReplicas(NUMEL, M, has_v, grad_bf16, device="cpu", has_vmax=has_vmax)
    assert mem.stride % 16384 == 0 and mem.stride >= int(NUMEL.sum())
    assert mem.record_bytes % 65536 == 0
    assert mem.pool.numel() == M * mem.record_bytes == PackedReplicas.bytes_needed(NUMEL, M, has_v, grad_bf16, has_vmax)
    base = mem.pool.data_ptr()
    names = ["x", "u"] + (["v"] if has_v else []) + (["vmax"] if has_vmax else []) + ["g"]
    assert mem.v is None or has_v
    assert mem.vmax is None or has_vmax
    spans = []
    for m in range(M):
        expect = m * mem.record_bytes
        for n in names:
            row = mem.array(n)[m]
            es = row.element_size()
            assert row.is_contiguous() and row.numel() == mem.stride
            assert row.data_ptr() - base == expect
            if n != "g":
                assert (row.data_ptr() - base) % 65536 == 0   # every fp32 stream congruent modulo 64 KiB
            spans.append((row.data_ptr() - base, row.data_ptr() - base + mem.stride * es))
            expect += mem.stride * es
        assert expect <= (m + 1) * mem.record_bytes
    spans.sort()
    assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))  # no two rows overlap
    assert (mem.g.dtype == torch.bfloat16) == grad_bf16


def test_pointer_table_follows_the_records():
    M = 4
    mem = PackedReplicas(NUMEL, M, True, True, device="cpu")
    starts = np.concatenate(([0], np.cumsum(NUMEL)[:-1])).astype(np.uint64)
    for name, es in (("x", 4), ("u", 4), ("v", 4), ("g", 2)):
        t = mem.array(name)
        tab = mem.table(t).reshape(M, len(NUMEL))
        for m in range(M):
            assert (tab[m] == np.uint64(t[m].data_ptr()) + starts * np.uint64(es)).all()
    assert mem.table(None) is None


def test_placement_inside_a_pool():
    M = 2
    need = PackedReplicas.bytes_needed(NUMEL, M, True, False)
    pool = torch.zeros(need + 3 * PackedReplicas.ALIGN + 3, dtype=torch.uint8)  # odd length on purpose
    mem = PackedReplicas(NUMEL, M, True, False, device="cpu", pool=pool, pool_offset=PackedReplicas.ALIGN)
    first = (-pool.data_ptr()) % PackedReplicas.ALIGN + PackedReplicas.ALIGN
    assert mem.x[0].data_ptr() - pool.data_ptr() == first
    assert mem.x[0].data_ptr() % PackedReplicas.ALIGN == 0
    mem.x[1, :3] = 5.0
    at = (first + mem.record_bytes) // 4
    assert pool[:-3].view(torch.float32)[at:at + 4].tolist() == [5.0, 5.0, 5.0, 0.0]
    with pytest.raises(AssertionError):
        PackedReplicas(NUMEL, M, True, False, device="cpu", pool=pool, pool_offset=4 * PackedReplicas.ALIGN)


def test_groups_of_tensors_hold_every_replica_side_by_side():
    from paper_2505_22549_amd.runtime import GroupedReplicas
    numel = np.array([1000, 70000, 0, 3, 20000, 5], dtype=np.uint64)
    M = 3
    mem = GroupedReplicas(numel, M, True, True, device="cpu", has_vmax=True, group_bytes=300_000)
    assert mem.groups == [[0, 1, 2, 3], [4, 5]]       # 71003 elements fit in 300 kB, the next tensor does not
    base = mem.pool.data_ptr()
    names = ["x", "u", "v", "vmax", "g"]
    spans = []
    for grp in mem.groups:
        n_j = sum(int(numel[k]) for k in grp)
        for m in range(M):
            for n in names:
                arr = getattr(mem, n)[m]
                first = next(k for k in grp if numel[k])
                start = arr[first].data_ptr()
                if n != "g":
                    assert start % 65536 == 0            # every fp32 run starts on a 64 KiB boundary
                at = start
                for k in grp:                           # tensors of a group back to back
                    if numel[k]:
                        assert arr[k].data_ptr() == at and arr[k].is_contiguous() and arr[k].numel() == numel[k]
                        at += int(numel[k]) * arr[k].element_size()
                spans.append((start - base, at - base))
                assert at - start == n_j * arr[first].element_size()
    spans.sort()
    assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))
    # inside a group: replica 0's x, u, v, vmax, g, then replica 1's, ...
    x0, u0, g0, x1 = (getattr(mem, n)[m][0].data_ptr() for n, m in (("x", 0), ("u", 0), ("g", 0), ("x", 1)))
    assert x0 < u0 < g0 < x1
    # the pointer table lists them tensor by tensor; empty tensors get a non-null dummy
    tab = mem.table(mem.x).reshape(M, len(numel))
    assert tab[1, 4] == mem.x[1][4].data_ptr() and tab[0, 2] == 0x10
    # a snapshot buffer arranged like the array itself
    buf, stab = mem.snapshot_buffer("u")
    stab = stab.reshape(M, len(numel))
    lo, hi = buf.data_ptr(), buf.data_ptr() + buf.numel()
    for m in range(M):
        for k in range(len(numel)):
            if numel[k]:
                assert lo <= stab[m, k] and stab[m, k] + int(numel[k]) * 4 <= hi
    assert stab[0, 1] - stab[0, 0] == 4000 and stab[0, 0] % 65536 == 0 and stab[1, 4] % 65536 == 0


def test_snapshot_arrays_inside_the_groups():
    from paper_2505_22549_amd.runtime import GroupedReplicas
    numel = np.array([1000, 70000, 0, 3, 20000, 5], dtype=np.uint64)
    M = 3
    mem = GroupedReplicas(numel, M, True, False, device="cpu", group_bytes=300_000, snapshots=("u", "x"))
    plain = GroupedReplicas(numel, M, True, False, device="cpu", group_bytes=300_000)
    assert mem.bytes > plain.bytes and plain.array("snap_u") is None
    buf, tab = mem.snapshot_buffer("u")
    assert buf is mem.pool
    tab = tab.reshape(M, len(numel))
    for m in range(M):
        for k in range(len(numel)):
            if numel[k]:
                assert tab[m, k] == mem.snap_u[m][k].data_ptr()
    # after the replica's own g and before the next replica's x, on a 64 KiB boundary, laid out like u
    g0, s0, sx0, x1 = (getattr(mem, n)[m][0].data_ptr() for n, m in (("g", 0), ("snap_u", 0), ("snap_x", 0), ("x", 1)))
    assert g0 < s0 < sx0 < x1 and s0 % 65536 == 0
    assert tab[0, 1] - tab[0, 0] == 4000
    # a state without a reserved array still gets a buffer of its own
    vbuf, _ = mem.snapshot_buffer("v")
    assert vbuf is not mem.pool
    with pytest.raises(AssertionError):
        GroupedReplicas(numel, M, False, False, device="cpu", snapshots=("v",))   # SGDM has no v


def test_packed_and_separate_snapshot_buffers():
    from paper_2505_22549_amd.runtime import SeparateReplicas
    mem = PackedReplicas(NUMEL, 2, True, False, device="cpu")
    buf, tab = mem.snapshot_buffer("u")
    assert buf.shape == (2, mem.stride) and tab[0] == buf.data_ptr()
    sep = SeparateReplicas(NUMEL, 2, True, False, device="cpu")
    buf, tab = sep.snapshot_buffer("x")
    tab = tab.reshape(2, len(NUMEL))
    assert tab[0, 1] - tab[0, 0] == 4000 and tab[1, 0] - tab[0, 0] == buf.stride(0) * 4


@pytest.mark.parametrize("layout", ["grouped", "separate"])
def test_staging_copies_round_trip(layout):
    from paper_2505_22549_amd.runtime import GroupedReplicas, SeparateReplicas
    numel = np.array([1000, 70000, 0, 3, 20000, 5, 0], dtype=np.uint64)
    tot, M = int(numel.sum()), 3
    mem = (GroupedReplicas(numel, M, True, True, device="cpu", group_bytes=300_000) if layout == "grouped"
           else SeparateReplicas(numel, M, True, True, device="cpu"))
    for m in range(M):
        mem.grad_destination(m)[:] = (torch.arange(tot) % 251 + m).to(torch.bfloat16)
        mem.grads_written(m)
    packed = mem.packed_view("g")
    for m in range(M):
        assert torch.equal(packed[m, :tot], (torch.arange(tot) % 251 + m).to(torch.bfloat16))
        at = 0
        for k, n in enumerate(int(v) for v in numel):   # the per-tensor views see the same data
            assert torch.equal(mem.g[m][k], packed[m, at:at + n])
            at += n
    mem.x0_destination()[:] = torch.arange(tot).float()
    mem.x0_written()
    assert torch.equal(mem.packed_view("x")[0, :tot], torch.arange(tot).float())
    assert not mem.packed_view("x")[1:].any()
