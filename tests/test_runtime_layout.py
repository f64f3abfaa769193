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
