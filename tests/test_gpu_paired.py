"""GPU parity of the paired mapping: strided layouts whose fp32 streams all start at the same
offset modulo 64 KiB hand out whole 64 KiB groups so that the halves of each vector access lie
32 KiB apart.  Every element must still be updated exactly once and exactly as the oracle does,
whatever the phase, the head before the first boundary and the tail after the last one."""
import numpy as np
import pytest

import oracle as O
from paper_2505_22549_amd import binding as B
from test_gpu_parity import HYP, HostCase

pytestmark = pytest.mark.gpu

G = 16384  # elements per group


def _run(orc, variant, M, numel, phase, T, flags=0, bf16=False, Ks=None, seed=0, packed=True):
    Ks = Ks or ((2, 3, 5) if variant != O.SGDM else (2, 3, 0))
    case = HostCase(variant, M, numel, Ks, HYP[variant], flags=flags, bf16=bf16, seed=seed,
                    phase_bytes=phase, packed=packed)
    info = B.desloc_get_plan(case.ctx)
    nbit = case.run(orc, T)
    case.close()
    return info, nbit


@pytest.mark.parametrize("M", [1, 3, 4, 8])
@pytest.mark.parametrize("variant", [O.ADAM, O.ADOPT, O.SGDM])
def test_paired_mapping_every_mask_class(orc, variant, M):
    # two whole groups, a ragged tail, several tensors packed into the segment
    numel = [G + 5, 3, G - 8 + 777, 1, 50]
    info, nbit = _run(orc, variant, M, numel, 0, 31, seed=300 + 10 * variant + M)
    assert info.strided == 1 and info.paired_numel == 2 * G
    assert info.n_chunks == 2 * 64 + -(-(sum(numel) - 2 * G) // 256)
    print(f"paired, variant {variant}, M {M}: {nbit} elements not bit-identical")


@pytest.mark.parametrize("phase", [16, 4096, 32768, 65536 - 16])
def test_paired_mapping_with_a_head_before_the_first_boundary(orc, phase):
    # phase p: the first (65536 - p) / 4 elements precede the first 64 KiB boundary
    head = (65536 - phase) // 4
    numel = [head + 3 * G + 1234 + 3]
    info, _ = _run(orc, O.ADAM, 4, numel, phase, 11, seed=phase)
    assert info.paired_numel == 3 * G
    info, _ = _run(orc, O.ADOPT, 5, numel, phase, 11, seed=phase + 1,
                   flags=B.FLAG_ADOPT_INIT_G0SQ)
    assert info.paired_numel == 3 * G


@pytest.mark.parametrize("n,groups", [(G, 1), (G - 4, 0), (G + 1, 1), (2 * G - 1, 1), (4 * G, 4)])
def test_paired_mapping_boundary_sizes(orc, n, groups):
    info, _ = _run(orc, O.ADAM, 4, [n], 0, 7, seed=n)
    assert info.paired_numel == groups * G


def test_paired_mapping_bf16_gradients_and_norm_clip(orc):
    # bf16 gradient arrays are exempt from the phase condition: give them another phase
    numel = [2 * G + 300, 17]
    case = HostCase(O.SGDM, 4, numel, (2, 3, 0), HYP[O.SGDM], bf16=True, seed=5, phase_bytes=0)
    assert B.desloc_get_plan(case.ctx).paired_numel == 2 * G
    case.run(orc, 9)
    case.close()
    info, _ = _run(orc, O.ADAM, 4, numel, 256, 9, flags=B.FLAG_NORM_CLIP, seed=6)
    assert info.paired_numel == 1 * G  # the 256-byte phase costs the first group


@pytest.mark.parametrize("flags", [B.FLAG_POST_AVERAGE, B.FLAG_POST_AVERAGE | B.FLAG_AMSGRAD])
@pytest.mark.parametrize("M", [3, 4])
def test_paired_mapping_update_then_average(orc, flags, M):
    info, _ = _run(orc, O.ADAM, M, [G + 100, 2 * G + 7], 0, 11, flags=flags, seed=40 + M + flags)
    assert info.paired_numel == 3 * G


@pytest.mark.parametrize("M", [1, 3, 4, 8])
@pytest.mark.parametrize("variant", [O.ADAM, O.ADOPT, O.SGDM])
def test_paired_records_of_separately_allocated_tensors(orc, variant, M):
    # table layouts: every tensor a segment of its own; those whose streams are congruent modulo 64 KiB
    # get paired chunk records for their whole groups (two wave slots per record: both for one workgroup
    # on steps without a gate, one each on gated steps)
    numel = [G + 5, 3, 2 * G + 777, 0, 100, G]
    info, nbit = _run(orc, variant, M, numel, 0, 31, seed=500 + 10 * variant + M, packed=False)
    assert info.strided == 0 and info.n_segments == 5 and info.paired_numel == 4 * G
    assert info.n_chunks == 4 * 32 + 1 + 1 + 2 + 1  # paired records + tails / small tensors (512-element records)
    info, _ = _run(orc, variant, M, numel, 4096, 13, seed=600 + 10 * variant + M, packed=False)
    assert info.paired_numel == 1 * G  # the head of (65536 - 4096) / 4 elements leaves one group in the third tensor


def test_paired_records_with_norm_clip_bf16_and_update_then_average(orc):
    numel = [2 * G + 300, 17, G + 1]
    info, _ = _run(orc, O.ADAM, 4, numel, 0, 9, flags=B.FLAG_NORM_CLIP, seed=71, packed=False)
    assert info.paired_numel == 3 * G
    info, _ = _run(orc, O.SGDM, 4, numel, 0, 9, bf16=True, seed=72, packed=False)
    assert info.paired_numel == 3 * G
    info, _ = _run(orc, O.ADAM, 3, numel, 0, 9, flags=B.FLAG_POST_AVERAGE | B.FLAG_AMSGRAD, seed=73, packed=False)
    assert info.paired_numel == 3 * G
    info, _ = _run(orc, O.ADAM, 8, numel, 0, 9, flags=B.FLAG_POST_AVERAGE, seed=74, packed=False)
    assert info.paired_numel == 3 * G
    # a chunk size chosen by the caller keeps plain records
    case = HostCase(O.ADAM, 4, numel, (2, 3, 5), HYP[O.ADAM], seed=75, phase_bytes=0, packed=False, chunk_elems=1024)
    assert B.desloc_get_plan(case.ctx).paired_numel == 0
    case.run(orc, 7)
    case.close()


def test_plan_reports_granted_occupancy(orc):
    case = HostCase(O.ADAM, 4, [4 * G], (4, 8, 16), HYP[O.ADAM], seed=1, phase_bytes=0)
    info = B.desloc_get_plan(case.ctx)
    case.close()
    # the dynamic-LDS request is there to cap the resident single-wave workgroups per compute
    # unit; the runtime must grant exactly what the request aims at
    assert list(info.resident_workgroups) == list(info.intended_workgroups) == [13, 9]
    # the same with a chunk size of the caller's: the strided path for every launch
    case = HostCase(O.ADAM, 4, [4 * G], (4, 8, 16), HYP[O.ADAM], seed=1, phase_bytes=0, chunk_elems=1024)
    info = B.desloc_get_plan(case.ctx)
    case.close()
    assert list(info.resident_workgroups) == list(info.intended_workgroups) == [10, 9]
    # separately allocated tensors (table path): 13 without a gate
    case = HostCase(O.ADAM, 4, [4 * G, 100], (4, 8, 16), HYP[O.ADAM], seed=1, phase_bytes=0, packed=False)
    info = B.desloc_get_plan(case.ctx)
    case.close()
    assert info.strided == 0
    assert list(info.resident_workgroups) == list(info.intended_workgroups) == [13, 8]
