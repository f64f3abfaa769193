"""CPU-only checks of the C ABI: every declared symbol is exported, the schedule
function matches the oracle bit for bit, and the host planning / validation logic
behaves as the header says.  No GPU compute is called here."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

import oracle as O
from conftest import ROOT

B = pytest.importorskip("paper_2505_22549_amd.binding")

if not os.path.exists(B.LIBRARY):  # the driver builds before testing; be loud if it did not
    pytest.fail(f"{B.LIBRARY} missing: run python -c 'import __graft_entry__ as g; g.build()'",
                pytrace=False)


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "desloc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(desloc_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert {"desloc_init", "desloc_step", "desloc_sync_mask", "desloc_read_state"} <= set(names)
    lib = ctypes.CDLL(B.LIBRARY)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/desloc.h but not exported"


def test_inputs_library_exports():
    from paper_2505_22549_amd.inputs import generator as G
    lib = ctypes.CDLL(G.LIBRARY)
    for n in ("desloc_inputs_fill", "desloc_inputs_philox_raw", "desloc_inputs_philox_host"):
        assert hasattr(lib, n)


def test_version_and_strerror():
    assert B.desloc_version() == 100
    for s in range(0, -8, -1):
        assert B.desloc_strerror(s) and "unknown" not in B.desloc_strerror(s)
    assert "unknown" in B.desloc_strerror(-99)


@pytest.mark.parametrize("Ks", [(16, 32, 64), (32, 96, 192), (64, 192, 384), (128, 384, 768),
                                (1, 1, 1), (0, 0, 0), (3, 0, 7), (5, 7, 11), (2, 2, 0)])
def test_sync_mask_matches_oracle_bit_exact(orc, Ks):
    cfg = O.Config(O.ADAM, 2, *Ks)
    L = math.lcm(*[k for k in Ks if k]) if any(Ks) else 10
    T = min(2 * L + 3, 5000)
    got = [B.desloc_sync_mask_k(t, *Ks) for t in range(T)]
    want = [orc.sync_mask(cfg, t) for t in range(T)]
    assert got == want
    big = [2 ** 40 + 5, 2 ** 63 - 1, 2 ** 64 - 1, 3 * 2 ** 33]
    assert [B.desloc_sync_mask_k(t, *Ks) for t in big] == [orc.sync_mask(cfg, t) for t in big]


def test_sync_mask_null_ctx_is_zero():
    assert B.lib().desloc_sync_mask(None, 0) == 0


# ---- planning: pointer values are compared, never dereferenced, so fake addresses do ----

def _plan(numel, M=2, variant=B.ADAM, base=0x10000000, gap=0, stride=None, gdt=B.F32, **kw):
    numel = np.asarray(numel, dtype=np.uint64)
    total = int(numel.sum()) + gap * len(numel)
    stride = stride or (total * 4 + 4096) // 16 * 16

    def tab(off, es):
        starts = np.concatenate(([0], np.cumsum(numel + np.uint64(gap))[:-1])).astype(np.uint64)
        rep = (np.arange(M, dtype=np.uint64) * np.uint64(stride))[:, None]
        return (np.uint64(base + off) + rep + starts[None, :] * np.uint64(es)).reshape(-1)

    big = 1 << 34
    args = dict(variant=variant, M=M, numel=numel, Kx=1, Ku=1, Kv=1, lr=1e-3, beta1=0.9, beta2=0.999,
                eps=1e-8, rho=float("inf"), x=tab(0, 4), u=tab(big, 4),
                v=None if variant == B.SGDM else tab(2 * big, 4),
                g=tab(3 * big, 2 if gdt == B.BF16 else 4), grad_dtype=gdt)
    args.update(kw)
    return B.desloc_plan(**args)


def test_plan_merges_packed_tensors_into_one_segment():
    info = _plan([5, 7, 1000, 3, 4096, 1])
    assert info.n_segments == 1
    assert info.total_numel == 5 + 7 + 1000 + 3 + 4096 + 1
    assert info.chunk_elems % 256 == 0 and info.chunk_elems >= 256
    assert info.n_chunks == math.ceil(info.total_numel / info.chunk_elems)


def test_plan_keeps_gapped_tensors_apart():
    # a gap of 4 elements keeps every base 16-byte aligned but breaks adjacency
    numel = [8, 4096 * 2 + 4, 12, 4]
    info = _plan(numel, gap=4, chunk_elems=4096)
    assert info.n_segments == 4
    assert info.n_chunks == sum(math.ceil(n / 4096) for n in numel)


def test_plan_skips_empty_tensors_and_merges_across_them():
    info = _plan([16, 0, 16, 0, 0, 32])
    assert info.n_segments == 1 and info.total_numel == 64 and info.n_chunks == 1
    info = _plan([0, 0])
    assert info.n_segments == 0 and info.n_chunks == 0


def test_plan_default_chunk_follows_the_layout(monkeypatch):
    """One uniformly strided segment: addresses come from kernel arguments, one 256-element tile per
    workgroup.  Anything else reads chunk records: two tiles per record.  A non-uniform replica
    stride turns a single segment into a table layout too.  The production library reads no
    environment variables: the sweep switches of a -DDESLOC_TUNING build change nothing here."""
    packed = _plan([5, 7, 1000, 3, 4096, 1], M=4)
    assert packed.n_segments == 1 and packed.chunk_elems == 256
    gapped = _plan([8, 4096 * 2 + 4, 12, 4], gap=4, M=4)
    assert gapped.n_segments == 4 and gapped.chunk_elems == 512
    assert gapped.n_chunks == sum(math.ceil(n / 512) for n in [8, 4096 * 2 + 4, 12, 4])
    # replicas of x not equally spaced (third replica moved by 64 bytes)
    numel = np.array([4096], dtype=np.uint64)
    reps = np.array([0, 1 << 20, (2 << 20) + 64], dtype=np.uint64)
    even = np.array([0, 1 << 20, 2 << 20], dtype=np.uint64)
    args = dict(variant=B.SGDM, M=3, numel=numel, Kx=1, Ku=1, Kv=0, lr=1e-3, beta1=0.9, beta2=0.0, eps=1e-8,
                rho=float("inf"), x=np.uint64(0x10000000) + reps, u=np.uint64(0x20000000) + even, v=None,
                g=np.uint64(0x30000000) + even, grad_dtype=B.F32)
    uneven = B.desloc_plan(**args)
    assert uneven.n_segments == 1 and uneven.chunk_elems == 512
    assert packed.strided == 1 and gapped.strided == 0 and uneven.strided == 0
    monkeypatch.setenv("DESLOC_NO_STRIDED", "1")
    monkeypatch.setenv("DESLOC_NO_PAIRING", "1")
    monkeypatch.setenv("DESLOC_LDS_BYTES", "4096")
    same = _plan([5, 7, 1000, 3, 4096, 1], M=4)
    assert same.n_segments == 1 and same.chunk_elems == 256 and same.strided == 1
    assert list(same.lds_limiter_bytes) == list(packed.lds_limiter_bytes)


def test_plan_paired_mapping_needs_congruent_stream_bases():
    """Strided layouts whose fp32 streams all start at the same offset modulo 64 KiB hand out the
    elements between the first and the last 64 KiB boundary in 16384-element groups (64 single-wave
    workgroups each); what lies before and after is cut into contiguous 256-element chunks."""
    G = 16384
    n = 5 * G + 1000
    # aligned bases, stride a multiple of 64 KiB: everything but the tail is paired
    info = _plan([n], M=4, base=0x10000000, stride=(n + G - 1) // G * G * 4)
    assert info.strided == 1 and info.paired_numel == 5 * G
    assert info.n_chunks == 5 * 64 + math.ceil(1000 / 256)
    # a common phase of 4 KiB: the first 15360 elements form the head
    head = (65536 - 4096) // 4
    info = _plan([n], M=4, base=0x10000000 + 4096, stride=(n + G - 1) // G * G * 4)
    assert info.paired_numel == (n - head) // G * G
    tail = n - head - info.paired_numel
    assert info.n_chunks == info.paired_numel // 256 + math.ceil(head / 256) + math.ceil(tail / 256)
    # a stride that is not a multiple of 64 KiB, or one array out of phase: plain contiguous chunks
    assert _plan([n], M=4, stride=n * 4 + 4096).paired_numel == 0
    numel = np.array([n], dtype=np.uint64)
    reps = np.arange(4, dtype=np.uint64) * np.uint64(6 * G * 4)
    args = dict(variant=B.ADAM, M=4, numel=numel, Kx=1, Ku=1, Kv=1, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8,
                rho=1.0, x=np.uint64(0x10000000) + reps, u=np.uint64(0x30000000) + reps,
                v=np.uint64(0x50000000) + reps, g=np.uint64(0x70000000) + reps, grad_dtype=B.F32)
    assert B.desloc_plan(**args).paired_numel == 5 * G
    args["v"] = np.uint64(0x50000000 + 512) + reps
    assert B.desloc_plan(**args).paired_numel == 0
    # bf16 gradients are exempt from the phase condition (8-byte alignment is all they need)
    args["v"] = None
    args.update(variant=B.SGDM, g=np.uint64(0x70000008) + reps // np.uint64(2), grad_dtype=B.BF16)
    assert B.desloc_plan(**args).paired_numel == 5 * G
    # a single replica has no stride to satisfy; too short a tensor has no whole group
    assert _plan([n], M=1).paired_numel == 5 * G
    assert _plan([G - 4], M=2, stride=G * 4).paired_numel == 0
    # a chunk size chosen by the caller keeps the contiguous decomposition
    assert _plan([n], M=4, stride=6 * G * 4, chunk_elems=1024).paired_numel == 0


def test_plan_reports_the_occupancy_limiters():
    info = _plan([4096], M=4)
    # one strided segment: launches without a gate read chunk records like a table layout (13 resident
    # workgroups per CU), gated launches form their addresses from kernel arguments (9)
    assert list(info.lds_limiter_bytes) == [12500, 17500]
    assert list(info.intended_workgroups) == [160 * 1024 // 12500, 160 * 1024 // 17500] == [13, 9]
    assert list(info.resident_workgroups) == [0, 0]  # not queried without a GPU
    assert info.gated_chunk_elems == 256
    sg = _plan([4096], M=4, variant=B.SGDM)
    assert sg.lds_limiter_bytes[0] == 12500 and sg.intended_workgroups[0] == 13
    # a chunk size chosen by the caller keeps the contiguous strided decomposition for every launch
    own = _plan([4096], M=4, chunk_elems=1024)
    assert list(own.lds_limiter_bytes) == [15500, 17500] and list(own.intended_workgroups) == [10, 9]
    assert _plan([4096], M=4, variant=B.SGDM, chunk_elems=1024).lds_limiter_bytes[0] == 11500
    # table layouts (here: two tensors with a gap): 13 resident workgroups without a gate, any variant
    for variant in (B.ADAM, B.SGDM):
        numel = np.array([4096, 4096], dtype=np.uint64)
        off = np.array([[0, 5000 * 4], [1 << 20, (1 << 20) + 5000 * 4]], dtype=np.uint64).reshape(-1)
        tb = B.desloc_plan(variant=variant, M=2, numel=numel, Kx=1, Ku=1, Kv=0 if variant == B.SGDM else 1, lr=1e-3,
                           beta1=0.9, beta2=0.999, eps=1e-8, rho=1.0, x=np.uint64(0x10000000) + off,
                           u=np.uint64(0x20000000) + off, v=None if variant == B.SGDM else np.uint64(0x30000000) + off,
                           g=np.uint64(0x40000000) + off, grad_dtype=B.F32)
        assert tb.strided == 0 and tb.n_segments == 2
        # M = 2 runs the runtime replica loop: 12 resident workgroups on gated steps
        assert list(tb.lds_limiter_bytes) == [12500, 13000] and list(tb.intended_workgroups) == [13, 12]


def test_gated_occupancy_on_table_layouts_follows_the_distance_between_replicas():
    numel = np.array([1 << 20, 1 << 20], dtype=np.uint64)

    def plan(replica_gap):
        off = np.array([[0, (1 << 22) + 4096], [replica_gap, replica_gap + (1 << 22) + 4096],
                        [2 * replica_gap, 2 * replica_gap + (1 << 22) + 4096],
                        [3 * replica_gap, 3 * replica_gap + (1 << 22) + 4096]], dtype=np.uint64).reshape(-1)
        return B.desloc_plan(variant=B.ADAM, M=4, numel=numel, Kx=1, Ku=1, Kv=1, lr=1e-3, beta1=0.9, beta2=0.999,
                             eps=1e-8, rho=1.0, x=np.uint64(1 << 40) + off, u=np.uint64(1 << 41) + off,
                             v=np.uint64(3 << 40) + off, g=np.uint64(1 << 42) + off, grad_dtype=B.F32)

    far = plan(1 << 30)       # arrays a TiB apart: a gated launch sweeps streams far from each other
    assert far.strided == 0 and list(far.lds_limiter_bytes) == [12500, 17500]
    # everything of one segment within 8 GiB: x, u, v, g of four replicas 64 MiB apart
    off = np.array([[m * (64 << 20), m * (64 << 20) + (1 << 22) + 4096] for m in range(4)], dtype=np.uint64).reshape(-1)
    near = B.desloc_plan(variant=B.ADAM, M=4, numel=numel, Kx=1, Ku=1, Kv=1, lr=1e-3, beta1=0.9, beta2=0.999,
                         eps=1e-8, rho=1.0, x=np.uint64(1 << 40) + off, u=np.uint64((1 << 40) + (16 << 20)) + off,
                         v=np.uint64((1 << 40) + (32 << 20)) + off, g=np.uint64((1 << 40) + (48 << 20)) + off,
                         grad_dtype=B.F32)
    assert near.strided == 0 and list(near.lds_limiter_bytes) == [12500, 20000]
    assert list(near.intended_workgroups) == [13, 8]


def test_plan_rejects_more_workgroups_than_a_launch_holds():
    # 2^26 - 1 single-wave workgroups fit in one launch dimension; launches without a gate use two
    # workgroups per two-tile chunk record, so an even number of tiles is the most that fits
    limit = (1 << 26) - 1
    ok = _plan([(limit - 1) * 256], M=1)
    assert ok.n_chunks == limit - 1
    for n in (limit * 256, limit * 256 + 1):
        with pytest.raises(B.DeslocError) as e:
            _plan([n], M=1, stride=(limit * 256 + 4096) * 4 + 4096)
        assert e.value.status == B.ERR_BAD_ARG
    assert _plan([limit * 256 + 1], M=1, chunk_elems=1024).n_chunks == math.ceil((limit * 256 + 1) / 1024)


def test_plan_chunk_size_argument():
    info = _plan([10000], chunk_elems=1024)
    assert info.n_chunks == 10 and info.chunk_elems == 1024
    for bad in (1000, 128, 384, (1 << 20) + 256):
        with pytest.raises(B.DeslocError) as e:
            _plan([10000], chunk_elems=bad)
        assert e.value.status == B.ERR_BAD_ARG


def test_plan_alignment_errors():
    with pytest.raises(B.DeslocError) as e:
        _plan([8, 8], base=0x10000004)
    assert e.value.status == B.ERR_ALIGN
    # odd tensor followed by a gap: second segment base is misaligned
    with pytest.raises(B.DeslocError) as e:
        _plan([5, 8], gap=2)
    assert e.value.status == B.ERR_ALIGN
    # bf16 gradients need only 8-byte alignment for g, and merging uses 2-byte elements
    info = _plan([6, 10, 4], gdt=B.BF16, variant=B.SGDM)
    assert info.n_segments == 1


@pytest.mark.parametrize("kw,status", [
    (dict(M=0), B.ERR_BAD_ARG), (dict(M=1025), B.ERR_BAD_ARG), (dict(variant=3), B.ERR_BAD_ARG),
    (dict(beta1=1.0), B.ERR_BAD_ARG), (dict(beta2=-0.1), B.ERR_BAD_ARG), (dict(eps=0.0), B.ERR_BAD_ARG),
    (dict(rho=0.0), B.ERR_BAD_ARG), (dict(rho=float("nan")), B.ERR_BAD_ARG),
    (dict(lr=float("inf")), B.ERR_BAD_ARG), (dict(flags=64), B.ERR_BAD_ARG),
    (dict(flags=B.FLAG_ADOPT_INIT_G0SQ), B.ERR_VARIANT), (dict(init_mode=3), B.ERR_BAD_ARG),
    (dict(grad_dtype=2), B.ERR_BAD_ARG),
])
def test_plan_rejects_bad_arguments(kw, status):
    with pytest.raises(B.DeslocError) as e:
        if "M" in kw:
            M = kw.pop("M")
            # pointer tables sized for a legal M, then M overwritten
            m = B._Marshalled(variant=B.ADAM, M=2, numel=[8], Kx=1, Ku=1, Kv=1, lr=1e-3, beta1=0.9,
                              beta2=0.999, eps=1e-8, rho=1.0, x=[16, 160], u=[320, 480], v=[640, 800],
                              g=[960, 1120])
            m.cfg.M = M
            info = B.desloc_plan_info()
            B._check(B.lib().desloc_plan(ctypes.byref(m.cfg), ctypes.byref(info)), "desloc_plan")
        else:
            _plan([8], **kw)
    assert e.value.status == status


def test_plan_variant_array_rules():
    with pytest.raises(B.DeslocError) as e:  # SGDM must not get a v table
        _plan([8], variant=B.SGDM, v=np.array([4096, 8192], dtype=np.uint64))
    assert e.value.status == B.ERR_VARIANT
    with pytest.raises(B.DeslocError) as e:  # Adam needs one
        _plan([8], variant=B.ADAM, v=None)
    assert e.value.status == B.ERR_NULL
    with pytest.raises(B.DeslocError) as e:
        _plan([8], variant=B.ADOPT, flags=B.FLAG_ADAM_LITERAL)
    assert e.value.status == B.ERR_VARIANT
    info = _plan([8], variant=B.ADOPT, flags=B.FLAG_ADOPT_INIT_G0SQ | B.FLAG_ADOPT_AVG_NORMALISER)
    assert info.n_segments == 1


def test_plan_post_average_and_amsgrad_rules():
    vm = np.array([1 << 20, 1 << 21], dtype=np.uint64)
    info = _plan([8], variant=B.ADAM, flags=B.FLAG_POST_AVERAGE)
    assert info.n_segments == 1
    info = _plan([8], variant=B.SGDM, flags=B.FLAG_POST_AVERAGE)
    assert info.n_segments == 1
    info = _plan([8], variant=B.ADAM, flags=B.FLAG_POST_AVERAGE | B.FLAG_AMSGRAD, vmax=vm)
    assert info.n_segments == 1
    for kw, status in [
        (dict(variant=B.ADOPT, flags=B.FLAG_POST_AVERAGE), B.ERR_VARIANT),
        (dict(variant=B.ADAM, flags=B.FLAG_AMSGRAD, vmax=vm), B.ERR_VARIANT),          # needs POST_AVERAGE
        (dict(variant=B.SGDM, flags=B.FLAG_POST_AVERAGE | B.FLAG_AMSGRAD, vmax=vm), B.ERR_VARIANT),
        (dict(variant=B.ADAM, flags=B.FLAG_POST_AVERAGE | B.FLAG_AMSGRAD), B.ERR_NULL),  # no vmax table
        (dict(variant=B.ADAM, flags=B.FLAG_POST_AVERAGE, vmax=vm), B.ERR_VARIANT),       # vmax without the flag
    ]:
        with pytest.raises(B.DeslocError) as e:
            _plan([8], **kw)
        assert e.value.status == status, kw
    # a misaligned or non-adjacent vmax table splits / rejects like any other array
    with pytest.raises(B.DeslocError) as e:
        _plan([8], variant=B.ADAM, flags=B.FLAG_POST_AVERAGE | B.FLAG_AMSGRAD, vmax=vm + np.uint64(4))
    assert e.value.status == B.ERR_ALIGN


def test_plan_struct_size_is_checked():
    m = B._Marshalled(variant=B.ADAM, M=1, numel=[8], Kx=1, Ku=1, Kv=1, lr=1e-3, beta1=0.9,
                      beta2=0.999, eps=1e-8, rho=1.0, x=[16], u=[160], v=[320], g=[480])
    m.cfg.struct_size -= 4
    info = B.desloc_plan_info()
    assert B.lib().desloc_plan(ctypes.byref(m.cfg), ctypes.byref(info)) == B.ERR_BAD_ARG
    assert B.lib().desloc_plan(None, ctypes.byref(info)) == B.ERR_NULL
    assert B.lib().desloc_step(None, 0) == B.ERR_NULL
    assert B.lib().desloc_destroy(None) == B.OK


def test_benchmark_tensor_lists_match_their_stated_sizes():
    from paper_2505_22549_amd.inputs import recipes as R
    want = {1: (1, 1048576), 2: (148, 124439808), 3: (292, 354823168), 5: (218, 1713639424)}
    for i, (nt, total) in want.items():
        w = R.CONFIGS[i]()
        assert (w.n_tensors, w.total_numel) == (nt, total)
    w4 = R.config4()
    assert w4.n_tensors == 7000 and 64 <= w4.numel.min() and w4.numel.max() < 262144
    assert 1.9e8 < w4.total_numel < 2.5e8
    # a packed list of thousands of small tensors is a single segment
    info = _plan(w4.numel, M=4, variant=B.SGDM, gdt=B.BF16, stride=1 << 31)
    assert info.n_segments == 1 and info.n_chunks == math.ceil(w4.total_numel / info.chunk_elems)


def test_philox_known_answers():
    # Known-answer vectors of Philox4x32-10 (Random123 distribution, kat_vectors).
    from paper_2505_22549_amd.inputs import generator as G
    kat = [
        ([0, 0, 0, 0], [0, 0], [0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8]),
        ([0xffffffff] * 4, [0xffffffff] * 2, [0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd]),
        ([0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344], [0xa4093822, 0x299f31d0],
         [0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1]),
    ]
    for c, k, want in kat:
        assert G.philox_host(c, k).tolist() == want
        assert G.philox4x32_10_numpy(np.array([c]), np.array([k]))[0].tolist() == want
