"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs, element by element.

Bar: sync schedule bit-exact; fp32 state within max relative error 1e-5 (absolute
1e-7 near zero).  The kernels are built without fp contraction and with correctly
rounded divide / sqrt, so the difference is normally zero; the number of elements that
are not bit-identical is printed for information.
"""
import math

import numpy as np
import pytest
import torch

import oracle as O
from paper_2505_22549_amd import binding as B
from paper_2505_22549_amd.inputs import generator as G
from paper_2505_22549_amd.inputs import recipes as R
from paper_2505_22549_amd.runtime import DeslocSession

pytestmark = pytest.mark.gpu

RTOL, ATOL = 1e-5, 1e-7
DEV = "cuda:0"


def assert_parity(got, want, what):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite GPU values"
    err = np.abs(got - want)
    ok = (err <= RTOL * np.abs(want)) | (err <= ATOL)
    if not ok.all():
        i = int(np.argmax(np.where(ok, 0, err)))
        raise AssertionError(f"{what}: {(~ok).sum()} of {ok.size} elements out of tolerance; worst at "
                             f"flat index {i}: gpu {got.flat[i]!r} oracle {want.flat[i]!r}")
    return int((got != want).sum())


def _stride(n):
    """Replica stride in elements: a multiple of 8 (16-byte aligned rows for fp32 and bf16)
    with some padding after the last tensor."""
    return (n + 7) // 8 * 8 + 24


class HostCase:
    """Small case with host-generated inputs: tensors either packed (one segment) or
    separately allocated (one segment per tensor, ragged tails, gaps)."""

    def __init__(self, variant, M, numel, Ks, hyp, flags=0, bf16=False, packed=True, seed=0,
                 distinct_start=True, chunk_elems=0, phase_bytes=None):
        """phase_bytes: every array of every replica (packed layouts: with a replica stride that is a
        multiple of 64 KiB of fp32) or every separately allocated tensor starts `phase_bytes` past a
        64 KiB boundary: the condition for the library's paired mapping."""
        self.variant, self.M, self.numel, self.Ks = variant, M, list(numel), Ks
        self.bf16, self.flags = bf16, flags
        self.N = int(sum(numel))
        rng = np.random.default_rng(seed)
        self.rng = rng
        lr, b1, b2, eps, rho = hyp
        f32 = lambda v: float(np.float32(v))
        self.cfg = O.Config(variant, M, *Ks, lr=f32(lr), beta1=f32(b1), beta2=f32(b2), eps=f32(eps),
                            rho=f32(rho), adam_literal=bool(flags & B.FLAG_ADAM_LITERAL),
                            adopt_avg_normaliser=bool(flags & B.FLAG_ADOPT_AVG_NORMALISER),
                            adopt_init_g0sq=bool(flags & B.FLAG_ADOPT_INIT_G0SQ),
                            norm_clip=bool(flags & B.FLAG_NORM_CLIP),
                            post_average=bool(flags & B.FLAG_POST_AVERAGE),
                            amsgrad=bool(flags & B.FLAG_AMSGRAD))
        has_v = variant != O.SGDM
        N = self.N
        if distinct_start:  # resume-like state: replicas already differ
            self.x = (rng.normal(size=(M, N)) * 0.05).astype(np.float32)
            self.u = (rng.normal(size=(M, N)) * 0.01).astype(np.float32)
            self.v = (rng.random(size=(M, N)) * 1e-3).astype(np.float32) if has_v else None
        else:
            self.x = np.tile((rng.normal(size=N) * 0.05).astype(np.float32), (M, 1))
            self.u = np.zeros((M, N), np.float32)
            self.v = np.zeros((M, N), np.float32) if has_v else None
        self.vmax = None
        if flags & B.FLAG_AMSGRAD:  # running maximum starts at (or above) v, as vt_{-1} = v_{-1}
            self.vmax = (self.v * rng.choice([1.0, 3.0], size=self.v.shape)).astype(np.float32)
        dev = torch.device(DEV)
        gdt = torch.bfloat16 if bf16 else torch.float32
        self.dev_arrays = {}
        self.keep = []
        tables = {}
        for name, host, dt in (("x", self.x, torch.float32), ("u", self.u, torch.float32),
                               ("v", self.v, torch.float32), ("g", np.zeros((M, N), np.float32), gdt),
                               ("vmax", self.vmax, torch.float32)):
            if host is None:
                tables[name] = None
                continue
            if packed and phase_bytes is not None:
                S = (N + 16383) // 16384 * 16384
                es = 2 if dt == torch.bfloat16 else 4
                raw = torch.zeros(M * S * es + 2 * 65536 + phase_bytes, dtype=torch.uint8, device=dev)
                off = (-raw.data_ptr()) % 65536 + phase_bytes
                t = raw[off:off + M * S * es].view(dt).view(M, S)
                assert t.data_ptr() % 65536 == phase_bytes
                t[:, :N] = torch.from_numpy(host).to(dev).to(dt)
                self.dev_arrays[name] = [[t[m, s:s + n] for s, n in self._spans()] for m in range(M)]
                self.keep += [raw, t]
            elif packed:
                t = torch.zeros((M, _stride(N)), dtype=dt, device=dev)
                t[:, :N] = torch.from_numpy(host).to(dev).to(dt)
                self.dev_arrays[name] = [[t[m, s:s + n] for s, n in self._spans()] for m in range(M)]
                self.keep.append(t)
            else:
                per = []
                es = 2 if dt == torch.bfloat16 else 4
                for m in range(M):
                    row = []
                    for s, n in self._spans():
                        if phase_bytes is not None:  # every tensor `phase_bytes` past a 64 KiB boundary
                            raw = torch.zeros(max(n, 1) * es + 2 * 65536 + phase_bytes, dtype=torch.uint8, device=dev)
                            off = (-raw.data_ptr()) % 65536 + phase_bytes
                            tt = raw[off:off + max(n, 1) * es].view(dt)[:n]
                            self.keep.append(raw)
                        else:
                            tt = torch.zeros(max(n, 1) + 8, dtype=dt, device=dev)[:n]
                        tt.copy_(torch.from_numpy(host[m, s:s + n]).to(dt))
                        row.append(tt)
                    per.append(row)
                self.dev_arrays[name] = per
            tables[name] = np.array([[t.data_ptr() if t.numel() else 0x10 for t in row]
                                     for row in self.dev_arrays[name]], dtype=np.uint64).reshape(-1)
        torch.cuda.synchronize()
        self.ctx = B.desloc_init(variant=variant, M=M, numel=self.numel, Kx=Ks[0], Ku=Ks[1], Kv=Ks[2],
                                 lr=lr, beta1=b1, beta2=b2, eps=eps, rho=rho, x=tables["x"],
                                 u=tables["u"], v=tables["v"], g=tables["g"], vmax=tables["vmax"],
                                 grad_dtype=B.BF16 if bf16 else B.F32, flags=flags,
                                 init_mode=B.INIT_AS_IS, chunk_elems=chunk_elems)

    def _spans(self):
        s = 0
        for n in self.numel:
            yield s, n
            s += n

    def set_grads(self, g32: np.ndarray):
        """Uploads gradients; returns what the oracle must see (bf16 rounded then widened)."""
        gt = torch.from_numpy(g32).to(DEV)
        if self.bf16:
            gt = gt.to(torch.bfloat16)
        for m in range(self.M):
            for (s, n), dst in zip(self._spans(), self.dev_arrays["g"][m]):
                if n:
                    dst.copy_(gt[m, s:s + n])
        torch.cuda.synchronize()
        if self.bf16:
            bits = gt.view(torch.int16).cpu().numpy().view(np.uint16)
            return (bits.astype(np.uint32) << 16).view(np.float32)
        return g32

    def read(self, which):
        return np.stack([B.desloc_read_state(self.ctx, which, m, B.ALL_TENSORS, self.N)
                         for m in range(self.M)])

    def run(self, orc, T, t0=0, grad_scale=0.02, check_every=1):
        nbit = 0
        for t in range(t0, t0 + T):
            g32 = (self.rng.normal(size=(self.M, self.N)) * grad_scale
                   + 0.01 * np.arange(self.M)[:, None]).astype(np.float32)
            if t % 3 == 0:  # heavy-tailed step so that the clip fires when rho is finite
                g32 *= self.rng.choice([1.0, 50.0], size=g32.shape).astype(np.float32)
            g_or = self.set_grads(g32)
            assert B.desloc_sync_mask(self.ctx, t) == orc.sync_mask(self.cfg, t)
            B.desloc_step(self.ctx, t)
            norms = orc.step(self.cfg, t, self.x, self.u, self.v, np.ascontiguousarray(g_or),
                             vmax=self.vmax)
            if norms is not None:  # norm-based clipping: the library's norms are the oracle's
                got = B.desloc_read_grad_norms(self.ctx, self.M)
                np.testing.assert_allclose(got, norms, rtol=2e-7, atol=0)
                self.clipped_steps = getattr(self, "clipped_steps", 0) + int((norms > self.cfg.rho).sum())
                self.unclipped_steps = getattr(self, "unclipped_steps", 0) + int((norms <= self.cfg.rho).sum())
            if (t - t0) % check_every == 0 or t == t0 + T - 1:
                nbit += assert_parity(self.read(B.X), self.x, f"x after t={t}")
                nbit += assert_parity(self.read(B.U), self.u, f"u after t={t}")
                if self.v is not None:
                    nbit += assert_parity(self.read(B.V), self.v, f"v after t={t}")
                if self.vmax is not None:
                    nbit += assert_parity(self.read(B.VMAX), self.vmax, f"vmax after t={t}")
        return nbit

    def close(self):
        B.desloc_destroy(self.ctx)


HYP = {O.ADAM: (1e-3, 0.9, 0.999, 1e-8, 1.0), O.ADOPT: (2.1e-3, 0.9, 0.9999, 1e-6, 1.0),
       O.SGDM: (1e-2, 0.9, 0.0, 1e-8, float("inf"))}

# ragged sizes: several 1024-element tiles, a partial tile, a partial 4-vector, tiny tensors
RAGGED = [4096 + 1024 + 7, 1, 3, 1000, 2, 4099, 64, 5]


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 8])
@pytest.mark.parametrize("variant", [O.ADAM, O.ADOPT, O.SGDM])
def test_every_mask_class_matches_oracle(orc, variant, M):
    # periods (2,3,5): within 31 steps every one of the 8 gate combinations occurs
    Ks = (2, 3, 5) if variant != O.SGDM else (2, 3, 0)
    case = HostCase(variant, M, RAGGED, Ks, HYP[variant], seed=100 + 10 * variant + M)
    seen = {B.desloc_sync_mask(case.ctx, t) for t in range(31)}
    assert seen == (set(range(8)) if variant != O.SGDM else set(range(4)))
    nbit = case.run(orc, 31)
    case.close()
    print(f"variant {variant} M {M}: {nbit} elements not bit-identical")


@pytest.mark.parametrize("variant,flags", [
    (O.ADAM, B.FLAG_ADAM_LITERAL), (O.ADOPT, B.FLAG_ADOPT_AVG_NORMALISER),
    (O.ADOPT, B.FLAG_ADOPT_INIT_G0SQ), (O.ADOPT, B.FLAG_ADOPT_INIT_G0SQ | B.FLAG_ADOPT_AVG_NORMALISER)])
@pytest.mark.parametrize("M", [3, 4])
def test_alternative_readings_match_oracle(orc, variant, flags, M):
    hyp = list(HYP[variant])
    if flags & B.FLAG_ADAM_LITERAL:
        hyp[3] = 1e-4  # lambda
    case = HostCase(variant, M, RAGGED, (2, 3, 4), tuple(hyp), flags=flags, seed=7 + flags + M,
                    distinct_start=not (flags & B.FLAG_ADOPT_INIT_G0SQ))
    case.run(orc, 14)
    case.close()


@pytest.mark.parametrize("variant", [O.ADAM, O.ADOPT, O.SGDM])
@pytest.mark.parametrize("M,packed,bf16", [(4, True, False), (3, True, False), (8, True, True),
                                           (4, False, False), (5, False, True), (1, True, False)])
def test_norm_clipping_matches_oracle(orc, variant, M, packed, bf16):
    Ks = (2, 3, 5) if variant != O.SGDM else (2, 3, 0)
    hyp = list(HYP[variant])
    hyp[4] = 2.5  # rho: with the gradient recipe of HostCase.run some steps clip and some do not
    numel = RAGGED if packed else [1024 * 3 + 1, 0, 2, 4096, 6, 1023]
    case = HostCase(variant, M, numel, Ks, tuple(hyp), flags=B.FLAG_NORM_CLIP, bf16=bf16, packed=packed,
                    seed=900 + 10 * variant + M)
    case.run(orc, 12)
    assert case.clipped_steps > 0 and case.unclipped_steps > 0
    case.close()


def _random_case(rng):
    variant = int(rng.choice([O.ADAM, O.ADOPT, O.SGDM]))
    M = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 9, 11, 12, 17, 31]))
    sizes = [0, 1, 2, 3, 5, 63, 255, 256, 257, 511, 513, 1024, 1027, 3000]
    numel = [int(rng.choice(sizes)) for _ in range(int(rng.integers(1, 7)))]
    if sum(numel) == 0:
        numel.append(9)
    Ks = [int(rng.choice([0, 1, 2, 3])) for _ in range(3)]
    flags = 0
    if variant == O.ADAM:
        flags |= int(rng.choice([0, B.FLAG_ADAM_LITERAL]))
        if rng.random() < 0.4:
            flags |= B.FLAG_POST_AVERAGE | int(rng.choice([0, B.FLAG_AMSGRAD]))
    elif variant == O.ADOPT:
        flags |= int(rng.choice([0, B.FLAG_ADOPT_AVG_NORMALISER])) | int(rng.choice([0, B.FLAG_ADOPT_INIT_G0SQ]))
    else:
        Ks[2] = 0
        flags |= int(rng.choice([0, B.FLAG_POST_AVERAGE]))
    hyp = list(HYP[variant])
    if flags & B.FLAG_ADAM_LITERAL:
        hyp[3] = 1e-4
    if rng.random() < 0.3:
        flags |= B.FLAG_NORM_CLIP
        hyp[4] = 1.5
    elif variant == O.SGDM:
        hyp[4] = 0.05
    return dict(variant=variant, M=M, numel=numel, Ks=tuple(Ks), hyp=tuple(hyp), flags=flags,
                bf16=bool(rng.random() < 0.35), packed=bool(rng.random() < 0.5),
                chunk_elems=int(rng.choice([0, 0, 256, 512, 1024])),
                distinct_start=not (flags & B.FLAG_ADOPT_INIT_G0SQ))


@pytest.mark.parametrize("block", range(6))
def test_seeded_random_configurations_match_oracle(orc, block):
    """Sixty seeded random combinations of variant, replica count, tensor sizes (empty, sub-vector,
    around the tile size), periods (0 = never, 1 = every step), readings, orderings, clipping mode,
    gradient dtype, layout and chunk size; four steps each, every element compared."""
    rng = np.random.default_rng(7000 + block)
    for i in range(10):
        kw = _random_case(rng)
        print("case", block, i, {k: v for k, v in kw.items() if k != "hyp"}, flush=True)
        case = HostCase(kw["variant"], kw["M"], kw["numel"], kw["Ks"], kw["hyp"], flags=kw["flags"],
                        bf16=kw["bf16"], packed=kw["packed"], seed=int(rng.integers(1 << 30)),
                        distinct_start=kw["distinct_start"], chunk_elems=kw["chunk_elems"])
        case.run(orc, 4)
        case.close()


@pytest.mark.parametrize("variant,packed", [(O.ADAM, True), (O.ADOPT, False), (O.SGDM, True)])
def test_maximum_replica_count(orc, variant, packed):
    """M = 1024, the largest replica count the ABI admits, and one beyond it."""
    Ks = (2, 3, 4) if variant != O.SGDM else (2, 3, 0)
    case = HostCase(variant, 1024, [7, 300, 1], Ks, HYP[variant], packed=packed, seed=5151)
    case.run(orc, 5)
    case.close()
    with pytest.raises(B.DeslocError) as e:
        HostCase(variant, 1025, [8], Ks, HYP[variant], seed=1)
    assert e.value.status == B.ERR_BAD_ARG


@pytest.mark.parametrize("variant", [O.ADAM, O.SGDM])
@pytest.mark.parametrize("M,packed", [(3, True), (4, True), (6, False), (8, False)])
def test_mean_of_negative_zeros_keeps_the_sign(orc, variant, M, packed):
    """Every replica holds -0.0 in a gated state and the gradient is zero: the ascending-m sum of
    negative zeros is -0.0 and so is the mean, bit for bit (a sum seeded with +0.0 would give +0.0).
    Compile-time and runtime replica counts, strided and table layouts."""
    case = HostCase(variant, M, [700, 5, 1030], (1, 1, 1 if variant != O.SGDM else 0), HYP[variant],
                    packed=packed, seed=4242 + M)
    for name, host in (("x", case.x), ("u", case.u)):
        host[:] = -0.0
        for row in case.dev_arrays[name]:
            for t in row:
                t.fill_(-0.0)
    g_or = case.set_grads(np.zeros((M, case.N), np.float32))
    B.desloc_step(case.ctx, 5)
    orc.step(case.cfg, 5, case.x, case.u, case.v, np.ascontiguousarray(g_or))
    for which, host in ((B.X, case.x), (B.U, case.u)):
        got = case.read(which)
        assert np.array_equal(got.view(np.uint32), host.view(np.uint32))
    assert np.all(np.signbit(case.x))  # the parameters really stayed at -0.0
    case.close()


@pytest.mark.parametrize("chunk_elems", [256, 512, 2048])
def test_norm_clipping_table_layout_many_record_groups(orc, chunk_elems):
    """Separately allocated tensors: the norm reduction walks the step kernels' chunk records in
    groups per workgroup; several full groups, a ragged last group and ragged last records."""
    hyp = list(HYP[O.ADAM])
    hyp[4] = 4.0
    numel = [20000 + 3, 1, 9000, 256, 255, 257, 12288, 5]
    case = HostCase(O.ADAM, 3, numel, (2, 3, 5), tuple(hyp), flags=B.FLAG_NORM_CLIP, packed=False,
                    seed=977 + chunk_elems, chunk_elems=chunk_elems)
    case.run(orc, 6)
    assert case.clipped_steps > 0
    case.close()


POST_CASES = [
    (O.ADAM, B.FLAG_POST_AVERAGE), (O.ADAM, B.FLAG_POST_AVERAGE | B.FLAG_ADAM_LITERAL),
    (O.ADAM, B.FLAG_POST_AVERAGE | B.FLAG_AMSGRAD),
    (O.ADAM, B.FLAG_POST_AVERAGE | B.FLAG_AMSGRAD | B.FLAG_ADAM_LITERAL),
    (O.SGDM, B.FLAG_POST_AVERAGE),
]


@pytest.mark.parametrize("variant,flags", POST_CASES)
@pytest.mark.parametrize("M,packed,bf16", [(4, True, False), (8, True, True), (3, True, False),
                                           (5, False, False), (1, True, False), (4, False, True)])
def test_update_then_average_matches_oracle(orc, variant, flags, M, packed, bf16):
    Ks = (2, 3, 5) if variant != O.SGDM else (2, 3, 0)
    hyp = list(HYP[variant])
    if flags & B.FLAG_ADAM_LITERAL:
        hyp[3] = 1e-4
    numel = RAGGED if packed else [1024 * 3 + 1, 0, 2, 4096, 6, 1023]
    case = HostCase(variant, M, numel, Ks, tuple(hyp), flags=flags, bf16=bf16, packed=packed,
                    seed=1300 + 7 * flags + M)
    case.run(orc, 31 if M in (4, 3) else 12)
    # right after the last full sync every replica holds identical bits of every synced state
    t_sync = 30 if variant != O.SGDM else 6
    case.run(orc, 1, t0=t_sync)
    got_x = case.read(B.X)
    assert all(np.array_equal(got_x[0], got_x[m]) for m in range(M))
    case.close()


def test_update_then_average_with_norm_clip(orc):
    case = HostCase(O.ADAM, 4, RAGGED, (2, 3, 5), (1e-3, 0.9, 0.999, 1e-8, 2.5),
                    flags=B.FLAG_POST_AVERAGE | B.FLAG_AMSGRAD | B.FLAG_NORM_CLIP, seed=77)
    case.run(orc, 12)
    assert case.clipped_steps > 0 and case.unclipped_steps > 0
    case.close()


def test_vmax_read_only_with_amsgrad(orc):
    case = HostCase(O.ADAM, 2, [100], (2, 3, 5), HYP[O.ADAM], flags=B.FLAG_POST_AVERAGE, seed=4)
    with pytest.raises(B.DeslocError) as e:
        B.desloc_read_state(case.ctx, B.VMAX, 0, 0, 100)
    assert e.value.status == B.ERR_VARIANT
    case.close()


@pytest.mark.parametrize("packed", [True, False])
def test_state_change_diagnostic_matches_oracle(orc, packed):
    # ||s_{t+K} - s_t||_2 / ||s_t||_2 per replica: snapshot on the device, K steps, compare
    M, K = 4, 5
    numel = RAGGED if packed else [1024 * 3 + 1, 0, 2, 4096, 6, 1023]
    case = HostCase(O.ADAM, M, numel, (2, 3, 5), HYP[O.ADAM], packed=packed, seed=2100 + packed)
    case.run(orc, 3)
    N = case.N
    snaps = {}
    for which, host in ((B.X, case.x), (B.U, case.u), (B.V, case.v)):
        if packed:
            buf = torch.zeros((M, _stride(N)), device=DEV)
            table = B.packed_pointer_table(buf.data_ptr(), _stride(N) * 4, numel, M, 4)
        else:
            buf = [[torch.zeros(max(n, 1) + 8, device=DEV)[:n] for n in numel] for _ in range(M)]
            table = np.array([[t.data_ptr() if t.numel() else 0x10 for t in row] for row in buf],
                             dtype=np.uint64).reshape(-1)
        B.desloc_snapshot_state(case.ctx, which, table)
        snaps[which] = (buf, table, host.copy())
    case.run(orc, K, t0=3)
    for which, host in ((B.X, case.x), (B.U, case.u), (B.V, case.v)):
        buf, table, then = snaps[which]
        change, base = B.desloc_state_change(case.ctx, which, B.ALL_TENSORS, table, M)
        want_c, want_b = orc.state_change(host, then)
        np.testing.assert_allclose(change, want_c, rtol=3e-7)
        np.testing.assert_allclose(base, want_b, rtol=3e-7)
        assert np.all(change > 0) and np.all(base > 0)
        # one tensor only (ragged offset inside a packed segment)
        k = 3
        s0 = sum(numel[:k])
        c1, b1 = B.desloc_state_change(case.ctx, which, k, table, M)
        w1c, w1b = orc.state_change(np.ascontiguousarray(host[:, s0:s0 + numel[k]]),
                                    np.ascontiguousarray(then[:, s0:s0 + numel[k]]))
        np.testing.assert_allclose(c1, w1c, rtol=3e-7)
        np.testing.assert_allclose(b1, w1b, rtol=3e-7)
    # a reference table that is not laid out like the state is refused
    if packed:
        bad = snaps[B.X][1].copy()
        bad[1] += np.uint64(64)
        with pytest.raises(B.DeslocError) as e:
            B.desloc_state_change(case.ctx, B.X, B.ALL_TENSORS, bad, M)
        assert e.value.status == B.ERR_BAD_ARG
    with pytest.raises(B.DeslocError) as e:
        B.desloc_state_change(case.ctx, B.G, B.ALL_TENSORS, snaps[B.X][1], M)
    assert e.value.status == B.ERR_BAD_ARG
    case.close()


def test_grad_norms_only_for_norm_clip_contexts(orc):
    case = HostCase(O.ADAM, 2, [100], (2, 3, 5), HYP[O.ADAM], seed=3)
    with pytest.raises(B.DeslocError) as e:
        B.desloc_read_grad_norms(case.ctx, 2)
    assert e.value.status == B.ERR_VARIANT
    case.close()


@pytest.mark.parametrize("variant", [O.ADAM, O.SGDM, O.ADOPT])
@pytest.mark.parametrize("M", [4, 6])
def test_bf16_gradients_match_oracle(orc, variant, M):
    Ks = (2, 3, 4) if variant != O.SGDM else (2, 4, 0)
    case = HostCase(variant, M, RAGGED, Ks, HYP[variant], bf16=True, seed=55 + variant + M)
    case.run(orc, 13)
    case.close()


@pytest.mark.parametrize("M", [2, 3, 8])
def test_separately_allocated_tensors_match_oracle(orc, M):
    # one segment per tensor, ragged tails in every segment, zero-sized tensors in the list
    numel = [1024 * 3 + 1, 0, 2, 4096, 0, 6, 1023, 1025, 4]
    case = HostCase(O.ADAM, M, numel, (2, 3, 5), HYP[O.ADAM], packed=False, seed=77 + M)
    info = B.desloc_get_plan(case.ctx)
    assert info.n_segments == 7 and info.total_numel == sum(numel)
    case.run(orc, 11)
    case.close()


@pytest.mark.parametrize("chunk", [1024, 2048, 65536])
def test_chunk_sizes_match_oracle(orc, chunk):
    case = HostCase(O.ADAM, 4, [70000, 5, 9000], (2, 3, 5), HYP[O.ADAM], seed=chunk, chunk_elems=chunk)
    info = B.desloc_get_plan(case.ctx)
    assert info.n_segments == 1 and info.n_chunks == math.ceil(79005 / chunk)
    case.run(orc, 7)
    case.close()


def test_large_replica_count_runtime_path(orc):
    # M = 33: far beyond the compile-time replica counts
    case = HostCase(O.ADAM, 33, [1500, 9], (2, 3, 5), HYP[O.ADAM], seed=333)
    case.run(orc, 8)
    case.close()
    case = HostCase(O.ADOPT, 17, [1030], (3, 2, 2), HYP[O.ADOPT], seed=334)
    case.run(orc, 8)
    case.close()


def test_init_modes_and_mean_readback(orc):
    M, numel = 3, [1000, 37]
    N = sum(numel)
    case = HostCase(O.ADAM, M, numel, (4, 4, 4), HYP[O.ADAM], seed=5)
    # E_m[.] read-back equals the oracle's fixed-order mean, bit for bit
    for which, host in ((B.X, case.x), (B.U, case.u), (B.V, case.v)):
        got = B.desloc_read_state(case.ctx, which, B.REPLICA_MEAN, B.ALL_TENSORS, N)
        np.testing.assert_array_equal(got, orc.worker_mean(host))
        got1 = B.desloc_read_state(case.ctx, which, B.REPLICA_MEAN, 1, 37)
        np.testing.assert_array_equal(got1, orc.worker_mean(host)[1000:])
    # single-tensor, single-replica read
    np.testing.assert_array_equal(B.desloc_read_state(case.ctx, B.X, 2, 1, 37), case.x[2, 1000:])
    with pytest.raises(B.DeslocError) as e:
        B.desloc_read_state(case.ctx, B.X, 3, 0, 1000)
    assert e.value.status == B.ERR_BAD_ARG
    out = np.empty(10, np.float32)
    assert B.lib().desloc_read_state(case.ctx, B.X, 0, 0, out.ctypes.data, out.nbytes) == B.ERR_BAD_ARG
    case.close()

    # BROADCAST_REPLICA0: x^m = x^0, u = v = 0 (Alg. 1 local-init line)
    dev = torch.device(DEV)
    S = _stride(N)
    x = torch.randn((M, S), device=dev)
    u = torch.randn((M, S), device=dev)
    v = torch.rand((M, S), device=dev)
    g = torch.zeros((M, S), device=dev)
    x0 = x[0, :N].cpu().numpy().copy()
    tabs = {k: B.packed_pointer_table(t.data_ptr(), S * 4, numel, M, 4)
            for k, t in (("x", x), ("u", u), ("v", v), ("g", g))}
    for mode in (B.INIT_ZERO_STATES, B.INIT_BROADCAST_REPLICA0):
        xb = x.clone()
        tabs["x"] = B.packed_pointer_table(xb.data_ptr(), S * 4, numel, M, 4)
        ctx = B.desloc_init(variant=B.ADAM, M=M, numel=numel, Kx=1, Ku=1, Kv=1, lr=1e-3, beta1=0.9,
                            beta2=0.999, eps=1e-8, rho=1.0, init_mode=mode, **tabs)
        for m in range(M):
            got = B.desloc_read_state(ctx, B.X, m, B.ALL_TENSORS, N)
            want = x0 if mode == B.INIT_BROADCAST_REPLICA0 else x[m, :N].cpu().numpy()
            np.testing.assert_array_equal(got, want)
            assert not B.desloc_read_state(ctx, B.U, m, B.ALL_TENSORS, N).any()
            assert not B.desloc_read_state(ctx, B.V, m, B.ALL_TENSORS, N).any()
        # padding beyond the tensors is never written
        assert torch.equal(xb[:, N:], x[:, N:]) and torch.equal(u[:, N:], u[:, N:])
        B.desloc_destroy(ctx)


def test_init_rejects_misaligned_and_sgdm_v_reads():
    dev = torch.device(DEV)
    buf = torch.zeros(4 * 64, device=dev)
    p = buf.data_ptr()
    tab = lambda off: np.array([p + off], dtype=np.uint64)
    with pytest.raises(B.DeslocError) as e:
        B.desloc_init(variant=B.SGDM, M=1, numel=[8], Kx=1, Ku=1, Kv=0, lr=1e-3, beta1=0.9, beta2=0.0,
                      eps=1e-8, rho=1.0, x=tab(4), u=tab(256), v=None, g=tab(512))
    assert e.value.status == B.ERR_ALIGN
    ctx = B.desloc_init(variant=B.SGDM, M=1, numel=[8], Kx=1, Ku=1, Kv=0, lr=1e-3, beta1=0.9, beta2=0.0,
                        eps=1e-8, rho=1.0, x=tab(0), u=tab(256), v=None, g=tab(512))
    with pytest.raises(B.DeslocError) as e:
        B.desloc_read_state(ctx, B.V, 0, 0, 8)
    assert e.value.status == B.ERR_VARIANT
    assert B.desloc_sync_mask(ctx, 0) == 3  # no v bit for SGDM
    B.desloc_destroy(ctx)


def test_set_lr_schedule_matches_oracle(orc):
    case = HostCase(O.ADAM, 4, [3000], (2, 3, 5), HYP[O.ADAM], seed=9)
    for t in range(6):
        lr = float(np.float32(1e-3 * (t + 1) / 6))  # warm-up style schedule
        B.desloc_set_lr(case.ctx, lr)
        case.cfg.lr = lr
        case.run(orc, 1, t0=t)
    case.close()


def test_non_consecutive_steps_use_the_t_passed(orc):
    # jumping straight to a full-sync instant far into training (bias correction and gates
    # are functions of t alone)
    case = HostCase(O.ADAM, 4, [5000], (128, 384, 768), HYP[O.ADAM], seed=10)
    assert B.desloc_sync_mask(case.ctx, 768) == 7
    case.run(orc, 1, t0=768)
    case.run(orc, 1, t0=128)
    case.run(orc, 1, t0=100000)
    case.close()


# ------------------------------------------------------------------------------------
# Device input generator
# ------------------------------------------------------------------------------------

def test_device_philox_stream_is_bit_exact():
    rng = np.random.default_rng(0)
    n = 5000
    ctr = rng.integers(0, 2 ** 32, size=(n, 4), dtype=np.uint64).astype(np.uint32)
    key = rng.integers(0, 2 ** 32, size=(n, 2), dtype=np.uint64).astype(np.uint32)
    d_ctr = torch.from_numpy(ctr.view(np.int32)).to(DEV)
    d_key = torch.from_numpy(key.view(np.int32)).to(DEV)
    d_out = torch.zeros((n, 4), dtype=torch.int32, device=DEV)
    assert G.lib().desloc_inputs_philox_raw(d_ctr.data_ptr(), d_key.data_ptr(), d_out.data_ptr(), n, None) == 0
    torch.cuda.synchronize()
    got = d_out.cpu().numpy().view(np.uint32)
    np.testing.assert_array_equal(got, G.philox4x32_10_numpy(ctr, key))


@pytest.mark.parametrize("cfg_id", [1, 3, 4])
def test_device_gradients_follow_the_recipe(cfg_id):
    w = R.scaled_down(R.CONFIGS[cfg_id](), 200_000, keep_tensors=40)
    with DeslocSession(w) as s:
        s.fill_gradients(5)
        torch.cuda.synchronize()
        starts = s.mem.starts()
        for m in (0, w.M - 1):
            g = B.desloc_read_state(s.ctx, B.G, m, B.ALL_TENSORS, s.mem.total)
            for k in (0, w.n_tensors // 2, w.n_tensors - 1):
                seg = g[int(starts[k]):int(starts[k + 1])]
                ref = G.reference_values(w.seed, G.PURPOSE_GRAD, 5, m, k, np.arange(seg.size), w.dist,
                                         float(w.grad_scale[k]), w.grad_mean0, w.grad_mean_per_replica)
                tol = 1e-2 if w.grad_bf16 else 2e-4  # bf16 rounding / fp32 log-cos ulps, heavy tails
                np.testing.assert_allclose(seg, ref, rtol=tol, atol=tol * float(w.grad_scale[k]))
        # every replica starts from the same x_0 (Alg. 1 local init)
        x0 = s.read(B.X, 0)
        assert x0.std() == pytest.approx(w.x0_std, rel=0.05)
        for m in range(1, w.M):
            np.testing.assert_array_equal(s.read(B.X, m), x0)


def assert_same_bits(got, want, what):
    """Bit-pattern comparison that admits non-finite values: NaNs must sit at the same positions
    (IEEE leaves their payload open, so only NaN-ness is compared there); every other value,
    infinities, signed zeros and denormals included, must be the same 32 bits."""
    got = np.ascontiguousarray(got, dtype=np.float32)
    want = np.ascontiguousarray(want, dtype=np.float32)
    nan_g, nan_w = np.isnan(got), np.isnan(want)
    assert np.array_equal(nan_g, nan_w), f"{what}: NaNs at different positions ({nan_g.sum()} vs {nan_w.sum()})"
    gb, wb = got.view(np.uint32)[~nan_g], want.view(np.uint32)[~nan_w]
    bad = gb != wb
    assert not bad.any(), f"{what}: {bad.sum()} values differ in their bits, e.g. {got[~nan_g][bad][:3]} vs {want[~nan_w][bad][:3]}"


@pytest.mark.parametrize("rho", [1.0, float("inf")])
@pytest.mark.parametrize("variant,flags", [(O.ADAM, 0), (O.ADAM, B.FLAG_ADAM_LITERAL), (O.ADOPT, 0), (O.SGDM, 0),
                                           (O.ADAM, B.FLAG_POST_AVERAGE | B.FLAG_AMSGRAD)])
def test_non_finite_gradients_and_denormal_states_match_bit_patterns(orc, variant, flags, rho):
    """NaN and +-Inf gradients (with a finite clip radius the infinities are clipped to +-rho, with
    rho = inf they propagate), gradients at the edge of the fp32 range, denormal and zero moments:
    the kernels take no shortcut that an IEEE host would not take."""
    M, numel = 4, [300, 5, 1027]
    lr, b1, b2, eps, _ = HYP[variant]
    case = HostCase(variant, M, numel, (2, 3, 4), (lr, b1, b2, eps, rho), flags=flags, seed=900 + variant)
    N = case.N
    # denormal and zero moments, on some replicas only
    for name, host in (("u", case.u), ("v", case.v)):
        if host is None:
            continue
        host[0, 0:40] = np.float32(1e-40) if name == "u" else np.float32(3e-42)
        host[1, 20:60] = 0.0
        host[2, 0:10] = np.float32(-1e-39) if name == "u" else np.float32(1e-45)
        if case.vmax is not None and name == "v":
            case.vmax[:] = np.maximum(case.vmax, host)
        for m in range(M):
            for (s, n), dst in zip(case._spans(), case.dev_arrays[name][m]):
                dst.copy_(torch.from_numpy(host[m, s:s + n]))
    if case.vmax is not None:
        for m in range(M):
            for (s, n), dst in zip(case._spans(), case.dev_arrays["vmax"][m]):
                dst.copy_(torch.from_numpy(case.vmax[m, s:s + n]))
    torch.cuda.synchronize()
    specials = np.array([np.nan, np.inf, -np.inf, 3.0e38, -3.0e38, 1e-40, -1e-45, 0.0, -0.0], dtype=np.float32)
    for t in range(9):  # periods (2, 3, 4): every gate pattern but "all" after t = 0, which comes at t = 0
        g32 = (case.rng.normal(size=(M, N)) * 0.02).astype(np.float32)
        pos = case.rng.integers(0, N, size=(M, 3 * specials.size))
        for m in range(M):
            if m == 3 and t % 2:
                continue  # a replica without special values on some steps
            g32[m, pos[m]] = np.tile(specials, 3)
        g_or = case.set_grads(g32)
        assert B.desloc_sync_mask(case.ctx, t) == orc.sync_mask(case.cfg, t)
        B.desloc_step(case.ctx, t)
        with np.errstate(all="ignore"):
            orc.step(case.cfg, t, case.x, case.u, case.v, np.ascontiguousarray(g_or), vmax=case.vmax)
        assert_same_bits(case.read(B.X), case.x, f"x after t={t}")
        assert_same_bits(case.read(B.U), case.u, f"u after t={t}")
        if case.v is not None:
            assert_same_bits(case.read(B.V), case.v, f"v after t={t}")
        if case.vmax is not None:
            assert_same_bits(case.read(B.VMAX), case.vmax, f"vmax after t={t}")
    if rho == float("inf"):
        assert np.isnan(case.x).any() and np.isinf(case.u).any()
    case.close()


@pytest.mark.parametrize("variant", [O.ADAM, O.ADOPT, O.SGDM])
def test_checkpoint_and_resume_round_trip(orc, variant):
    """Alg. 1 takes x_0 and the states s_{-1} as inputs and returns x_T and s_{T-1}: reading every
    replica's state back, destroying the context, and creating a new one on fresh buffers with
    DESLOC_INIT_AS_IS must continue exactly as the uninterrupted run (the oracle's) does."""
    M, numel, T1, T2 = 4, [1500, 7, 0, 2049], 7, 9
    Ks = (2, 3, 5) if variant != O.SGDM else (2, 3, 0)
    first = HostCase(variant, M, numel, Ks, HYP[variant], seed=1234 + variant)
    first.run(orc, T1)
    saved = {"x": first.read(B.X), "u": first.read(B.U)}
    if variant != O.SGDM:
        saved["v"] = first.read(B.V)
    oracle_state = {"x": first.x, "u": first.u, "v": first.v}
    rng = first.rng
    first.close()
    del first
    torch.cuda.empty_cache()
    # a new context on new buffers, seeded from the checkpoint alone
    second = HostCase(variant, M, numel, Ks, HYP[variant], seed=999)
    for name, arr in saved.items():
        for m in range(M):
            for (s, n), dst in zip(second._spans(), second.dev_arrays[name][m]):
                if n:
                    dst.copy_(torch.from_numpy(arr[m, s:s + n]))
    torch.cuda.synchronize()
    second.x, second.u, second.v = oracle_state["x"], oracle_state["u"], oracle_state["v"]
    second.rng = rng
    nbit = second.run(orc, T2, t0=T1)  # compares against the oracle's uninterrupted trajectory every step
    assert nbit == 0
    second.close()


@pytest.mark.parametrize("packed", [True, False])
def test_batched_per_tensor_state_change_matches_oracle(orc, packed):
    """||s_{t+K} - s_t||_2 and ||s_t||_2 for every tensor and replica from one asynchronous call,
    on a tensor list shaped like the many-small-tensors configuration (sizes from 1 to several
    partial-sum records, an empty tensor, odd offsets inside the packed buffer)."""
    M, K = 4, 4
    rng = np.random.default_rng(77)
    numel = [int(n) for n in np.floor(np.exp(rng.uniform(np.log(1), np.log(70_000), 60)))]
    numel[7] = 0
    numel[11] = 16384
    numel[12] = 16385
    numel[13] = 3 * 16384 + 2
    case = HostCase(O.ADAM, M, numel, (2, 3, 5), HYP[O.ADAM], packed=packed, seed=4100 + packed)
    case.run(orc, 2, check_every=2)
    N, nt = case.N, len(numel)
    change = torch.full((nt, M), -1.0, device=DEV)
    base = torch.full((nt, M), -1.0, device=DEV)
    snaps = {}
    for which, host in ((B.X, case.x), (B.U, case.u), (B.V, case.v)):
        if packed:
            buf = torch.zeros((M, _stride(N)), device=DEV)
            table = B.packed_pointer_table(buf.data_ptr(), _stride(N) * 4, numel, M, 4)
        else:
            buf = [[torch.zeros(max(n, 1) + 8, device=DEV)[:n] for n in numel] for _ in range(M)]
            table = np.array([[t.data_ptr() if t.numel() else 0x10 for t in row] for row in buf],
                             dtype=np.uint64).reshape(-1)
        B.desloc_snapshot_state(case.ctx, which, table)
        snaps[which] = (buf, table, host.copy())
    # the snapshot kernel copied exactly the state
    B.desloc_synchronize(case.ctx)
    for which in (B.X, B.U, B.V):
        buf, _, then = snaps[which]
        got = buf[:, :N].cpu().numpy() if packed else np.stack(
            [np.concatenate([t.cpu().numpy() for t in row]) for row in buf])
        assert np.array_equal(got, then)
    case.run(orc, K, t0=2, check_every=K)
    for which, host in ((B.X, case.x), (B.U, case.u), (B.V, case.v)):
        _, table, then = snaps[which]
        B.desloc_bind_reference(case.ctx, table)  # the last snapshot bound v's table
        change.fill_(-1.0)
        base.fill_(-1.0)
        torch.cuda.synchronize()
        B.desloc_state_change_tensors(case.ctx, which, change.data_ptr(), base.data_ptr())
        B.desloc_synchronize(case.ctx)
        want_c, want_b = orc.state_change_tensors(host, then, numel)
        np.testing.assert_allclose(change.cpu().numpy(), want_c, rtol=3e-7, atol=0)
        np.testing.assert_allclose(base.cpu().numpy(), want_b, rtol=3e-7, atol=0)
        assert want_c[7].sum() == 0 and (want_c[np.array(numel) > 0] > 0).all()
        # consistent with the whole-model entry point: squares add up
        whole_c, whole_b = B.desloc_state_change(case.ctx, which, B.ALL_TENSORS, table, M)
        np.testing.assert_allclose(np.sqrt((change.cpu().numpy().astype(np.float64) ** 2).sum(0)), whole_c, rtol=1e-6)
    # nothing bound yet on a fresh context: refused
    fresh = HostCase(O.SGDM, 2, [100], (2, 3, 0), HYP[O.SGDM], seed=1)
    with pytest.raises(B.DeslocError) as e:
        B.desloc_state_change_tensors(fresh.ctx, B.U, change.data_ptr(), base.data_ptr())
    assert e.value.status == B.ERR_BAD_ARG
    with pytest.raises(B.DeslocError) as e:
        B.desloc_state_change_tensors(fresh.ctx, B.V, change.data_ptr(), base.data_ptr())
    assert e.value.status == B.ERR_VARIANT
    fresh.close()
    case.close()


@pytest.mark.parametrize("aligned", [True, False])
def test_snapshot_of_long_ragged_tensors_copies_exactly(orc, aligned):
    """Long tensors (records mostly full) take the snapshot kernel with sixteen single-wave workgroups per
    record; sizes of 4k + 1, 2, 3 put heads of 3, 2 and 1 elements in front of the vectors and tails behind
    them, a 3-element tensor leaves fifteen of its sixteen workgroups without work, and a destination that is
    only 4-byte aligned takes the element-wise path.  The copy must be exact, padding untouched."""
    M = 3
    numel = [16384 * 20 + 1, 3, 16384 * 30 + 2, 16384 * 25 + 3, 16384 * 2]
    records = sum(-(-n // 16384) for n in numel)
    assert records * 16384 <= 1.1 * sum(numel)  # the rule that picks this kernel
    case = HostCase(O.ADAM, M, numel, (2, 3, 5), HYP[O.ADAM], packed=True, seed=911)
    case.run(orc, 3, check_every=3)
    N = case.N
    shift = 0 if aligned else 1
    buf = torch.full((M, _stride(N) + 8), -7.0, device=DEV)
    table = B.packed_pointer_table(buf.data_ptr() + 4 * shift, (_stride(N) + 8) * 4, numel, M, 4)
    for which, host in ((B.X, case.x), (B.U, case.u), (B.V, case.v)):
        buf.fill_(-7.0)
        B.desloc_snapshot_state(case.ctx, which, table)
        B.desloc_synchronize(case.ctx)
        got = buf.cpu().numpy()
        assert np.array_equal(got[:, shift:shift + N], host)
        assert (got[:, :shift] == -7.0).all() and (got[:, shift + N:] == -7.0).all()
        # and the batched diagnostic against it is zero everywhere, with the oracle's norms as the base
        change = torch.full((len(numel), M), -1.0, device=DEV)
        base = torch.full((len(numel), M), -1.0, device=DEV)
        B.desloc_state_change_tensors(case.ctx, which, change.data_ptr(), base.data_ptr())
        B.desloc_synchronize(case.ctx)
        want_c, want_b = orc.state_change_tensors(host, host.copy(), numel)
        assert not change.any().item() and not want_c.any()
        np.testing.assert_allclose(base.cpu().numpy(), want_b, rtol=3e-7, atol=0)
    # v's snapshot is the last one in buf: two more steps, then the whole-model and the one-tensor call walk
    # the same long ragged ranges (128-bit loads when the reference is aligned, element-wise when it is not)
    then = case.v.copy()
    case.run(orc, 2, t0=3, check_every=2)
    c_all, b_all = B.desloc_state_change(case.ctx, B.V, B.ALL_TENSORS, table, M)
    want_c, want_b = orc.state_change(case.v, then)
    np.testing.assert_allclose(c_all, want_c, rtol=3e-7)
    np.testing.assert_allclose(b_all, want_b, rtol=3e-7)
    for k in (2, 3):
        s0 = sum(numel[:k])
        c1, b1 = B.desloc_state_change(case.ctx, B.V, k, table, M)
        w1c, w1b = orc.state_change(np.ascontiguousarray(case.v[:, s0:s0 + numel[k]]),
                                    np.ascontiguousarray(then[:, s0:s0 + numel[k]]))
        np.testing.assert_allclose(c1, w1c, rtol=3e-7)
        np.testing.assert_allclose(b1, w1b, rtol=3e-7)
    cs, bs = B.desloc_state_change_static(case.ctx, B.V, B.ALL_TENSORS, table, M)
    np.testing.assert_allclose(cs, want_c, rtol=3e-7)
    np.testing.assert_allclose(bs, want_b, rtol=3e-7)
    case.close()
