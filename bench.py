#!/usr/bin/env python3
"""Benchmark of the DES-LOC step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5]

A "step" is one desloc_step over every tensor and all M replicas of the workload (clip,
period-gated replica averages, moment and parameter updates: one kernel launch).  The
default workload is the 1.7B-parameter, M = 4 Adam configuration, the one the headline
metric is quoted on.  Gradients and state are resident in HBM before the timed region;
the timed steps are t = 0 .. K-1 of the configuration's own sync schedule.

Prints ONE JSON line: whole-job throughput in replica-parameter updates per second, the
roofline object of the step kernel (algorithmic bytes / HIP-event kernel time against
8 TB/s), the same per class of gated launch, and the CPU oracle timed on a bounded sample of
the same workload.

Other modes (each prints one JSON line of its own):
    --realloc N        frees and re-allocates the arrays N times in this process and reports the
                       spread of the kernel times (physical placement differs per allocation)
    --stream-ceiling   streaming yardsticks of the step's access shapes without its arithmetic
    --stream-spread G  the 4 read + 3 write yardstick against the distance between its streams
    --placement-map G  the step at a series of positions inside one pool, for three arrangements of
                       the arrays (groups of tensors, one record per replica, one block per array)
    --replica-sweep L  every class of launch for each replica count in the list
    --library PATH     with any mode: load another build of the step library (measurement builds)
"""
from __future__ import annotations

import argparse
import json
import math
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (0 = the configuration's step count)")
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--chunk", type=int, default=0, help="chunk_elems override (0 = library default)")
    ap.add_argument("--layout", default="grouped", choices=["grouped", "packed", "separate"],
                    help="grouped: one allocation, groups of consecutive tensors, inside a group the replicas' "
                         "x, u, v, g one after the other (one segment per group, chunk-record path); packed: one "
                         "record of whole arrays per replica (one segment, strided path); separate: one allocation "
                         "per array, replica and tensor (chunk-record path)")
    ap.add_argument("--placement-pool-gib", type=float, default=-1.0,
                    help="packed layout: size of the pool inside which the arrays' placement is chosen by "
                         "measurement at setup (0 = plain allocations, no search; default: 2.1 x the workload, "
                         "at most the free memory less 24 GiB)")
    ap.add_argument("--library", default="", metavar="PATH",
                    help="load this build of the step library instead of the in-tree one (a measurement build, "
                         "see paper_2505_22549_amd/build.py; its environment knobs then apply)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-mask-classes", action="store_true")
    ap.add_argument("--cpu-sample-elems", type=int, default=4 * 1024 * 1024)
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--norm-clip", action="store_true",
                    help="norm-based clipping (per-replica global L2 norm) instead of the coordinate clip: "
                         "one more read of the gradients per step")
    ap.add_argument("--post-average", action="store_true",
                    help="update-then-average ordering (the proof listings' semantics); Adam and SGDM configs")
    ap.add_argument("--amsgrad", action="store_true",
                    help="AMSGrad state (implies --post-average; Adam configs): 8 more bytes per update")
    ap.add_argument("--diagnostics", action="store_true",
                    help="also time the relative-rate-of-change diagnostic ||u_{t+K} - u_t|| / ||u_t|| (one more "
                         "replica-sized snapshot buffer is allocated)")
    ap.add_argument("--snapshot-apart", action="store_true",
                    help="with --diagnostics on the grouped layout: keep the snapshot in an allocation of its own "
                         "instead of inside the groups beside the state (comparison)")
    ap.add_argument("--calibration-copy-gib", type=float, default=0.0,
                    help="also run a plain copy kernel of this many GiB (read N, write N) three times: "
                         "the known-size yardstick for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs")
    ap.add_argument("--realloc", type=int, default=0,
                    help="allocate, measure and free the workload this many times in one process; reports "
                         "min / median / max of the kernel times instead of the usual line")
    ap.add_argument("--stream-ceiling", action="store_true",
                    help="run the streaming yardstick kernels (read-only, write-only, copy, 4r+3w, 16r+12w, "
                         "32r+24w; contiguous and 32 KiB-paired) and print their GB/s")
    ap.add_argument("--stream-gib", type=float, default=1.0, help="GiB per stream for --stream-ceiling")
    ap.add_argument("--stream-spread", type=float, default=0.0, metavar="POOL_GIB",
                    help="the 4 read + 3 write yardstick with its streams 1..32 GiB apart at a series of positions "
                         "inside one pool of this size; prints one JSON object and exits")
    ap.add_argument("--replica-sweep", default="", metavar="M,M,...",
                    help="Adam at about 2e9 replica-parameters for each replica count M listed (e.g. 1,2,3,4,6,8,16,32): "
                         "every class of launch; prints one JSON object and exits")
    ap.add_argument("--placement-map", type=float, default=0.0, metavar="POOL_GIB",
                    help="allocate one pool of this many GiB, place the workload's arrays at a series of offsets "
                         "inside it and time the step at each: how the kernel time depends on where in HBM the "
                         "arrays lie (same process, same binary, same data)")
    return ap.parse_args()


def read_traffic(workload_name: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, if there is one.
    Returns (bytes or None, source file or None): the figure is NOT measured in this run."""
    rel = os.path.join("profiles", f"pmc_traffic_{workload_name}.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None
    vals = {}
    with open(path) as fh:
        for line in fh:
            if "=" in line and not line.lstrip().startswith("#"):
                k, v = line.split("=", 1)
                try:
                    vals[k.strip()] = float(v.split()[0])
                except ValueError:
                    pass
    if "FETCH_BYTES_PER_LAUNCH" in vals and "WRITE_BYTES_PER_LAUNCH" in vals:
        return vals["FETCH_BYTES_PER_LAUNCH"] + vals["WRITE_BYTES_PER_LAUNCH"], rel
    return None, None


def cpu_baseline(w, sample_elems: int, budget_s: float, bytes_per_update: int):
    """The CPU oracle, as it stands, on the first `sample_elems` elements of the workload
    (all M replicas), single-threaded."""
    import numpy as np
    import oracle as O

    orc = O.Oracle()
    n = int(min(sample_elems, w.total_numel))
    M = w.M
    rng = np.random.default_rng(w.seed)
    x = np.tile((rng.standard_normal(n) * w.x0_std).astype(np.float32), (M, 1))
    u = np.zeros((M, n), np.float32)
    v = np.zeros((M, n), np.float32) if w.variant != O.SGDM else None
    g = (rng.standard_normal((M, n)) * 1e-2 + w.grad_mean_per_replica * np.arange(M)[:, None]).astype(np.float32)
    if w.grad_bf16:  # the oracle sees widened bf16 values, as the kernel does
        g = (g.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)
    cfg = O.Config(w.variant, M, w.Kx, w.Ku, w.Kv, lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps,
                   rho=w.rho, adam_literal=bool(w.flags & 1), adopt_avg_normaliser=bool(w.flags & 2),
                   adopt_init_g0sq=bool(w.flags & 4), norm_clip=bool(w.flags & 8),
                   post_average=bool(w.flags & 16), amsgrad=bool(w.flags & 32)).as_f32_hypers()
    vmax = np.zeros((M, n), np.float32) if w.flags & 32 else None
    t0 = time.perf_counter()
    orc.step(cfg, 0, x, u, v, g, vmax=vmax)
    one = time.perf_counter() - t0
    steps = max(1, min(w.steps - 1, int(budget_s / max(one, 1e-6))))
    t0 = time.perf_counter()
    for t in range(1, 1 + steps):
        orc.step(cfg, t, x, u, v, g, vmax=vmax)
    dt = time.perf_counter() - t0
    rate = M * n * steps / dt
    return {"value": rate, "unit": "replica-param updates/s", "cores": 1, "kind": "oracle",
            "sample": f"first {n} elements x M={M} replicas of {w.name}, steps t=1..{steps} "
                      f"({dt:.1f} s, single thread, {os.cpu_count()} host cores visible)",
            "gbps_effective": rate * bytes_per_update / 1e9}


def class_instants(w):
    """One step instant per class of launch: none, x, x+u (Adam/ADOPT: u gated as well), all."""
    lcm = math.lcm(*[k for k in (w.Kx, w.Ku, w.Kv) if k]) if any((w.Kx, w.Ku, w.Kv)) else 0
    return {"none": 10_000_019, "x": w.Kx, "x+u": w.Ku, "all": lcm}


def time_classes(sess, stream, w, bytes_per_launch, reps=5):
    import torch
    out = {}
    for name, t in class_instants(w).items():
        if not t:
            continue
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        sess.step(t)
        e0.record(stream)
        for _ in range(reps):
            sess.step(t)
        e1.record(stream)
        sess.synchronize()
        ms = e0.elapsed_time(e1) / reps
        gbps = bytes_per_launch / (ms * 1e-3) / 1e9
        out[name] = {"t": t, "mask": sess.sync_mask(t), "ms": ms, "gbps": gbps, "frac": gbps / HBM_PEAK_GBPS}
    return out


def plan_dict(plan):
    return {"segments": int(plan.n_segments), "strided": bool(plan.strided), "chunk_elems": int(plan.chunk_elems),
            "workgroups_per_replica": int(plan.n_chunks), "paired_numel": int(plan.paired_numel),
            "lds_limiter_bytes": list(plan.lds_limiter_bytes),
            "intended_workgroups_per_cu": list(plan.intended_workgroups),
            "resident_workgroups_per_cu": list(plan.resident_workgroups), "lanes_per_workgroup": 64}


def stream_ceiling(args):
    """Streaming yardsticks: the step's access shapes without its arithmetic."""
    import torch
    from paper_2505_22549_amd.inputs import generator as gen
    stream = torch.cuda.Stream(device="cuda:0")
    sb = int(args.stream_gib * (1 << 30)) // 65536 * 65536
    shapes = [("read-only", 1, 0, False), ("write-only", 0, 1, False), ("copy 1r+1w", 1, 1, False),
              ("3r+2w in place (SGDM step)", 3, 2, True), ("4r+3w in place (Adam step, one replica)", 4, 3, True),
              ("16r+12w in place (gated step, M=4)", 16, 12, True),
              ("32r+24w in place (gated step, M=8)", 32, 24, True)]
    rows = []
    for name, r, wr, inplace in shapes:
        n_streams = r if inplace else r + wr
        buf = torch.zeros(n_streams * sb // 4 + 65536, dtype=torch.float32, device="cuda:0")
        base = (buf.data_ptr() + 65535) // 65536 * 65536
        torch.cuda.synchronize()
        row = {"shape": name, "reads": r, "writes": wr, "bytes_per_launch": (r + wr) * sb}
        for paired in (False, True):
            best = None
            for waves in (6, 8, 9, 10, 12, 16):
                lds = 163840 // waves - 64
                gen.stream(base, sb, sb, r, wr, inplace, paired, lds, stream.cuda_stream)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(5):
                    gen.stream(base, sb, sb, r, wr, inplace, paired, lds, stream.cuda_stream)
                e1.record(stream)
                stream.synchronize()
                gbps = (r + wr) * sb / (e0.elapsed_time(e1) / 5 * 1e-3) / 1e9
                row.setdefault("paired" if paired else "contiguous", {})[f"{waves}_waves_per_cu"] = round(gbps, 1)
                best = gbps if best is None or gbps > best else best
            row["best_paired_gbps" if paired else "best_contiguous_gbps"] = round(best, 1)
        rows.append(row)
        del buf
        torch.cuda.empty_cache()
    print(json.dumps({"mode": "stream-ceiling", "gib_per_stream": sb / (1 << 30), "peak_gbps": HBM_PEAK_GBPS,
                      "note": "single-wave workgroups, 1 KiB per stream and wave, streaming loads, write-through "
                              "stores; resident waves per CU capped by an untouched dynamic-LDS request",
                      "shapes": rows}))


def stream_spread(args):
    """The 4 read + 3 write yardstick with its four 1 GiB streams S GiB apart, at a series of
    positions inside one pool: streams that are swept together are slower when they lie in
    different physically contiguous blocks of device memory (which virtual ranges share a block
    shows as the positions where short separations dip)."""
    import torch
    from paper_2505_22549_amd.inputs import generator as gen
    GiB = 1 << 30
    stream = torch.cuda.Stream(device="cuda:0")
    pool = torch.zeros(int(args.stream_spread * GiB), dtype=torch.uint8, device="cuda:0")
    base = (pool.data_ptr() + (2 << 20) - 1) // (2 << 20) * (2 << 20)
    top = (pool.data_ptr() + pool.numel() - base) // GiB
    lds = 163840 // 10 - 64

    def timed(addr, sep, reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        gen.stream(addr, sep, GiB, 4, 3, True, True, lds, stream.cuda_stream)
        e0.record(stream)
        for _ in range(reps):
            gen.stream(addr, sep, GiB, 4, 3, True, True, lds, stream.cuda_stream)
        e1.record(stream)
        stream.synchronize()
        return 7 * GiB / (e0.elapsed_time(e1) / reps * 1e-3) / 1e9

    timed(base, GiB, 200)  # the first tenths of a second after start-up run at half speed
    rows = []
    for sep in (1, 4, 8, 16, 24, 32):
        if 3 * sep + 1 > top:
            continue
        pos = list(range(0, int(top) - 3 * sep - 1, 8))
        rows.append({"separation_gib": sep, "position_gib": pos,
                     "gbps": [round(timed(base + p * GiB, sep * GiB, 3), 1) for p in pos]})
    print(json.dumps({"mode": "stream-spread", "pool_gib": args.stream_spread, "peak_gbps": HBM_PEAK_GBPS,
                      "note": "4 read + 3 write streams in place, 1 GiB each, paired mapping, 10 waves per CU",
                      "rows": rows}))


def replica_sweep(args):
    """Every class of launch against the replica count at a fixed total of replica-parameters."""
    import numpy as np
    import torch
    from paper_2505_22549_amd import binding as B
    from paper_2505_22549_amd.inputs import recipes as R
    from paper_2505_22549_amd.runtime import DeslocSession
    stream = torch.cuda.Stream(device="cuda:0")
    rows = []
    for M in [int(v) for v in args.replica_sweep.split(",")]:
        N = int(2.0e9 // M)
        # three tensors of ragged sizes, back to back in one packed buffer per replica
        numel = np.array([N // 3 + 5, N // 3 + 2, N - 2 * (N // 3) - 7], dtype=np.uint64)
        w = R.Workload(f"adam_sweep_M{M}", R.ADAM, M, 16, 4, 8, 16, numel, np.full(3, 1e-2, np.float32), rho=1.0, seed=11)
        sess = DeslocSession(w, stream=stream, layout="grouped")
        sess.fill_gradients(0)
        sess.synchronize()
        classes = time_classes(sess, stream, w, M * w.total_numel * w.bytes_per_update)
        plan = B.desloc_get_plan(sess.ctx)
        rows.append({"M": M, "numel_per_replica": int(w.total_numel), "paired_numel": int(plan.paired_numel),
                     "compile_time_M": M in (4, 8), "segments": int(plan.n_segments),
                     "gbps": {k: round(v["gbps"], 1) for k, v in classes.items()},
                     "frac": {k: round(v["frac"], 4) for k, v in classes.items()}})
        sess.close()
        del sess
        torch.cuda.empty_cache()
    print(json.dumps({"mode": "replica-sweep", "variant": "adam", "K": [4, 8, 16], "peak_gbps": HBM_PEAK_GBPS,
                      "note": "classes: none = no gate, x = x gated, x+u = x and u gated, all = x, u, v gated; "
                              "M = 1 has no gated launch (the mean of one replica is the replica)", "rows": rows}))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build keeps all M replicas in ONE GPU's HBM and has no multi-GPU path; "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2505_22549_amd import binding as B
    from paper_2505_22549_amd.inputs import recipes as R
    from paper_2505_22549_amd.runtime import DeslocSession

    if args.library:
        if not os.path.exists(args.library):
            print(f"bench.py: {args.library} does not exist", file=sys.stderr)
            sys.exit(2)
        B.LIBRARY = os.path.abspath(args.library)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    if args.stream_ceiling:
        stream_ceiling(args)
        return
    if args.stream_spread > 0:
        stream_spread(args)
        return
    if args.replica_sweep:
        replica_sweep(args)
        return

    w = R.CONFIGS[args.config]()
    grad_bytes = 2 if w.grad_bf16 else 4
    bytes_per_update = w.bytes_per_update
    if args.norm_clip:
        w.flags |= B.FLAG_NORM_CLIP
        w.name += "_normclip"
        if not math.isfinite(w.rho):
            w.rho = 1.0
        bytes_per_update += grad_bytes  # the norm pass reads the gradients once more
    if args.post_average or args.amsgrad:
        if w.variant == B.ADOPT:
            print("bench.py: --post-average is defined for the Adam and SGDM configurations", file=sys.stderr)
            sys.exit(2)
        w.flags |= B.FLAG_POST_AVERAGE
        w.name += "_postavg"
        if args.amsgrad:
            if w.variant != B.ADAM:
                print("bench.py: --amsgrad needs an Adam configuration", file=sys.stderr)
                sys.exit(2)
            w.flags |= B.FLAG_AMSGRAD
            w.name += "_amsgrad"
            bytes_per_update += 8  # vmax read and written
    if args.layout != "grouped":
        w.name += {"separate": "_separate", "packed": "_records"}[args.layout]
    K = args.steps if args.steps > 0 else w.steps
    W = args.warmup
    stream = torch.cuda.Stream(device="cuda:0")  # default priority
    updates_per_step = w.M * w.total_numel
    bytes_per_launch = updates_per_step * bytes_per_update

    if args.placement_map > 0:
        # The same launches with the arrays at a series of offsets inside one pool, in three arrangements:
        # "groups" (the default layout: per group of tensors the replicas' x, u, v, g side by side),
        # "records" (replica m's whole x, u, v, g next to each other) and "arrays" (one [M][stride]
        # block per array, so that streams swept together lie M * stride apart).
        from paper_2505_22549_amd.runtime import GroupedReplicas, PackedReplicas
        GiB = 1 << 30
        has_v, has_vmax = w.variant != B.SGDM, bool(w.flags & B.FLAG_AMSGRAD)
        es_g = 2 if w.grad_bf16 else 4
        need = PackedReplicas.bytes_needed(w.numel, w.M, has_v, w.grad_bf16, has_vmax)
        pool = torch.zeros(int(args.placement_map * GiB), dtype=torch.uint8, device="cuda:0")
        base = (pool.data_ptr() + (2 << 20) - 1) // (2 << 20) * (2 << 20)
        room = pool.data_ptr() + pool.numel() - base - need - (1 << 30)  # the groups' rounding needs a little more
        if room < 0:
            print("bench.py: the pool is smaller than the workload", file=sys.stderr)
            sys.exit(2)

        def tables(arrangement, off):
            if arrangement == "groups":
                mem = GroupedReplicas(w.numel, w.M, has_v, w.grad_bf16, has_vmax=has_vmax, pool=pool,
                                      pool_offset=base - (pool.data_ptr() + (-pool.data_ptr()) % 65536) + off)
                return {n: mem.table(mem.array(n)) for n in ("x", "u", "v", "vmax", "g")}
            mem = PackedReplicas(w.numel, w.M, has_v, w.grad_bf16, has_vmax=has_vmax, pool=pool, pool_offset=off)
            if arrangement == "records":
                return {n: mem.table(mem.array(n)) for n in ("x", "u", "v", "vmax", "g")}
            tabs, addr = {}, base + off
            for n in ("x", "u", "v", "vmax", "g"):
                if mem.array(n) is None:
                    tabs[n] = None
                    continue
                es = es_g if n == "g" else 4
                tabs[n] = B.packed_pointer_table(addr, mem.stride * es, w.numel, w.M, es)
                addr += w.M * mem.stride * es
            return tabs

        ARRANGEMENTS = ("groups", "records", "arrays")
        step_gib = max(1, int(room / GiB) // 16)
        rows = []
        for a_gib in range(0, int(room / GiB) + 1, step_gib):
            row = {"offset_gib": a_gib}
            for arrangement in ARRANGEMENTS:
                tabs = tables(arrangement, a_gib * GiB)
                ctx = B.desloc_init(variant=w.variant, M=w.M, numel=w.numel, Kx=w.Kx, Ku=w.Ku, Kv=w.Kv, lr=w.lr,
                                    beta1=w.beta1, beta2=w.beta2, eps=w.eps, rho=w.rho, x=tabs["x"], u=tabs["u"],
                                    v=tabs["v"], g=tabs["g"], vmax=tabs["vmax"],
                                    grad_dtype=B.BF16 if w.grad_bf16 else B.F32,
                                    flags=w.flags, init_mode=B.INIT_AS_IS, stream=stream.cuda_stream)
                res = {}
                for name, t in class_instants(w).items():
                    if not t or name == "x+u":
                        continue
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    B.desloc_step(ctx, t)
                    e0.record(stream)
                    for _ in range(3):
                        B.desloc_step(ctx, t)
                    e1.record(stream)
                    B.desloc_synchronize(ctx)
                    res[name + "_ms"] = e0.elapsed_time(e1) / 3
                    res[name + "_gbps"] = bytes_per_launch / (res[name + "_ms"] * 1e-3) / 1e9
                B.desloc_destroy(ctx)
                row[arrangement] = res
            rows.append(row)
        summary = {}
        for arrangement in ARRANGEMENTS:
            for cls in ("none", "x", "all"):
                vals = [r[arrangement][cls + "_gbps"] for r in rows if cls + "_gbps" in r[arrangement]]
                if vals:
                    summary[f"{arrangement}_{cls}_gbps_min_max"] = [min(vals), max(vals)]
        print(json.dumps({"mode": "placement-map", "workload": w.name, "pool_gib": args.placement_map,
                          "workload_gib": need / GiB, "summary": summary, "rows": rows}))
        return

    if args.realloc > 0:
        # The same binary, the same process, fresh allocations each round: how much of the spread in
        # the kernel time comes with where the arrays land in HBM.
        rounds = []
        for r in range(args.realloc):
            sess = DeslocSession(w, chunk_elems=args.chunk, stream=stream, layout=args.layout)
            sess.fill_gradients(0)
            for i in range(W):
                sess.step(10_000_019 + i)
            sess.step(0)
            sess.synchronize()
            rounds.append(time_classes(sess, stream, w, bytes_per_launch, reps=max(5, min(K, 10))))
            # hold on to a differently sized block so that the next round's arrays land elsewhere
            sess.close()
            del sess
            torch.cuda.empty_cache()
            pad = torch.empty((r + 1) * (64 << 20), dtype=torch.uint8, device="cuda:0")  # noqa: F841
        summary = {}
        for name in rounds[0]:
            ms = [rd[name]["ms"] for rd in rounds]
            gb = [rd[name]["gbps"] for rd in rounds]
            summary[name] = {"ms_min": min(ms), "ms_median": statistics.median(ms), "ms_max": max(ms),
                             "gbps_min": min(gb), "gbps_median": statistics.median(gb), "gbps_max": max(gb),
                             "frac_min": min(gb) / HBM_PEAK_GBPS, "frac_median": statistics.median(gb) / HBM_PEAK_GBPS,
                             "frac_max": max(gb) / HBM_PEAK_GBPS, "ms_all": ms}
        print(json.dumps({"mode": "realloc", "rounds": args.realloc, "workload": w.name, "layout": args.layout,
                          "bytes_per_launch_algorithmic": bytes_per_launch, "classes": summary}))
        return

    pool_gib = args.placement_pool_gib
    if pool_gib < 0:  # default: room to choose from, but never most of the device
        from paper_2505_22549_amd.runtime import PackedReplicas
        need = PackedReplicas.bytes_needed(w.numel, w.M, w.variant != B.SGDM, w.grad_bf16,
                                           bool(w.flags & B.FLAG_AMSGRAD))
        free, _ = torch.cuda.mem_get_info()
        pool_gib = min(2.1 * need, free - (24 << 30)) / (1 << 30)
        if pool_gib * (1 << 30) < 1.2 * need or need < (1 << 30):
            pool_gib = 0.0  # nothing to choose from (or a workload too small for placement to matter)
    if args.layout != "packed" or args.diagnostics:
        pool_gib = 0.0
    # the diagnostic's snapshot of u lives inside the groups, next to u (grouped layout)
    snapshots = ("u",) if args.diagnostics and args.layout == "grouped" and not args.snapshot_apart else ()
    sess = DeslocSession(w, chunk_elems=args.chunk, stream=stream, layout=args.layout,
                         placement_pool_gib=pool_gib, snapshots=snapshots)
    sess.fill_gradients(0)
    stream.synchronize()
    torch.cuda.synchronize()
    plan = B.desloc_get_plan(sess.ctx)

    # The first tenths of a second of GPU work after an idle stretch run at about half speed (clocks):
    # keep the memory system busy with a plain streaming kernel on a scratch buffer for a moment,
    # so that short configurations are not timed on the ramp.  Not a step: no state is touched.
    from paper_2505_22549_amd.inputs import generator as gen
    scratch = torch.zeros(1 << 28, dtype=torch.float32, device="cuda:0")  # 1 GiB
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < 0.3:
        for _ in range(20):
            gen.stream(scratch.data_ptr(), 1 << 28, 1 << 28, 4, 3, True, False, 16320, stream.cuda_stream)
        stream.synchronize()
    del scratch

    # warm-up on non-sync and sync instants (compiles nothing, but loads code objects)
    for i in range(W):
        sess.step(10_000_019 + i)
    sess.step(0)
    sess.synchronize()

    events = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    events[0].record(stream)
    for t in range(K):
        sess.step(t)
        events[t + 1].record(stream)
    sess.synchronize()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    per_step_ms = [events[i].elapsed_time(events[i + 1]) for i in range(K)]
    all_steps_ms = sum(per_step_ms) / K
    # The roofline figure is for the dominant kernel, the launch without a gate (for a single
    # replica every step is one); gated launches are reported per class in roofline_gated.
    ungated = [ms for t, ms in enumerate(per_step_ms) if sess.sync_mask(t) == 0 or w.M == 1]
    dominant = ungated if ungated else per_step_ms
    kernel_ms = sum(dominant) / len(dominant)
    value = updates_per_step * K / wall
    achieved = bytes_per_launch / (kernel_ms * 1e-3) / 1e9

    masks = {} if args.no_mask_classes else time_classes(sess, stream, w, bytes_per_launch)
    traffic, traffic_source = read_traffic(w.name)

    out = {
        "metric": "replica-param updates/sec per DES-LOC step",
        "value": value,
        "unit": "replica-param updates/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": wall * 1e3 / K,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "variant": ["adam", "adopt", "sgdm"][w.variant], "M": w.M,
                   "n_tensors": w.n_tensors, "numel_per_replica": w.total_numel,
                   "K": [w.Kx, w.Ku, w.Kv], "grad_dtype": "bf16" if w.grad_bf16 else "f32",
                   "clip": "global-norm" if args.norm_clip else "coordinate",
                   "ordering": "update-then-average" if (w.flags & B.FLAG_POST_AVERAGE) else "average-then-update",
                   "amsgrad": bool(w.flags & B.FLAG_AMSGRAD), "layout": args.layout,
                   **({"library": args.library, "library_env": {k: v for k, v in os.environ.items()
                                                                 if k.startswith("DESLOC_")}} if args.library else {}),
                   "placement": sess.placement,
                   "timed_steps": f"t=0..{K - 1}", **plan_dict(plan)},
        "hbm_gbps_algorithmic": achieved,
        "pct_of_hbm_peak": 100.0 * achieved / HBM_PEAK_GBPS,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     # not measured in this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, separate passes
                     "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": "desloc::step_kernel, launches without a gate" + (" + sumsq kernels" if args.norm_clip else ""),
                     "kernel_ms_avg": kernel_ms,
                     "kernel_ms_min": min(dominant), "kernel_ms_max": max(dominant),
                     "kernel_launches_timed": len(dominant), "all_steps_ms_avg": all_steps_ms,
                     "bytes_per_launch_algorithmic": bytes_per_launch},
        # the sync steps (Alg. 1 gates): same bytes per launch, each class timed on 5 launches
        "roofline_gated": {name: {"mask": m["mask"], "kernel_ms": m["ms"], "achieved": m["gbps"], "frac": m["frac"]}
                           for name, m in masks.items() if name != "none"},
        "mask_classes": masks,
    }
    gated_fracs = [m["frac"] for name, m in masks.items() if name != "none"]
    if gated_fracs:
        out["roofline_gated_min_frac"] = min(gated_fracs)
    if args.norm_clip:
        # the same step without the norm pass, same process, same arrays: what the norm pass adds
        plain = B.desloc_init(
            variant=w.variant, M=w.M, numel=w.numel, Kx=w.Kx, Ku=w.Ku, Kv=w.Kv, lr=w.lr, beta1=w.beta1,
            beta2=w.beta2, eps=w.eps, rho=w.rho, x=sess.mem.table(sess.mem.x), u=sess.mem.table(sess.mem.u),
            v=sess.mem.table(sess.mem.v), g=sess.mem.table(sess.mem.g), vmax=sess.mem.table(sess.mem.vmax),
            grad_dtype=B.BF16 if w.grad_bf16 else B.F32, flags=w.flags & ~B.FLAG_NORM_CLIP,
            init_mode=B.INIT_AS_IS, stream=stream.cuda_stream, chunk_elems=args.chunk)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        B.desloc_step(plain, 10_000_019)
        e0.record(stream)
        for i in range(5):
            B.desloc_step(plain, 10_000_020 + i)
        e1.record(stream)
        B.desloc_synchronize(plain)
        out["plain_step_ms_same_process"] = e0.elapsed_time(e1) / 5
        out["norm_pass_ms"] = kernel_ms - out["plain_step_ms_same_process"]
        B.desloc_destroy(plain)
    if args.diagnostics:
        snap, table = sess.mem.snapshot_buffer("u")
        torch.cuda.synchronize()
        B.desloc_snapshot_state(sess.ctx, B.U, table)
        for i in range(4):
            sess.step(20_000_003 + i)
        sess.synchronize()
        B.desloc_state_change(sess.ctx, B.U, B.ALL_TENSORS, table, w.M)  # warm-up
        t1 = time.perf_counter()
        change, base = B.desloc_state_change(sess.ctx, B.U, B.ALL_TENSORS, table, w.M)
        dt = time.perf_counter() - t1
        out["diagnostics"] = {"snapshot": "inside the groups" if sess.mem.array("snap_u") is not None else "own allocation",
                              "state_change_u_ms": dt * 1e3, "gbps": updates_per_step * 8 / dt / 1e9,
                              "relative_change_after_4_steps": [float(c / b) for c, b in zip(change, base)]}
        # the batched per-tensor form: asynchronous, timed with events on the stream
        ch = torch.zeros((w.n_tensors, w.M), device="cuda:0")
        bs = torch.zeros((w.n_tensors, w.M), device="cuda:0")
        torch.cuda.synchronize()
        B.desloc_state_change_tensors(sess.ctx, B.U, ch.data_ptr(), bs.data_ptr())
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(5):
            B.desloc_state_change_tensors(sess.ctx, B.U, ch.data_ptr(), bs.data_ptr())
        e1.record(stream)
        sess.synchronize()
        ms = e0.elapsed_time(e1) / 5
        e0.record(stream)
        B.desloc_snapshot_state(sess.ctx, B.U, table)
        e1.record(stream)
        sess.synchronize()
        ratio = (ch / bs).cpu().numpy()
        out["diagnostics"].update({
            "state_change_tensors_u_ms": ms, "state_change_tensors_gbps": updates_per_step * 8 / (ms * 1e-3) / 1e9,
            "state_change_tensors_frac_of_peak": updates_per_step * 8 / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "snapshot_u_ms": e0.elapsed_time(e1),
            "snapshot_gbps": updates_per_step * 8 / (e0.elapsed_time(e1) * 1e-3) / 1e9,
            "per_tensor_relative_change_min_max": [float(ratio.min()), float(ratio.max())]})
        del ch, bs
        del snap
    if args.calibration_copy_gib > 0:
        from paper_2505_22549_amd.inputs import generator as gen
        nbytes = int(args.calibration_copy_gib * (1 << 30)) // 16 * 16
        src = torch.ones(nbytes // 4, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            gen.calibration_copy(dst.data_ptr(), src.data_ptr(), nbytes, stream.cuda_stream)
        sess.synchronize()
        del src, dst
        out["calibration_copy_bytes"] = nbytes
    sess.close()
    del sess
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_sample_elems, args.cpu_seconds, bytes_per_update)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
