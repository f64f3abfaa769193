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
8 TB/s) and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import math
import os
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
    ap.add_argument("--calibration-copy-gib", type=float, default=0.0,
                    help="also run a plain copy kernel of this many GiB (read N, write N) three times: "
                         "the known-size yardstick for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs")
    return ap.parse_args()


def read_traffic(workload_name: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, if there is one."""
    path = os.path.join(ROOT, "profiles", f"pmc_traffic_{workload_name}.txt")
    if not os.path.exists(path):
        return None
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
        return vals["FETCH_BYTES_PER_LAUNCH"] + vals["WRITE_BYTES_PER_LAUNCH"]
    return None


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

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)

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
    K = args.steps if args.steps > 0 else w.steps
    W = args.warmup
    stream = torch.cuda.Stream(device="cuda:0")  # default priority
    sess = DeslocSession(w, chunk_elems=args.chunk, stream=stream)
    sess.fill_gradients(0)
    stream.synchronize()
    torch.cuda.synchronize()
    plan = B.desloc_get_plan(sess.ctx)

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
    # replica every step is one); gated launches are reported per class below.
    ungated = [ms for t, ms in enumerate(per_step_ms) if sess.sync_mask(t) == 0 or w.M == 1]
    dominant = ungated if ungated else per_step_ms
    kernel_ms = sum(dominant) / len(dominant)
    updates_per_step = w.M * w.total_numel
    value = updates_per_step * K / wall
    bytes_per_launch = updates_per_step * bytes_per_update
    achieved = bytes_per_launch / (kernel_ms * 1e-3) / 1e9

    masks = {}
    if not args.no_mask_classes:
        lcm = math.lcm(*[k for k in (w.Kx, w.Ku, w.Kv) if k]) if any((w.Kx, w.Ku, w.Kv)) else 0
        cand = {"none": 10_000_019, "x": w.Kx, "x+u": w.Ku, "all": lcm}
        for name, t in cand.items():
            if not t:
                continue
            if name != "none" and t == 0:
                continue
            reps = 5
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            sess.step(t)
            e0.record(stream)
            for _ in range(reps):
                sess.step(t)
            e1.record(stream)
            sess.synchronize()
            ms = e0.elapsed_time(e1) / reps
            masks[name] = {"t": t, "mask": sess.sync_mask(t), "ms": ms,
                           "gbps": bytes_per_launch / (ms * 1e-3) / 1e9}

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
                   "amsgrad": bool(w.flags & B.FLAG_AMSGRAD),
                   "timed_steps": f"t=0..{K - 1}", "segments": int(plan.n_segments),
                   "chunk_elems": int(plan.chunk_elems), "chunks": int(plan.n_chunks),
                   "workgroups_per_ungated_step": int(plan.n_chunks) * w.M, "lanes_per_workgroup": 64},
        "hbm_gbps_algorithmic": achieved,
        "pct_of_hbm_peak": 100.0 * achieved / HBM_PEAK_GBPS,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": read_traffic(w.name),  # rocprofv3 --pmc, profiles/pmc_traffic_*.txt
                     "kernel": "desloc::step_kernel, launches without a gate" + (" + sumsq kernels" if args.norm_clip else ""),
                     "kernel_ms_avg": kernel_ms,
                     "kernel_ms_min": min(dominant), "kernel_ms_max": max(dominant),
                     "kernel_launches_timed": len(dominant), "all_steps_ms_avg": all_steps_ms,
                     "bytes_per_launch_algorithmic": bytes_per_launch},
        "mask_classes": masks,
    }
    if args.diagnostics:
        snap = torch.zeros_like(sess.mem.u)
        table = sess.mem.table(snap)
        torch.cuda.synchronize()
        B.desloc_snapshot_state(sess.ctx, B.U, table)
        for i in range(4):
            sess.step(20_000_003 + i)
        sess.synchronize()
        B.desloc_state_change(sess.ctx, B.U, B.ALL_TENSORS, table, w.M)  # warm-up
        t1 = time.perf_counter()
        change, base = B.desloc_state_change(sess.ctx, B.U, B.ALL_TENSORS, table, w.M)
        dt = time.perf_counter() - t1
        out["diagnostics"] = {"state_change_u_ms": dt * 1e3, "gbps": updates_per_step * 8 / dt / 1e9,
                              "relative_change_after_4_steps": [float(c / b) for c, b in zip(change, base)]}
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
