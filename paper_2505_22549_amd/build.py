"""Builds the gfx950 libraries in-tree with hipcc (cross-compiles without a GPU).

    python -m paper_2505_22549_amd.build
    python -m paper_2505_22549_amd.build --out /tmp/libdesloc_tuning.so DESLOC_TUNING=1   (a measurement build)

Outputs (git-ignored, shipped to the GPU machine with the tree):
    paper_2505_22549_amd/libdesloc.so          the DES-LOC step library (C ABI: include/desloc.h)
    paper_2505_22549_amd/inputs/libdesloc_inputs.so   the synthetic-input generator
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
BUILD = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libdesloc.so")
INPUTS_SRC = os.path.join(PKG, "inputs", "csrc", "desloc_inputs.hip")
INPUTS_LIB = os.path.join(PKG, "inputs", "libdesloc_inputs.so")

ARCH = "gfx950"
# -ffp-contract=off + correctly rounded divide/sqrt: one IEEE rounding per fp32 operation,
# in source order.  Packed-fp32 instructions are disabled as required on the test machines.
HIPCC_FLAGS = [
    f"--offload-arch={ARCH}", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-fast-math",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]

SOURCES = [
    "desloc_api.hip",
    "desloc_kernels_aux.hip",
    "desloc_kernels_adam.hip",
    "desloc_kernels_adopt.hip",
    "desloc_kernels_adopt_t0.hip",
    "desloc_kernels_sgdm.hip",
    "desloc_kernels_norm.hip",
    "desloc_kernels_post_adam.hip",
    "desloc_kernels_post_adam_ams.hip",
    "desloc_kernels_post_sgdm.hip",
]


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the packed-fp32 target feature: harmless, filtered
    out = "\n".join(l for l in proc.stdout.splitlines()
                    if "packed-fp32-ops" not in l and l.strip())
    if proc.returncode != 0:
        raise RuntimeError(f"command failed ({proc.returncode}): {' '.join(cmd)}\n{out}")
    if out:
        print(out, file=sys.stderr)


def build(extra_defines=(), jobs: int = 8, out: str = LIB) -> None:
    """Compile everything, every time it is called.  `out`: where the step library goes; a build
    with extra defines for measurements (e.g. DESLOC_TUNING=1) belongs somewhere else than the
    product library's place (bench.py --library loads it)."""
    variant = out != LIB
    bdir = BUILD + ("_variant" if variant else "")
    os.makedirs(bdir, exist_ok=True)
    defs = [f"-D{d}" for d in extra_defines]
    objs = []
    cmds = []
    for s in SOURCES:
        o = os.path.join(bdir, s.replace(".hip", ".o"))
        objs.append(o)
        cmds.append(["hipcc", *HIPCC_FLAGS, *defs, "-I", CSRC, "-c", os.path.join(CSRC, s), "-o", o])
    if not variant:
        cmds.append(["hipcc", *HIPCC_FLAGS, "-shared", INPUTS_SRC, "-o", INPUTS_LIB])
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        list(ex.map(_run, cmds))
    _run(["hipcc", f"--offload-arch={ARCH}", "-shared", "-fPIC", *objs, "-o", out])


if __name__ == "__main__":
    # python -m paper_2505_22549_amd.build [--out PATH] [DEFINE[=VALUE] ...]
    args = sys.argv[1:]
    out = LIB
    if args[:1] == ["--out"]:
        out, args = os.path.abspath(args[1]), args[2:]
    build(extra_defines=args, out=out)
    print(out)
    if out == LIB:
        print(INPUTS_LIB)
