"""CPU-only checks of bench.py's command-line contract (no GPU work)."""
import os
import subprocess
import sys

from conftest import ROOT


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True,
                          text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    p = _run("--gpus", "2")
    assert p.returncode == 2
    assert "one gpu" in p.stderr.lower() or "--gpus 1" in p.stderr
    assert p.stdout.strip() == ""


def test_help_lists_the_contract_flags():
    p = _run("--help")
    assert p.returncode == 0
    for flag in ("--gpus", "--steps", "--warmup", "--config", "--norm-clip", "--post-average", "--amsgrad"):
        assert flag in p.stdout


def test_traffic_summary_is_read_from_profiles():
    sys.path.insert(0, ROOT)
    import bench
    t = bench.read_traffic("c5_adam_1p7B_M4")
    alg = 1713639424 * 4 * 28
    assert t is not None and abs(t - alg) / alg < 0.01  # measured HBM traffic = algorithmic bytes
    assert bench.read_traffic("no_such_workload") is None
