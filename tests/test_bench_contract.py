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


def test_help_lists_the_measurement_modes():
    p = _run("--help")
    for flag in ("--layout", "--realloc", "--stream-ceiling", "--stream-spread", "--replica-sweep", "--placement-map",
                 "--library"):
        assert flag in p.stdout
    assert "grouped" in p.stdout and "packed" in p.stdout and "separate" in p.stdout


def test_a_missing_library_build_is_refused_before_any_gpu_work():
    p = _run("--library", "/nonexistent/libdesloc_other.so")
    assert p.returncode == 2 and "does not exist" in p.stderr


def test_traffic_figure_names_its_source(tmp_path, monkeypatch):
    """roofline.traffic is a figure from an earlier rocprofv3 --pmc pass, not a measurement of the
    run: read_traffic returns it together with the summary file it came from, or (None, None)."""
    sys.path.insert(0, ROOT)
    import bench
    (tmp_path / "profiles").mkdir()
    (tmp_path / "profiles" / "pmc_traffic_some_workload.txt").write_text(
        "# comment = 5\nFETCH_BYTES_PER_LAUNCH = 1000 bytes\nWRITE_BYTES_PER_LAUNCH = 750\nOTHER = x\n")
    (tmp_path / "profiles" / "pmc_traffic_half.txt").write_text("FETCH_BYTES_PER_LAUNCH = 1000\n")
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    assert bench.read_traffic("some_workload") == (1750.0, os.path.join("profiles", "pmc_traffic_some_workload.txt"))
    assert bench.read_traffic("half") == (None, None)
    assert bench.read_traffic("no_such_workload") == (None, None)
