"""bench.py's command line and its one-line JSON contract."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0
    assert "single-GPU" in p.stderr and p.stdout.strip() == ""


def test_bench_does_not_route_through_the_oracle():
    """The oracle may only appear in the CPU-baseline leg (imported inside it), never at module level."""
    import ast
    tree = ast.parse(open(BENCH).read())
    top = [n for n in tree.body if isinstance(n, (ast.Import, ast.ImportFrom))]
    names = {a.name for n in top for a in n.names} | {n.module for n in top if isinstance(n, ast.ImportFrom)}
    assert "oracle" not in names
    for rel in ("paper_2510_00932_amd/__init__.py", "paper_2510_00932_amd/binding.py", "paper_2510_00932_amd/build.py"):
        src = open(os.path.join(ROOT, rel)).read()
        assert "import oracle" not in src and "from oracle" not in src


@pytest.mark.gpu
def test_json_line_on_a_small_workload():
    p = subprocess.run([sys.executable, BENCH, "--steps", "3", "--warmup", "1", "--workload", "n2p20_f64",
                        "--n", "300007", "--offset-elems", "1"], capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [ln for ln in p.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["unit"] == "GB/s" and d["vs_baseline"] is None
    assert d["config"]["workload"].startswith("n2p20_f64") and d["config"]["n"] == 300007
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s"
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3
    assert d["cpu_baseline"]["kind"] == "oracle" and d["cpu_baseline"]["cores"] == 1
    assert d["check_vs_oracle"]["elementwise_bit_exact"] is True
    assert set(d["kernels"]) == {"copy", "scale", "add", "triad", "dot"}


@pytest.mark.gpu
def test_placement_scan_prints_every_setting():
    """The scan's JSON line has, for every skew, the three kernels under all four settings and leaves the library's
    switches as it found them (the scan runs in a process of its own, so only the line can be checked here)."""
    p = subprocess.run([sys.executable, BENCH, "--placement-scan", "0,1024", "--steps", "3", "--n", str((1 << 26) + 4096)],
                       capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [ln for ln in p.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert [r["skew_bytes"] for r in d["results"]] == [0, 1024]
    for r in d["results"]:
        for kernel in ("copy", "add", "triad"):
            for setting in ("paced", "paced_other_start", "paced_same_order", "ordered"):
                assert 20.0 < r["%s_%s" % (kernel, setting)] < 100.0, (kernel, setting, r)
