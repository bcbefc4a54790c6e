"""record_traffic.py's arithmetic on the stored rocprofv3 sample: counters are scaled by what the
1 GiB calibration copy reads, and the record carries the digest of the kernel sources."""
import json
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAMPLES = [os.path.join(ROOT, "tests", "golden", d) for d in ("rocprof_n2p28_f64", "rocprof_n2p28_f64_paced")]


@pytest.mark.parametrize("SAMPLE", SAMPLES, ids=["ordered", "paced"])
def test_traffic_record_from_the_sample(tmp_path, monkeypatch, SAMPLE):
    sys.path.insert(0, ROOT)
    from paper_2510_00932_amd import record_traffic as rt
    for sub in ("f", "w"):
        os.makedirs(tmp_path / sub)
        shutil.copy(os.path.join(SAMPLE, "sample_counter_collection.csv"), tmp_path / sub / "x_counter_collection.csv")
    monkeypatch.setattr(rt, "HERE", str(tmp_path))
    monkeypatch.setattr(sys, "argv", ["record_traffic.py", str(tmp_path / "f"), str(tmp_path / "w"), "n2p28_f64"])
    rt.main()
    rec = json.load(open(tmp_path / "measured_traffic.json"))
    assert rec["source_digest"] == rt.source_digest()
    w = rec["workloads"]["n2p28_f64"]
    n = 1 << 28
    for name, bytes_per_elem in (("copy", 16), ("scale", 16), ("add", 24), ("triad", 24), ("dot", 16)):
        assert abs(w[name] / (bytes_per_elem * n) - 1.0) < 0.01, name


def test_bench_uses_the_record_only_for_matching_sources():
    sys.path.insert(0, ROOT)
    import bench
    rec = json.load(open(os.path.join(ROOT, "paper_2510_00932_amd", "measured_traffic.json")))
    got = bench.measured_traffic("n2p28_f64", "triad")
    if rec["source_digest"] == bench.kernel_source_digest():
        assert got == rec["workloads"]["n2p28_f64"]["triad"]
    else:
        assert got is None
    assert bench.measured_traffic("no_such_workload", "triad") is None
