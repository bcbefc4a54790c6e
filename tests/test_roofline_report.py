"""The roofline-position report (observed against peak per component) on a stored rocprofv3 sample."""
import os

import pytest

from paper_2510_00932_amd import roofline_report as rr

SAMPLE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "rocprof_n2p28_f64")


@pytest.fixture(scope="module")
def report():
    return rr.analyse(SAMPLE, 1 << 28, "f64")


def test_every_kernel_is_reported(report):
    results, lines = report
    assert [name for name, _ in results] == ["copy", "scale", "add", "triad", "dot"]
    assert any(line.startswith("Roofline position") for line in lines)


def test_bandwidth_is_bytes_over_time(report):
    results = dict(report[0])
    n = 1 << 28
    for name, words in (("copy", 2), ("scale", 2), ("add", 3), ("triad", 3), ("dot", 2)):
        m = results[name]
        assert m["algorithmic_bytes"] == words * 8 * n
        assert m["hbm_bytes_per_s"] == pytest.approx(m["algorithmic_bytes"] / m["seconds"])
        assert m["hbm_frac"] == pytest.approx(m["hbm_bytes_per_s"] / 8.0e12)
        assert 0.5 < m["hbm_frac"] < 1.0
    # dot's time is both passes together
    stats = rr.read_kernel_stats(SAMPLE)
    t1 = rr.pick(stats, "dot_partial_kernel")[1]
    t2 = rr.pick(stats, "dot_final_kernel")[1]
    assert results["dot"]["seconds"] == pytest.approx((t1 + t2) * 1e-9)


def test_counters_are_calibrated_against_the_known_copy(report):
    results = dict(report[0])
    counters = rr.read_counters(SAMPLE)
    cal = rr.pick(counters["FETCH_SIZE"], rr.CAL_KERNEL)
    f = rr.pick(counters["FETCH_SIZE"], "(opal::Op)3")
    w = rr.pick(counters["WRITE_SIZE"], "(opal::Op)3")
    calw = rr.pick(counters["WRITE_SIZE"], rr.CAL_KERNEL)
    want = f * (1 << 30) / cal + w * (1 << 30) / calw
    assert results["triad"]["hbm_traffic_bytes"] == pytest.approx(want)
    for name in ("copy", "scale", "add", "triad", "dot"):
        assert 0.99 < results[name]["traffic_over_algorithmic"] < 1.01


def test_verdicts():
    assert any("binding" in v for v in rr.verdicts({"hbm_frac": 0.85}))
    assert any("under-used" in v for v in rr.verdicts({"hbm_frac": 0.4}))
    assert any("more than the algorithm needs" in v for v in rr.verdicts({"hbm_frac": 0.8, "traffic_over_algorithmic": 1.3}))
    assert any("write path" in v for v in rr.verdicts({"hbm_frac": 0.8, "ea_write_stall_frac": 0.2}))
    assert not any("write path" in v for v in rr.verdicts({"hbm_frac": 0.8, "ea_write_stall_frac": 0.01}))


def test_missing_counters_are_left_out(tmp_path):
    import shutil
    shutil.copy(os.path.join(SAMPLE, "sample_kernel_stats.csv"), tmp_path / "x_kernel_stats.csv")
    results, lines = rr.analyse(str(tmp_path), 1 << 28, "f64")
    m = dict(results)["copy"]
    assert "hbm_frac" in m and "l2_hit_rate" not in m and "hbm_traffic_bytes" not in m
