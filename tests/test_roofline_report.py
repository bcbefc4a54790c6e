"""The roofline-position report (observed against peak per component) on a stored rocprofv3 sample."""
import os

import pytest

from paper_2510_00932_amd import roofline_report as rr

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
SAMPLE = os.path.join(GOLDEN, "rocprof_n2p28_f64")                 # index-ordered shapes
SAMPLE_PACED = os.path.join(GOLDEN, "rocprof_n2p28_f64_paced")     # paced shapes (the default at this size)


@pytest.fixture(scope="module", params=[SAMPLE, SAMPLE_PACED], ids=["ordered", "paced"])
def sample(request):
    return request.param


@pytest.fixture(scope="module")
def report(sample):
    return rr.analyse(sample, 1 << 28, "f64")


def test_every_kernel_is_reported(report):
    results, lines = report
    assert [name for name, _ in results] == ["copy", "scale", "add", "triad", "dot"]
    assert any(line.startswith("Roofline position") for line in lines)


def test_bandwidth_is_bytes_over_time(report, sample):
    results = dict(report[0])
    n = 1 << 28
    for name, words in (("copy", 2), ("scale", 2), ("add", 3), ("triad", 3), ("dot", 2)):
        m = results[name]
        assert m["algorithmic_bytes"] == words * 8 * n
        assert m["hbm_bytes_per_s"] == pytest.approx(m["algorithmic_bytes"] / m["seconds"])
        assert m["hbm_frac"] == pytest.approx(m["hbm_bytes_per_s"] / 8.0e12)
        assert 0.5 < m["hbm_frac"] < 1.0
    # dot's time is both passes together
    stats = rr.read_kernel_stats(sample)
    t1 = rr.pick(stats, "dot_partial_kernel" if sample == SAMPLE else "paced_dot_kernel")[1]
    t2 = rr.pick(stats, "dot_final_kernel")[1]
    assert results["dot"]["seconds"] == pytest.approx((t1 + t2) * 1e-9)


def test_counters_are_calibrated_against_the_known_copy(report, sample):
    results = dict(report[0])
    counters = rr.read_counters(sample)
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


def _write_csvs(tmp_path, stats_rows, counter_rows):
    with open(tmp_path / "r_kernel_stats.csv", "w") as f:
        f.write('"Name","Calls","TotalDurationNs","AverageNs","Percentage","MinNs","MaxNs","StdDev"\n')
        for name, avg_ns in stats_rows:
            f.write('"%s",10,%d,%f,1.0,%d,%d,0.0\n' % (name, int(avg_ns * 10), avg_ns, int(avg_ns), int(avg_ns)))
    with open(tmp_path / "r_counter_collection.csv", "w") as f:
        f.write('"Kernel_Name","Counter_Name","Counter_Value"\n')
        for name, counter, value in counter_rows:
            f.write('"%s","%s",%f\n' % (name, counter, value))


def test_cache_levels_are_compared_with_their_peaks(tmp_path):
    """L2 and L1 carry the algorithmic bytes once; the report states their rate against the per-level peak
    and the request size the counters imply, and calls both under-used."""
    n = 1 << 28
    paced = "void opal::paced_stream_kernel<double, (opal::Op)3, 4, true>(double*, double const*, double const*, double, opal::plan::Paced, opal::Pace)"
    alg = 24 * n
    _write_csvs(tmp_path, [(paced, 920000.0)],
                [(paced, "TCC_REQ_sum", alg / 128), (paced, "TCP_TCC_READ_REQ_sum", 16 * n / 64),
                 (paced, "TCP_TCC_WRITE_REQ_sum", 8 * n / 64), (paced, "TCP_TOTAL_ACCESSES_sum", alg / 1024)])
    results, lines = rr.analyse(str(tmp_path), n, "f64")
    m = dict(results)["triad"]
    assert m["l2_bytes_per_request"] == pytest.approx(128.0) and m["l1_l2_bytes_per_request"] == pytest.approx(64.0)
    assert m["l2_frac"] == pytest.approx(alg / 920e-6 / (8 * 16 * 128 * 2.4e9))
    assert m["l1_frac"] == pytest.approx(alg / 920e-6 / (256 * 64 * 2.4e9))
    text = "\n".join(lines)
    assert "L2: " in text and "L1 (vector cache to L2)" in text
    assert "L2 is under-used" in text and "L1 is under-used" in text
    assert "HBM is the binding component" in text


def test_lds_kernel_is_compared_with_read_and_write_rates(tmp_path):
    name = "void opal::lds_stream_kernel<double, 256>(double const*, double*, double, unsigned int)"
    n, rep = 256 * 5 * 8 * 2048, 600
    lds_bytes = 32.0 * (n * 8 / 16) * rep
    t_ns = lds_bytes / 70.0e12 * 1e9          # 70 TB/s
    cycles = t_ns * 2.4                       # per compute unit
    _write_csvs(tmp_path, [(name, t_ns)], [(name, "SQ_LDS_BANK_CONFLICT", 0.0), (name, "SQ_LDS_IDX_ACTIVE", 0.5 * 256 * cycles),
                                           (name, "SQ_INSTS_LDS", 0.5 * 256 * cycles / 6.0)])
    lines = rr.analyse_lds(str(tmp_path), n, "f64", rep)
    text = "\n".join(lines)
    per_clk = 70.0e12 / 256 / 2.4e9           # 113.9 bytes per clock per compute unit
    assert "70000 GB/s" in text and "%.1f bytes" % per_clk in text
    assert "reads alone: %.1f %%" % (100 * per_clk / 2 / 256) in text
    # a pipe that reads at 209 and writes at 77 bytes per clock moves 2 / (1/209 + 1/77) = 112.5 when it does both in turn
    assert rr.lds_composed_rate() == pytest.approx(112.54, abs=0.01)
    assert rr.lds_composed_rate(128.0, 128.0) == pytest.approx(128.0)
    assert "at %.0f %% of that" % (100 * per_clk / 112.54) in text
    assert "bank conflicts: 0.00 %" in text and "index unit active 50 %" in text and "6.0 cycles per LDS instruction" in text
    assert "write rate is the binding component" in text and "read path is under-used" in text
    assert rr.analyse_lds(str(tmp_path), n, "f32", rep) == []     # no fp32 kernel in this run


def test_slow_lds_kernel_is_called_under_used(tmp_path):
    name = "void opal::lds_stream_kernel<double, 256>(double const*, double*, double, unsigned int)"
    n, rep = 256 * 5 * 8 * 2048, 600
    t_ns = 32.0 * (n * 8 / 16) * rep / 40.0e12 * 1e9
    _write_csvs(tmp_path, [(name, t_ns)], [])
    text = "\n".join(rr.analyse_lds(str(tmp_path), n, "f64", rep))
    assert "the LDS is under-used (58 % of what" in text
