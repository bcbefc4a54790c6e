"""Parity of the paced launch shapes (persistent wavefronts on a clock timetable, used for arrays of
several hundred MiB; forced here from 128 MiB on with opal_set_pacing(2)) with the CPU oracle, through the C ABI.  The timetable only decides WHEN a
wavefront issues its loads and stores, so results must be the same bits whatever the timetable:
the default one, one that asks far too much (every wavefront always late, feedback busy), one
that asks far too little (every wavefront waits), no feedback, and pacing switched off."""
import numpy as np
import pytest
import torch

import opal_inputs as oi
import paper_2510_00932_amd as opal

pytestmark = pytest.mark.gpu

# kind: TB/s, store_at, second_input_at, gap, tolerance, feedback.  DEFAULTS = the library's own (launch_shapes.hpp).
DEFAULTS = {0: (7.10, 0.75, 0.0, 0.035, 400, True), 1: (7.10, 0.0, 0.0, 0.03, 400, True), 2: (7.60, 0.0, 0.25, 0.0, 0, False)}
TIMETABLES = {
    "default": DEFAULTS,
    "asks_too_much": {0: (40.0, 0.75, 0.0, 0.0, 0, True), 1: (40.0, 0.5, 0.2, 0.01, 0, True), 2: (40.0, 0.0, 0.25, 0.0, 0, True)},
    "asks_too_little": {0: (2.5, 0.75, 0.0, 0.02, 50, True), 1: (2.5, 0.6, 0.1, 0.02, 50, True), 2: (2.5, 0.0, 0.5, 0.05, 50, True)},
    "no_feedback_stores_free": {0: (7.0, 0.0, 0.0, 0.0, 200, False), 1: (7.1, 0.0, 0.0, 0.0, 200, False), 2: (7.6, 0.0, 0.0, 0.0, 0, False)},
}


def _configure(table):
    for kind, (tb, store_at, second_at, gap, tol, fb) in table.items():
        opal.opal_pacing_configure(kind, tb, store_at, second_at, gap, tol, fb)


@pytest.fixture()
def pacing():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    opal.load()
    opal.opal_set_pacing(2)        # paced wherever the shape fits, so that moderate sizes exercise it
    yield
    _configure(DEFAULTS)
    opal.opal_set_pacing(1)


@pytest.fixture(scope="module")
def parity():
    import parity as _parity
    return _parity


def _sizes(dtype):
    # 24 chunks of the one-input timetable and a ragged rest; and larger, with a long rest after the last whole chunk
    per = 8 if dtype == np.float64 else 4
    return [(192 << 20) // per + 12345, (256 << 20) // per + (5 << 20) // per + 3]


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("timetable", list(TIMETABLES))
def test_paced_chain_matches_oracle(parity, pacing, dtype, timetable):
    _configure(TIMETABLES[timetable])
    w = oi.workload(4)   # sign-mixed values, s = -0.75
    n_max = max(_sizes(dtype))
    full = [oi.uniform_array(w.seed, k, n_max, dtype, w.lo, w.hi, threads=16) for k in range(3)]
    cases = [(_sizes(dtype)[0], (1, 1, 1)), (_sizes(dtype)[1], (0, 0, 0))]
    if timetable == "default":
        cases += [(_sizes(dtype)[0], (1, 2, 3)), (_sizes(dtype)[0], (0, 1, 0))]   # inputs misaligned against the output
    for n, offsets in cases:
        print("paced chain: %s n=%d offsets=%s timetable=%s" % (np.dtype(dtype).name, n, offsets, timetable), flush=True)
        parity.run_chain([x[:n].copy() for x in full], w.s, offsets, check_all_arrays_each_step=False)
        parity.run_fresh([x[:n].copy() for x in full], w.s, offsets)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_paced_closed_forms(pacing, dtype):
    """Ramps (every element is its own index), constants, the vector on which a fused triad differs, and dot
    sums of integers (exact in any order, so the paced dot must hit them bit for bit)."""
    import gpu_harness
    import pins
    n = _sizes(dtype)[0]
    for offsets in [(0, 0, 0), (1, 1, 1)]:
        impl = gpu_harness.GpuImpl(offsets)
        pins.pin_ramp(impl, dtype, n)
        pins.pin_constant_fill(impl, dtype, n)
        pins.pin_fma_discriminator(impl, dtype, n=n)
        pins.pin_dot_closed_forms(impl, dtype, [n])


def test_pacing_off_gives_the_same_bits(pacing):
    import gpu_harness
    dtype = np.float64
    n = _sizes(dtype)[0]
    w = oi.workload(0)
    ha, hb, hc = (oi.uniform_array(w.seed, k, n, dtype, w.lo, w.hi, threads=16) for k in range(3))
    results = {}
    for on in (True, False):
        opal.opal_set_pacing(2 if on else 0)
        assert opal.opal_get_pacing() == (2 if on else 0)
        a, b, c = (gpu_harness.GuardedArray(n, dtype, 1).upload(h) for h in (ha, hb, hc))
        torch.cuda.synchronize()
        opal.opal_triad(a.ptr, b.ptr, c.ptr, w.s, n, opal.OPAL_F64)
        opal.opal_copy(a.ptr, c.ptr, n, opal.OPAL_F64)
        r = gpu_harness.dot_device(a.ptr, b.ptr, n, opal.OPAL_F64)
        torch.cuda.synchronize()
        assert a.guards_intact() and b.guards_intact() and c.guards_intact()
        results[on] = (a.download(), c.download(), r)
    assert np.array_equal(results[True][0].view(np.uint64), results[False][0].view(np.uint64))
    assert np.array_equal(results[True][1].view(np.uint64), results[False][1].view(np.uint64))
    # the two dot shapes add in different orders: same value to rounding, each within tolerance of the oracle
    import oracle
    ref = oracle.dot(results[True][0], hb)
    for on in (True, False):
        assert abs(results[on][2] - ref) <= 1e-12 * abs(ref)


def test_paced_dot_is_reproducible(pacing):
    n = _sizes(np.float64)[0]
    ha = oi.uniform_array(5, 0, n, np.float64, -1.0, 1.0, threads=16)
    hb = oi.uniform_array(5, 1, n, np.float64, -1.0, 1.0, threads=16)
    a, b = torch.from_numpy(ha).cuda(), torch.from_numpy(hb).cuda()
    res = torch.full((2,), float("nan"), dtype=torch.float64, device="cuda:0")
    need = opal.opal_dot_workspace_bytes(n, opal.OPAL_F64)
    ws = torch.full((need // 8,), float("nan"), dtype=torch.float64, device="cuda:0")
    torch.cuda.synchronize()
    opal.opal_dot(a, b, n, opal.OPAL_F64, ws, need, res.data_ptr())
    opal.opal_dot(a, b, n, opal.OPAL_F64, ws, need, res.data_ptr() + 8)
    torch.cuda.synchronize()
    r = res.cpu().numpy()
    assert r[0] == r[1]
    import oracle
    ref, scale = oracle.dot(ha, hb), oracle.dot_abs(ha, hb)
    assert abs(r[0] - ref) <= 1e-12 * abs(ref), (r[0], ref, scale / abs(ref))


def test_paced_kernels_replay_from_a_hip_graph(parity, pacing):
    """The timetable keeps its feedback in device words that outlive a launch, and tells launches apart by a
    time stamp taken on the device: a captured paced kernel must replay like any other (same bits as the
    oracle after every replay, eager work in between)."""
    import gpu_harness
    from test_gpu_parity import graph_replay_check
    graph_replay_check(parity, gpu_harness, _sizes(np.float64)[0], np.float64, offsets=(1, 1, 1), replays=3)


def test_overlapping_paced_calls_on_two_streams(pacing):
    """Paced kernels on one GPU share the timetable's feedback words, so two that overlap may read each other's
    lateness reports: that may cost time, never a result bit.  Two independent chains on two streams, launched
    alternately without synchronising in between, each compared with the oracle."""
    import oracle
    n = _sizes(np.float64)[0]
    w = oi.workload(4)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    host, dev, res, ws = [], [], [], []
    need = opal.opal_dot_workspace_bytes(n, opal.OPAL_F64)
    for j in range(2):
        h = [oi.uniform_array(w.seed + j, k, n, np.float64, w.lo, w.hi, threads=16) for k in range(3)]
        host.append(h)
        dev.append([torch.from_numpy(x).cuda() for x in h])
        res.append(torch.full((1,), float("nan"), dtype=torch.float64, device="cuda:0"))
        ws.append(torch.empty(need // 8, dtype=torch.float64, device="cuda:0"))
    torch.cuda.synchronize()
    dt = opal.OPAL_F64
    for rep in range(3):
        for call in range(5):
            for j in range(2):
                a, b, c = dev[j]
                st = streams[j]
                if call == 0:
                    opal.opal_copy(a, c, n, dt, st)
                elif call == 1:
                    opal.opal_scale(b, c, w.s, n, dt, st)
                elif call == 2:
                    opal.opal_add(a, b, c, n, dt, st)
                elif call == 3:
                    opal.opal_triad(a, b, c, w.s, n, dt, st)
                else:
                    opal.opal_dot(a, b, n, dt, ws[j], need, res[j].data_ptr(), st)
    torch.cuda.synchronize()
    for j in range(2):
        ha, hb, hc = host[j]
        for rep in range(3):
            oracle.copy(ha, hc)
            oracle.scale(hb, hc, w.s)
            oracle.add(ha, hb, hc)
            oracle.triad(ha, hb, hc, w.s)
        ref = oracle.dot(ha, hb)
        for name, d, h in zip("abc", dev[j], (ha, hb, hc)):
            assert np.array_equal(d.cpu().numpy().view(np.uint64), h.view(np.uint64)), "chain %d, array %s" % (j, name)
        got = float(res[j].item())
        assert abs(got - ref) <= 1e-12 * abs(ref), (j, got, ref)


@pytest.mark.parametrize("setting", [0, 2])
def test_every_order_of_the_second_input_gives_the_same_bits(parity, pacing, setting):
    """The order in which a paced Add or Triad loads the runs of its second input (one of two orders matched to the
    first input's memory-channel classes, tried in turn and then learnt; the first input's own order when switched
    off) decides timing only.  The chain calls Add and Triad several times on the same arrays, so both matched
    orders run."""
    w = oi.workload(4)
    n = _sizes(np.float64)[0]
    arrays = [oi.uniform_array(w.seed, k, n, np.float64, w.lo, w.hi, threads=16) for k in range(3)]
    try:
        opal.opal_set_matched_order(setting)
        parity.run_chain([x.copy() for x in arrays], w.s, (0, 1, 0), check_all_arrays_each_step=False)
    finally:
        opal.opal_set_matched_order(1)
    parity.run_chain([x.copy() for x in arrays], w.s, (0, 1, 0), check_all_arrays_each_step=False)


def test_the_faster_matched_order_is_learnt(pacing):
    """Eight paced Add launches on the same arrays: the library has timed both matched orders twice and settled
    for the faster one; told to time the other order first it settles for the same one (where the two differ by
    more than launches of one order do), and other arrays start from nothing.  The sums are exact throughout."""
    n = (1 << 27) + 4096
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(20251127)
    a, b = (torch.rand(n, dtype=torch.float64, device=dev, generator=gen) + 0.5 for _ in range(2))
    c = torch.empty(n, dtype=torch.float64, device=dev)
    expect = a + b   # one rounding per element: the same bits as the oracle's sum
    stream = torch.cuda.current_stream()
    picks = []
    try:
        for first in (1, 2):
            opal.opal_set_matched_order(first)
            assert opal.opal_matched_order_state(c.data_ptr(), a.data_ptr(), b.data_ptr(), n, opal.OPAL_F64)[0] == 0
            for launch in range(8):
                c.zero_()
                opal.opal_add(a.data_ptr(), b.data_ptr(), c.data_ptr(), n, opal.OPAL_F64, stream)
                assert torch.equal(c, expect), "launch %d, setting %d" % (launch, first)
                launches, best0, best1, nxt = opal.opal_matched_order_state(c.data_ptr(), a.data_ptr(), b.data_ptr(),
                                                                            n, opal.OPAL_F64)
                assert launches == launch + 1
                if launch < 3:   # the first four launches alternate, starting with the order named first
                    assert nxt == ((first - 1) ^ (launch + 1)) & 1
            assert best0 != 0xFFFFFFFF and best1 != 0xFFFFFFFF
            assert nxt == (1 if best1 < best0 else 0)
            print("setting %d: shortest %d and %d ticks, order %d" % (first, best0, best1, nxt), flush=True)
            picks.append((nxt, abs(best1 - best0) / min(best0, best1)))
            # another pair of arrays has its own state
            assert opal.opal_matched_order_state(c.data_ptr(), b.data_ptr(), a.data_ptr(), n, opal.OPAL_F64)[0] == 0
        if all(gap > 0.025 for _, gap in picks):
            assert picks[0][0] == picks[1][0]
        # after 128 launches both orders are timed afresh (setting 2 is still on: order 1 goes first)
        for launch in range(8, 133):
            expected_order = opal.opal_matched_order_state(c.data_ptr(), a.data_ptr(), b.data_ptr(), n, opal.OPAL_F64)[3]
            if 128 <= launch < 132:
                assert expected_order == (1 ^ (launch - 128)) & 1, launch
            c.zero_()
            opal.opal_add(a.data_ptr(), b.data_ptr(), c.data_ptr(), n, opal.OPAL_F64, stream)
            if launch % 16 == 0 or launch >= 126:
                assert torch.equal(c, expect), "launch %d" % launch
        launches, best0, best1, nxt = opal.opal_matched_order_state(c.data_ptr(), a.data_ptr(), b.data_ptr(), n, opal.OPAL_F64)
        assert launches == 133 and best0 != 0xFFFFFFFF and best1 != 0xFFFFFFFF and nxt == (1 if best1 < best0 else 0)
    finally:
        opal.opal_set_matched_order(1)


@pytest.mark.parametrize("dtype", [torch.float64, torch.float32])
def test_learning_the_order_keeps_triad_exact(pacing, dtype):
    """Twelve paced Triad launches on the same arrays, fp64 and fp32: whichever order a launch uses, the result is
    the two-rounding triad of the inputs, bit for bit (torch's own mul and add round once each)."""
    n = (1 << 27) + 12345 if dtype == torch.float64 else (1 << 28) + 12345
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    b, c = (torch.rand(n, dtype=dtype, device=dev, generator=gen) - 0.5 for _ in range(2))
    a = torch.empty(n, dtype=dtype, device=dev)
    s = -0.75
    expect = torch.add(b, torch.mul(c, s))   # product rounded, then sum rounded
    code = opal.OPAL_F64 if dtype == torch.float64 else opal.OPAL_F32
    stream = torch.cuda.current_stream()
    opal.opal_set_matched_order(1)
    seen = set()
    for launch in range(12):
        seen.add(opal.opal_matched_order_state(a.data_ptr(), b.data_ptr(), c.data_ptr(), n, code)[3])
        a.fill_(float("nan"))
        opal.opal_triad(a.data_ptr(), b.data_ptr(), c.data_ptr(), s, n, code, stream)
        assert torch.equal(a, expect), "launch %d" % launch
    assert seen == {0, 1}


def test_pacing_configure_rejects_bad_values():
    for args in ((3, 7.0, 0.5, 0.0, 0.0, 100, 1), (-1, 7.0, 0.5, 0.0, 0.0, 100, 1), (0, 0.0, 0.5, 0.0, 0.0, 100, 1),
                 (0, 1e9, 0.5, 0.0, 0.0, 100, 1), (0, 7.0, 1.0, 0.0, 0.0, 100, 1), (0, 7.0, -0.1, 0.0, 0.0, 100, 1),
                 (2, 7.0, 0.0, 1.5, 0.0, 100, 1), (0, float("nan"), 0.5, 0.0, 0.0, 100, 1), (0, 7.0, 0.5, 0.0, 0.3, 100, 1), (0, 7.0, 0.5, 0.0, 0.0, 100, 1, 9)):
        with pytest.raises(opal.OpalError) as e:
            opal.opal_pacing_configure(*args)
        assert e.value.status == 6
