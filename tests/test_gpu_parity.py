"""Parity of the HIP kernels with the CPU oracle, through the C ABI, on a real MI355X.

Elementwise kernels: bit-exact.  Dot: relative error <= 1e-12 (fp64) / 1e-5 (fp32)
against the oracle's compensated long-double sum.
"""
import numpy as np
import pytest
import torch

import opal_inputs as oi
import paper_2510_00932_amd as opal

pytestmark = pytest.mark.gpu

DTYPES = [np.float64, np.float32]

# around one vector, one wavefront, one workgroup, one tile, and the point where the
# grid stops growing and workgroups start looping over several tiles
SMALL_SIZES = [0, 1, 2, 3, 4, 5, 7, 8, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257,
               511, 512, 513, 1023, 1024, 1025, 2047, 2048, 2049, 4095, 4096, 4097, 8191, 8192, 8193]
MID_SIZES = [65535, 65536, 65537, (1 << 20) - 1, (1 << 20) + 1, 1572869]
# ... and both sides of the array size (96 MiB) at which the library switches from cache-friendly to streaming accesses
LARGE_SIZES = [(1 << 22) - 1, (1 << 22) + 1, (1 << 23) + 2049, 3 * (1 << 22) - 1, 3 * (1 << 22) + 1,
               (1 << 24) + 12345, 3 * (1 << 23) - 1, 3 * (1 << 23) + 7]
OFFSETS = [(0, 0, 0), (1, 1, 1), (1, 0, 0), (0, 1, 0), (0, 0, 1), (3, 2, 1), (1, 2, 3), (5, 5, 5)]


@pytest.fixture(scope="module")
def gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    opal.load()
    return torch.device("cuda:0")


@pytest.fixture(scope="module")
def parity(gpu):
    import parity as _parity
    return _parity


@pytest.fixture(scope="module")
def harness(gpu):
    import gpu_harness
    return gpu_harness


# ------------------------------------------------------------------ the pins, on the GPU

@pytest.mark.parametrize("dtype", DTYPES)
def test_pins_hold_on_the_gpu(harness, dtype):
    import pins
    tol = 1e-12 if dtype == np.float64 else 1e-5
    for offsets in [(0, 0, 0), (1, 1, 1), (1, 2, 3)]:
        impl = harness.GpuImpl(offsets)
        for n in (0, 1, 5, 1000, 70001):
            pins.pin_constant_fill(impl, dtype, n)
            pins.pin_ramp(impl, dtype, n)
        pins.pin_exact_rational_elementwise(impl, dtype, n=700)
        pins.pin_fma_discriminator(impl, dtype, n=1)
        pins.pin_fma_discriminator(impl, dtype, n=5000)
        pins.pin_exact_dyadic_chain(impl, dtype, n=3000, dot_rel_tol=tol)
        pins.pin_dot_closed_forms(impl, dtype, [0, 1, 2, 3, 65, 1000, 4097, 100003])
        pins.pin_dot_exact_rational(impl, dtype, 3000, rel_tol=tol)
        pins.pin_dot_exact_rational(impl, dtype, 3000, rel_tol=tol, lo=0.5, hi=1.5)


@pytest.mark.parametrize("dtype", DTYPES)
def test_closed_forms_at_large_sizes(harness, dtype):
    """Facts that hold at any n, at sizes where every workgroup loops over several tiles."""
    import pins
    impl = harness.GpuImpl((0, 0, 0))
    n = (1 << 25) + 4099
    pins.pin_constant_fill(impl, dtype, n)
    pins.pin_ramp(impl, dtype, n)
    pins.pin_fma_discriminator(impl, dtype, n=n)
    pins.pin_dot_closed_forms(impl, dtype, [n])
    impl = harness.GpuImpl((1, 1, 1))
    pins.pin_ramp(impl, dtype, n)
    pins.pin_dot_closed_forms(impl, dtype, [n])


# ------------------------------------------------------------------ vs the oracle

@pytest.mark.parametrize("dtype", DTYPES)
def test_size_and_alignment_sweep(parity, dtype):
    w = oi.workload(4)  # sign-mixed values, s = -0.75
    full = [oi.uniform_array(w.seed, k, max(SMALL_SIZES + MID_SIZES), dtype, w.lo, w.hi) for k in range(3)]
    for n in SMALL_SIZES + MID_SIZES:
        for offsets in OFFSETS if n <= 8193 else OFFSETS[:4]:
            parity.run_chain([x[:n].copy() for x in full], w.s, offsets)
    w = oi.workload(0)  # positive values, s = 0.4
    full = [oi.uniform_array(w.seed, k, 8193, dtype, w.lo, w.hi) for k in range(3)]
    for n in SMALL_SIZES:
        parity.run_chain([x[:n].copy() for x in full], w.s, (0, 0, 0))
        parity.run_fresh([x[:n].copy() for x in full], w.s, (1, 0, 3))


@pytest.mark.parametrize("dtype", DTYPES)
def test_large_ragged_sizes(parity, dtype):
    w = oi.workload(4)
    full = [oi.uniform_array(w.seed, k, max(LARGE_SIZES), dtype, w.lo, w.hi) for k in range(3)]
    for n, offsets in zip(LARGE_SIZES, [(0, 0, 0), (1, 1, 1), (1, 0, 2), (0, 0, 0), (1, 1, 1), (0, 0, 0), (3, 3, 3),
                                        (2, 0, 1)]):
        parity.run_chain([x[:n].copy() for x in full], w.s, offsets)
        parity.run_fresh([x[:n].copy() for x in full], w.s, offsets)


def test_workload_0_chained_and_fresh(parity):
    w = oi.workload(0)
    arrays = oi.make_arrays(w)
    rel, kappa = parity.run_chain(arrays, w.s)
    assert kappa < 1.0 + 1e-9          # every term of the chained dot has one sign
    parity.run_fresh(arrays, w.s)


def test_idempotent_under_repeated_launches(parity):
    w = oi.workload(0)
    parity.run_chain(oi.make_arrays(w, n=(1 << 18) + 77), w.s, (1, 1, 1), iters=20)


def test_on_a_side_stream(parity):
    s = torch.cuda.Stream()
    w = oi.workload(0)
    arrays = oi.make_arrays(w, n=(1 << 18) + 3)
    parity.run_chain(arrays, w.s, (0, 0, 0), stream=s)
    parity.run_fresh(arrays, w.s, (1, 1, 1), stream=s)


@pytest.mark.parametrize("index", [1, 2, 3, 4])
def test_full_size_workloads(parity, index):
    """The four large workloads at their full sizes, every output element compared."""
    w = oi.workload(index)
    arrays = oi.make_arrays(w, threads=16)
    off = (w.offset_elems,) * 3
    rel_c, kappa_c = parity.run_chain(arrays, w.s, off, check_all_arrays_each_step=False)
    rel_f, kappa_f = parity.run_fresh(arrays, w.s, off)
    print("\n%s: chained dot rel err %.2e (kappa %.2e); fresh dot rel err %.2e (kappa %.2e)"
          % (w.name, rel_c, kappa_c, rel_f, kappa_f))
    if index == 4:
        assert kappa_f > 100.0          # the fresh dot of this workload really is sign-mixed


# ------------------------------------------------------------------ boundary behaviour on the device

def test_zero_length_dot_stores_zero(harness):
    res = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda:0")
    ws = torch.zeros(16, dtype=torch.float64, device="cuda:0")
    for dt in (opal.OPAL_F64, opal.OPAL_F32):
        res.fill_(float("nan"))
        opal.opal_dot(0, 0, 0, dt, ws.data_ptr(), 128, res.data_ptr(), None)
        torch.cuda.synchronize()
        assert res.item() == 0.0


def test_errors_enqueue_nothing(harness):
    n = 4096
    a = harness.GuardedArray(n, np.float64).upload(np.ones(n))
    c = harness.GuardedArray(n, np.float64).upload(np.zeros(n))
    with pytest.raises(opal.OpalError) as e:
        opal.opal_copy(a.ptr + 4, c.ptr, n, opal.OPAL_F64, None)
    assert e.value.status == 3
    with pytest.raises(opal.OpalError) as e:
        opal.opal_copy(a.ptr, c.ptr, n, 3, None)
    assert e.value.status == 2
    res = torch.full((1,), 7.0, dtype=torch.float64, device="cuda:0")
    ws = torch.zeros(8, dtype=torch.float64, device="cuda:0")
    with pytest.raises(opal.OpalError) as e:
        opal.opal_dot(a.ptr, c.ptr, 1 << 20, opal.OPAL_F64, ws.data_ptr(), 0, res.data_ptr(), None)
    assert e.value.status == 4
    torch.cuda.synchronize()
    assert (c.download() == 0).all() and res.item() == 7.0


def test_tensor_arguments(harness):
    n = 10007
    w = oi.workload(0)
    ha, hb, hc = oi.make_arrays(w, n=n)
    a, b, c = (torch.from_numpy(x).cuda() for x in (ha, hb, hc))
    opal.opal_triad(a, b, c, w.s, n)
    torch.cuda.synchronize()
    import oracle
    oracle.triad(ha, hb, hc, w.s)
    assert np.array_equal(a.cpu().numpy().view(np.uint64), ha.view(np.uint64))


def test_against_torch_as_a_sanity_check(harness):
    n = (1 << 20) + 5
    w = oi.workload(4)
    ha, hb, hc = oi.make_arrays(w, n=n)
    a, b, c = (torch.from_numpy(x).cuda() for x in (ha, hb, hc))
    out = torch.empty_like(a)
    opal.opal_add(a, b, out, n)
    assert torch.equal(out, a + b)
    opal.opal_scale(out, c, w.s, n)
    assert torch.equal(out, c * w.s)
    r = harness.dot_device(a.data_ptr(), b.data_ptr(), n, opal.OPAL_F64)
    assert abs(r - torch.dot(a, b).item()) <= 1e-9 * n


# ------------------------------------------------------------------ captured into a HIP graph

def graph_replay_check(parity, harness, n, dtype, offsets=(0, 1, 0), replays=5):
    """One pass copy -> scale -> add -> triad -> dot, eager, then captured into a HIP graph and replayed.
    Every replay (with the program's own eager launches and synchronisations in between) must leave
    exactly what that many oracle passes leave."""
    import oracle
    w = oi.workload(0)
    ha, hb, hc = (oi.uniform_array(w.seed, k, n, dtype, w.lo, w.hi, threads=16) for k in range(3))
    a, b, c = (harness.GuardedArray(n, dtype, off).upload(x) for x, off in zip((ha, hb, hc), offsets))
    dt = harness.opal_dtype(dtype)
    tol = 1e-12 if np.dtype(dtype) == np.float64 else 1e-5
    ws_bytes = opal.opal_dot_workspace_bytes(n, dt)
    ws = torch.zeros(ws_bytes // 8, dtype=torch.float64, device="cuda:0")
    res = torch.zeros(1, dtype=torch.float64, device="cuda:0")
    # eager scratch work that runs between the replays
    ea = harness.GuardedArray(4099, np.float64).upload(np.full(4099, 2.0))
    eb = harness.GuardedArray(4099, np.float64).upload(np.full(4099, 3.0))
    ec = harness.GuardedArray(4099, np.float64).upload(np.zeros(4099))

    def one_pass(stream):
        opal.opal_copy(a.ptr, c.ptr, n, dt, stream)
        opal.opal_scale(b.ptr, c.ptr, w.s, n, dt, stream)
        opal.opal_add(a.ptr, b.ptr, c.ptr, n, dt, stream)
        opal.opal_triad(a.ptr, b.ptr, c.ptr, w.s, n, dt, stream)
        opal.opal_dot(a.ptr, b.ptr, n, dt, ws.data_ptr(), ws_bytes, res.data_ptr(), stream)

    def oracle_pass():
        oracle.copy(ha, hc)
        oracle.scale(hb, hc, w.s)
        oracle.add(ha, hb, hc)
        oracle.triad(ha, hb, hc, w.s)
        return oracle.dot(ha, hb)

    def check(what, want_dot):
        torch.cuda.synchronize()
        for name, d, h in (("a", a, ha), ("b", b, hb), ("c", c, hc)):
            parity.assert_same_bits(d, h, "%s, array %s (n=%d %s)" % (what, name, n, np.dtype(dtype).name))
            assert d.guards_intact()
        got = float(res.item())
        assert abs(got - want_dot) <= tol * abs(want_dot), (what, got, want_dot)

    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    one_pass(side)                                    # eager pass (also warms the library's device query)
    side.synchronize()
    check("eager pass", oracle_pass())

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        one_pass(torch.cuda.current_stream())
    torch.cuda.synchronize()
    check("after capture (capturing must not execute)", oracle.dot(ha, hb))

    for k in range(replays):
        graph.replay()
        check("replay %d" % k, oracle_pass())
        opal.opal_add(ea.ptr, eb.ptr, ec.ptr, 4099, opal.OPAL_F64, None)      # eager work between replays
        torch.cuda.synchronize()
        assert (ec.download() == 5.0).all()
        res.fill_(float("nan"))
        torch.cuda.synchronize()


@pytest.mark.parametrize("n,dtype", [(2000896 + 3, np.float64), (4000768, np.float64), (6000640, np.float64),
                                     (2000896, np.float32), (6000640 + 1, np.float32)])
def test_graph_replay_matches_oracle(parity, harness, n, dtype):
    """The library neither allocates nor synchronises, so it can be captured into a HIP graph: the array
    sizes of the paper's Table 1 (one with a ragged tail), both element types."""
    graph_replay_check(parity, harness, n, dtype)


# ------------------------------------------------------------------ special values

@pytest.mark.parametrize("dtype", DTYPES)
def test_special_values(harness, dtype):
    """Signed zeros, subnormals, infinities, overflow and NaNs go through scale / add / triad exactly as
    on the CPU.  Results that are numbers must match bit for bit (so subnormals are not flushed and
    -0.0 stays -0.0); where the CPU result is a NaN the GPU result must be a NaN too (which NaN is
    produced by inf - inf or 0 * inf differs between the two instruction sets and is not compared)."""
    import oracle
    info = np.finfo(dtype)
    tiny, big = info.tiny, info.max
    sub = dtype(tiny) / dtype(8)                      # a subnormal
    specials = np.array([0.0, -0.0, sub, -sub, tiny, -tiny, 1.0, -1.0, big, -big, np.inf, -np.inf, np.nan,
                         1.5, 3.0 * float(sub), 0.75], dtype=dtype)
    # all ordered pairs (x, y) and, for the third operand, a rotation of the same list
    x = np.repeat(specials, specials.size)
    y = np.tile(specials, specials.size)
    z = np.roll(y, 5)
    pad = (-x.size) % 1024 + 1024 + 3                 # a few whole tiles and a ragged tail
    x, y, z = (np.concatenate([v, np.full(pad, 0.25, dtype)]) for v in (x, y, z))
    bits = np.uint64 if dtype == np.float64 else np.uint32

    def compare(got, want, what):
        nan_w, nan_g = np.isnan(want), np.isnan(got)
        assert np.array_equal(nan_w, nan_g), "%s: NaN positions differ" % what
        ok = nan_w | (got.view(bits) == want.view(bits))
        bad = np.nonzero(~ok)[0]
        assert bad.size == 0, "%s: %d differ, first i=%d gpu %r cpu %r" % (what, bad.size, bad[0], got[bad[0]], want[bad[0]])

    impl = harness.GpuImpl((0, 1, 0))
    for s in (0.4, -0.75, 0.0, float(big), 2.0):
        with np.errstate(all="ignore"):
            hb, gb = np.zeros_like(x), np.zeros_like(x)
            oracle.scale(hb, x.copy(), s)
            impl.scale(gb, x.copy(), s)
            compare(gb, hb, "scale by %r" % s)
            hc, gc = np.zeros_like(x), np.zeros_like(x)
            oracle.add(x.copy(), y.copy(), hc)
            impl.add(x.copy(), y.copy(), gc)
            compare(gc, hc, "add")
            ha, ga = np.zeros_like(x), np.zeros_like(x)
            oracle.triad(ha, y.copy(), z.copy(), s)
            impl.triad(ga, y.copy(), z.copy(), s)
            compare(ga, ha, "triad with s = %r" % s)
    # copy moves every bit pattern, NaN payloads included
    weird = np.arange(x.size, dtype=bits) * bits(0x9E3779B97F4A7C15 if dtype == np.float64 else 0x9E3779B9)
    src = weird.view(dtype)
    dst = np.zeros_like(src)
    impl.copy(src.copy(), dst)
    assert np.array_equal(dst.view(bits), weird)


def test_random_lengths_offsets_and_scalars(parity):
    """Seeded random cases: length, per-array misalignment, element type, value range and scalar."""
    rng = np.random.RandomState(20251)
    for case in range(80):
        dtype = DTYPES[rng.randint(2)]
        n = int(rng.randint(0, 1 << int(rng.randint(4, 19))))
        offsets = tuple(int(v) for v in rng.randint(0, 9, size=3))
        lo, hi = ((0.5, 1.5), (-1.0, 1.0), (-1e3, 1e3))[rng.randint(3)]
        s = float(rng.choice([0.4, -0.75, 1.0, -1.0, 3.0, 1e-3, float(rng.uniform(-2, 2))]))
        arrays = [oi.uniform_array(1000 + case, k, n, dtype, lo, hi) for k in range(3)]
        try:
            parity.run_chain(arrays, s, offsets)
        except AssertionError as e:
            raise AssertionError("case %d (dtype=%s n=%d offsets=%s range=(%g,%g) s=%r): %s"
                                 % (case, np.dtype(dtype).name, n, offsets, lo, hi, s, e))


def test_array_larger_than_4_gib(parity):
    """2^29 + 4099 fp64 elements per array: byte offsets no longer fit 32 bits."""
    w = oi.workload(4)
    n = (1 << 29) + 4099
    arrays = [oi.uniform_array(w.seed, k, n, np.float64, w.lo, w.hi, threads=16) for k in range(3)]
    parity.run_chain(arrays, w.s, (1, 1, 1), check_all_arrays_each_step=False)
