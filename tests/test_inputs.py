"""The seeded input generator: pinned to the published SplitMix64 definition."""
import numpy as np

import opal_inputs as oi


def _splitmix64_sequential(seed, count):
    """SplitMix64 in its sequential, stateful form, on Python ints."""
    mask = (1 << 64) - 1
    state = seed & mask
    out = []
    for _ in range(count):
        state = (state + 0x9E3779B97F4A7C15) & mask
        z = state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
        out.append(z ^ (z >> 31))
    return out


def test_known_answer_vector():
    # Widely published first outputs of SplitMix64 seeded with 1234567.
    want = [6457827717110365317, 3203168211198807973, 9817491932198370423,
            4593380528125082431, 16408922859458223821]
    assert [oi.splitmix64_output(1234567, j) for j in range(5)] == want
    assert oi.raw_u64(1234567, 0, 5).tolist() == want


def test_counter_form_equals_sequential_form():
    for seed in (0, 42, (1 << 64) - 1, 0xDEADBEEFCAFEF00D):
        seq = _splitmix64_sequential(seed, 300)
        assert oi.raw_u64(seed, 0, 300).tolist() == seq
        assert oi.raw_u64(seed, 137, 50).tolist() == seq[137:187]


def test_arrays_are_prefix_stable_and_chunk_independent():
    big = oi.uniform_array(42, 1, (1 << 21) * 2 + 12345, np.float64, 0.5, 1.5)
    small = oi.uniform_array(42, 1, 1000, np.float64, 0.5, 1.5)
    assert np.array_equal(big[:1000], small)
    one_thread = oi.uniform_array(42, 1, big.shape[0], np.float64, 0.5, 1.5, threads=1)
    assert np.array_equal(big, one_thread)
    # element i rebuilt alone from the definition
    ss = oi.splitmix64_output(42, 1)
    for i in (0, 1, (1 << 21) - 1, 1 << 21, big.shape[0] - 1):
        z = oi.mix64(ss + (i + 1) * oi.GAMMA)
        assert big[i] == 0.5 + (z >> 11) * 2.0 ** -53


def test_ranges_and_streams_differ():
    for w in oi.WORKLOADS:
        a, b, c = oi.make_arrays(w, n=4096)
        for x in (a, b, c):
            assert x.dtype == w.np_dtype
            assert x.min() >= w.lo and x.max() <= w.hi
        assert not np.array_equal(a, b) and not np.array_equal(b, c)
    w = oi.workload(4)
    a, _, _ = oi.make_arrays(w, n=4096)
    assert (a < 0).any() and (a > 0).any()
    assert abs(a.mean()) < 0.05


def test_f32_values_are_exact_24_bit_fractions():
    a = oi.uniform_array(42, 0, 4096, np.float32, 0.5, 1.5)
    ss = oi.splitmix64_output(42, 0)
    for i in (0, 7, 4095):
        z = oi.mix64(ss + (i + 1) * oi.GAMMA)
        assert a[i] == np.float32(0.5) + np.float32((z >> 40) * 2.0 ** -24)


def test_workload_table():
    ws = oi.WORKLOADS
    assert [w.n for w in ws] == [1 << 20, 1 << 25, 1 << 28, 1 << 28, 300000007]
    assert [w.dtype for w in ws] == ["f64", "f64", "f64", "f32", "f64"]
    assert [w.s for w in ws] == [0.4, 0.4, 0.4, 0.4, -0.75]
    assert ws[4].offset_elems == 1 and ws[4].lo == -1.0
