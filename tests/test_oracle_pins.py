"""The CPU oracle against facts fixed by mathematics (no GPU needed).

The paper prints no worked example, value or bandwidth for Copy / Mul / Add /
Triad / Dot (Table 1 only names them), so the oracle is pinned by closed
forms, exact rational arithmetic and library cross-checks instead.  The last
section shows that the pins have teeth: wrong implementations (written here,
in numpy) each fail at least one of them.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

import opal_inputs as oi
import pins

DTYPES = [np.float64, np.float32]
SIZES = [0, 1, 2, 3, 5, 64, 1000, 4097]


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("n", SIZES)
def test_constant_fill(oracle, dtype, n):
    pins.pin_constant_fill(oracle, dtype, n)
    pins.pin_constant_fill(oracle, dtype, n, a0=-0.3, b0=0.1, c0=1.7, s=-0.75)


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("n", SIZES)
def test_ramp(oracle, dtype, n):
    pins.pin_ramp(oracle, dtype, n)


@pytest.mark.parametrize("dtype", DTYPES)
def test_exact_rational_elementwise(oracle, dtype):
    pins.pin_exact_rational_elementwise(oracle, dtype, s=0.4, lo=0.5, hi=1.5)
    pins.pin_exact_rational_elementwise(oracle, dtype, s=-0.75, lo=-1.0, hi=1.0, seed=4)


@pytest.mark.parametrize("dtype", DTYPES)
def test_fma_discriminator(oracle, dtype):
    b0, s, c0, two_step, fused = pins.read_fma_discriminator(dtype)
    # the stored expectations really are the two roundings / the one rounding
    t = np.dtype(dtype).type
    prod = Fraction(float(t(s))) * Fraction(c0)
    assert Fraction(float(t(float(prod)))) != prod          # the product needs rounding
    assert float(t(b0) + t(s) * t(c0)) == two_step          # numpy scalars never fuse
    pins.pin_fma_discriminator(oracle, dtype, n=1)
    pins.pin_fma_discriminator(oracle, dtype, n=67)


@pytest.mark.parametrize("dtype", DTYPES)
def test_exact_dyadic_chain(oracle, dtype):
    pins.pin_exact_dyadic_chain(oracle, dtype)


@pytest.mark.parametrize("dtype", DTYPES)
def test_dot_closed_forms(oracle, dtype):
    pins.pin_dot_closed_forms(oracle, dtype, [0, 1, 2, 3, 63, 64, 65, 1000, 4097, 100003])


@pytest.mark.parametrize("dtype", DTYPES)
def test_dot_exact_rational(oracle, dtype):
    # within one unit in the last place of double of the exact sum, sign-mixed and same-sign
    for n in (1, 2, 17, 3000):
        pins.pin_dot_exact_rational(oracle, dtype, n, rel_tol=2.0 ** -52)
        pins.pin_dot_exact_rational(oracle, dtype, n, rel_tol=2.0 ** -52, lo=0.5, hi=1.5, seed=10)


@pytest.mark.parametrize("dtype", DTYPES)
def test_dot_brute_force_long_double_sum(oracle, dtype):
    # the plain running long-double sum on small n agrees with the compensated one
    for n in (1, 10, 1000, 20000):
        a = oi.uniform_array(21, 0, n, dtype, -1.0, 1.0)
        b = oi.uniform_array(21, 1, n, dtype, -1.0, 1.0)
        r, p = oracle.dot(a, b), oracle.dot_plain(a, b)
        scale = oracle.dot_abs(a, b)
        assert abs(r - p) <= 4 * 2.0 ** -53 * scale
        assert oracle.dot(a, b) == oracle.dot(b, a)
        assert float(oracle.dot_longdouble(a, b)) == r


def test_dot_compensation_survives_cancellation(oracle):
    # 1e30 + 1 - 1e30: the running long-double sum loses the 1, the compensated sum keeps it.
    a = np.array([1e30, 1.0, -1e30, 0.5], dtype=np.float64)
    b = np.ones(4, dtype=np.float64)
    assert oracle.dot(a, b) == 1.5
    assert oracle.dot_plain(a, b) == 0.5
    a = np.array([2.0 ** 70, -3.0, -2.0 ** 70, 1.0, 2.0 ** -40], dtype=np.float64)
    b = np.array([1.0, 1.0, 1.0, 2.0, 1.0], dtype=np.float64)
    assert oracle.dot(a, b) == -1.0 + 2.0 ** -40


@pytest.mark.parametrize("dtype", DTYPES)
def test_dot_against_libraries(oracle, dtype):
    n = 1 << 20
    w = oi.workload(0)
    a = oi.uniform_array(w.seed, 0, n, dtype, w.lo, w.hi)
    b = oi.uniform_array(w.seed, 1, n, dtype, w.lo, w.hi)
    r = oracle.dot(a, b)
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    assert abs(r - float(np.dot(a64, b64))) <= 1e-13 * abs(r)
    assert abs(r - math.fsum((a64 * b64).tolist())) <= 1e-15 * abs(r) * 2
    assert abs(oracle.dot_abs(a, b) - r) <= 1e-15 * r      # all terms positive
    # sign-mixed
    w = oi.workload(4)
    a = oi.uniform_array(w.seed, 0, n, dtype, w.lo, w.hi).astype(np.float64)
    b = oi.uniform_array(w.seed, 1, n, dtype, w.lo, w.hi).astype(np.float64)
    r = oracle.dot(a, b)
    s_abs = oracle.dot_abs(a, b)
    assert abs(r - math.fsum((a * b).tolist())) <= 2.0 ** -52 * s_abs
    assert abs(s_abs - float(np.abs(a * b).sum())) <= 1e-12 * s_abs


def test_scalar_is_rounded_once_to_float(oracle):
    # s = 0.4 is not a float: the fp32 kernels use float(0.4), not the double.
    c = np.array([1.2345678], dtype=np.float32)
    b = np.zeros(1, dtype=np.float32)
    oracle.scale(b, c, 0.4)
    assert b[0] == np.float32(0.4) * c[0]
    seen_difference = False
    for v in oi.uniform_array(2, 0, 200, np.float32, 0.5, 1.5):
        c[0] = v
        oracle.scale(b, c, 0.4)
        assert b[0] == np.float32(0.4) * v
        seen_difference |= b[0] != np.float32(np.float64(0.4) * np.float64(v))
    assert seen_difference


def test_wrapper_rejects_bad_arrays(oracle):
    a = np.zeros(4)
    with pytest.raises(ValueError):
        oracle.copy(a, np.zeros(5))
    with pytest.raises(ValueError):
        oracle.copy(a, np.zeros(4, dtype=np.float32))
    with pytest.raises(ValueError):
        oracle.copy(a[::2], np.zeros(2))
    with pytest.raises(TypeError):
        oracle.copy(np.zeros(4, dtype=np.int32), np.zeros(4, dtype=np.int32))


# ----------------------------------------------------------------------------
# The pins have teeth: plausible mistakes, planted in numpy stand-ins, are caught.

class _Good:
    """A correct numpy stand-in (numpy ufuncs round once per operation)."""

    @staticmethod
    def copy(a, c):
        c[:] = a

    @staticmethod
    def scale(b, c, s):
        b[:] = c.dtype.type(s) * c

    @staticmethod
    def add(a, b, c):
        c[:] = a + b

    @staticmethod
    def triad(a, b, c, s):
        a[:] = b + c.dtype.type(s) * c

    @staticmethod
    def dot(a, b):
        return float(pins.exact_dot(a, b))


def _mutant(**overrides):
    return type("Mutant", (_Good,), {k: staticmethod(v) for k, v in overrides.items()})


def _fused_triad(a, b, c, s):
    st = Fraction(float(c.dtype.type(s)))
    for i in range(len(a)):
        q = Fraction(float(b[i])) + st * Fraction(float(c[i]))
        a[i] = q.numerator / q.denominator


def _triad_swapped(a, b, c, s):
    a[:] = c + c.dtype.type(s) * b


def _triad_minus(a, b, c, s):
    a[:] = b - c.dtype.type(s) * c


def _scale_double_scalar(b, c, s):
    b[:] = (np.float64(s) * c.astype(np.float64)).astype(c.dtype)


def _copy_shifted(a, c):
    c[1:] = a[:-1]
    if len(a):
        c[0] = a[0]


def _copy_skip_last(a, c):
    c[:-1] = a[:-1]


def _add_sub(a, b, c):
    c[:] = a - b


def _add_a_twice(a, b, c):
    c[:] = a + a


def _dot_skip_last(a, b):
    return float(pins.exact_dot(a[:-1], b[:-1]))


def _dot_double_count(a, b):
    return float(pins.exact_dot(a, b)) + (float(a[0]) * float(b[0]) if len(a) else 0.0)


def _dot_f32_accumulate(a, b):
    acc = np.float32(0)
    for x, y in zip(a.astype(np.float32), b.astype(np.float32)):
        acc = np.float32(acc + x * y)
    return float(acc)


def _dot_aa(a, b):
    return float(pins.exact_dot(a, a))


def _run_all_pins(impl, dtype):
    for n in (0, 1, 5, 1000):
        pins.pin_constant_fill(impl, dtype, n)
        pins.pin_ramp(impl, dtype, n)
    pins.pin_exact_rational_elementwise(impl, dtype, n=300)
    pins.pin_fma_discriminator(impl, dtype, n=3)
    pins.pin_exact_dyadic_chain(impl, dtype, n=300)
    pins.pin_dot_closed_forms(impl, dtype, [0, 1, 65, 1000])
    pins.pin_dot_exact_rational(impl, dtype, 700, rel_tol=2.0 ** -52)


@pytest.mark.parametrize("dtype", DTYPES)
def test_stand_in_passes_all_pins(dtype):
    _run_all_pins(_Good, dtype)


MUTANTS = {
    "triad fused": dict(triad=_fused_triad),
    "triad operands swapped": dict(triad=_triad_swapped),
    "triad sign": dict(triad=_triad_minus),
    "copy shifted by one": dict(copy=_copy_shifted),
    "copy misses the last element": dict(copy=_copy_skip_last),
    "add subtracts": dict(add=_add_sub),
    "add reads a twice": dict(add=_add_a_twice),
    "dot misses the last element": dict(dot=_dot_skip_last),
    "dot counts the first element twice": dict(dot=_dot_double_count),
    "dot of a with itself": dict(dot=_dot_aa),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
@pytest.mark.parametrize("dtype", DTYPES)
def test_planted_mistake_is_caught(name, dtype):
    with pytest.raises(pins.PinFailure):
        _run_all_pins(_mutant(**MUTANTS[name]), dtype)


def test_planted_precision_mistakes_are_caught():
    with pytest.raises(pins.PinFailure):
        _run_all_pins(_mutant(scale=_scale_double_scalar), np.float32)
    with pytest.raises(pins.PinFailure):
        _run_all_pins(_mutant(dot=_dot_f32_accumulate), np.float64)
