"""Pins: facts about Copy / Mul(scale) / Add / Triad / Dot (Table 1) that hold by
mathematics alone, written as checks that take an implementation `impl`.

`impl` is any object with
    copy(a, c)   scale(b, c, s)   add(a, b, c)   triad(a, b, c, s)   dot(a, b) -> float
working in place on 1-D numpy arrays (float64 or float32).  The CPU oracle is
checked against these pins on the CPU; the GPU library, wrapped so that it
accepts numpy arrays, is checked against the same pins on the GPU, at sizes of
the caller's choosing (every fact here holds at any n).

Expected values come from closed forms, from numpy scalar arithmetic (IEEE
operations, never fused) or from exact rational arithmetic; none come from
either implementation.
"""
import os
from fractions import Fraction

import numpy as np

import opal_inputs as oi

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


class PinFailure(AssertionError):
    pass


def _bits(x):
    return x.view(np.uint64 if x.dtype == np.float64 else np.uint32)


def _require_same_bits(got, want, what):
    if got.shape != want.shape or got.dtype != want.dtype:
        raise PinFailure("%s: shape/dtype mismatch" % what)
    bad = np.nonzero(_bits(got) != _bits(want))[0]
    if bad.size:
        i = int(bad[0])
        raise PinFailure("%s: %d of %d elements differ, first at i=%d: got %r want %r"
                         % (what, bad.size, got.size, i, got[i], want[i]))


def _rn(q, dtype):
    """Exact rational -> correctly rounded value of dtype (as a numpy scalar)."""
    d = q.numerator / q.denominator  # correctly rounded to binary64
    if np.dtype(dtype) == np.float64:
        return np.float64(d)
    # Callers only pass rationals that are exactly representable in binary64
    # (products / sums of two binary32 values of similar magnitude), so this
    # second rounding is the only one.
    if Fraction(d) != q:
        raise ValueError("rational not exact in binary64; double rounding possible")
    return np.float32(d)


def _s_typed(s, dtype):
    return np.dtype(dtype).type(s)


# ------------------------------------------------------------------ elementwise

def pin_constant_fill(impl, dtype, n, a0=0.7, b0=1.3, c0=0.9, s=0.4):
    """Constant arrays: every output element equals a scalar closed form."""
    t = np.dtype(dtype).type
    a, b, c = (oi.constant_array(n, dtype, v) for v in (a0, b0, c0))
    a0, b0, c0, st = t(a0), t(b0), t(c0), t(s)

    impl.copy(a, c)
    _require_same_bits(c, np.full(n, a0, dtype), "copy of constants")
    _require_same_bits(a, np.full(n, a0, dtype), "copy left its input alone")

    c[:] = c0
    impl.scale(b, c, s)
    _require_same_bits(b, np.full(n, st * c0, dtype), "scale of constants")
    _require_same_bits(c, np.full(n, c0, dtype), "scale left its input alone")

    b[:] = b0
    impl.add(a, b, c)
    _require_same_bits(c, np.full(n, a0 + b0, dtype), "add of constants")

    c[:] = c0
    impl.triad(a, b, c, s)
    prod = st * c0              # numpy scalar ops: one IEEE rounding each
    _require_same_bits(a, np.full(n, b0 + prod, dtype), "triad of constants")
    _require_same_bits(b, np.full(n, b0, dtype), "triad left b alone")
    _require_same_bits(c, np.full(n, c0, dtype), "triad left c alone")


def pin_ramp(impl, dtype, n):
    """Index-valued arrays: catches shifted, permuted, duplicated or skipped elements."""
    mod = 0 if np.dtype(dtype) == np.float64 else (1 << 22)
    i = oi.ramp_array(n, dtype, mod)
    three = np.full(n, 3, dtype)

    c = np.full(n, -1, dtype)
    impl.copy(i.copy(), c)
    _require_same_bits(c, i, "copy of ramp")

    b = np.full(n, -1, dtype)
    impl.scale(b, i.copy(), 2.0)
    _require_same_bits(b, i * 2, "scale of ramp by 2")

    c = np.full(n, -1, dtype)
    impl.add(i.copy(), three.copy(), c)
    _require_same_bits(c, i + 3, "add ramp + 3")
    # a - role and b - role both read: i + 2i
    impl.add(i.copy(), (i * 2), c)
    _require_same_bits(c, i * 3, "add ramp + 2*ramp")

    a = np.full(n, -1, dtype)
    impl.triad(a, three.copy(), i.copy(), 4.0)     # a = 3 + 4*i: b is the addend, c the scaled one
    _require_same_bits(a, i * 4 + 3, "triad 3 + 4*ramp")
    impl.triad(a, i.copy(), three.copy(), 4.0)     # a = i + 12
    _require_same_bits(a, i + 12, "triad ramp + 4*3")


def pin_exact_rational_elementwise(impl, dtype, n=1500, s=0.4, seed=3, lo=0.5, hi=1.5):
    """Random values: each output equals the exact rational result rounded once per operation."""
    t = np.dtype(dtype).type
    a, b, c = (oi.uniform_array(seed, k, n, dtype, lo, hi) for k in range(3))
    fs = Fraction(float(t(s)))
    fa = [Fraction(float(x)) for x in a]
    fb = [Fraction(float(x)) for x in b]
    fc = [Fraction(float(x)) for x in c]

    out = np.empty(n, dtype)
    impl.scale(out, c.copy(), s)
    want = np.array([_rn(fs * x, dtype) for x in fc], dtype)
    _require_same_bits(out, want, "scale vs exact rational")

    impl.add(a.copy(), b.copy(), out)
    want = np.array([_rn(x + y, dtype) for x, y in zip(fa, fb)], dtype)
    _require_same_bits(out, want, "add vs exact rational")

    impl.triad(out, b.copy(), c.copy(), s)
    prod = [Fraction(float(_rn(fs * x, dtype))) for x in fc]
    want = np.array([_rn(y + p, dtype) for y, p in zip(fb, prod)], dtype)
    _require_same_bits(out, want, "triad vs exact rational, two roundings")
    fused = np.array([np.float64((y + fs * x).numerator / (y + fs * x).denominator) for x, y in zip(fc, fb)])
    if np.dtype(dtype) == np.float64 and not (fused != want).any():
        raise PinFailure("test vector too weak: fused and unfused triad agree everywhere")


def read_fma_discriminator(dtype):
    key = "f64" if np.dtype(dtype) == np.float64 else "f32"
    with open(os.path.join(GOLDEN, "fma_discriminator.txt")) as f:
        for line in f:
            if line.startswith(key + " "):
                return [float.fromhex(x) for x in line.split()[1:]]
    raise KeyError(key)


def pin_fma_discriminator(impl, dtype, n=1):
    """A stored (b, s, c) on which fl(b + fl(s*c)) != fl(b + s*c): triad must give the former."""
    b0, s, c0, two_step, fused = read_fma_discriminator(dtype)
    assert two_step != fused
    a = np.zeros(n, dtype)
    impl.triad(a, np.full(n, b0, dtype), np.full(n, c0, dtype), s)
    _require_same_bits(a, np.full(n, two_step, dtype), "triad on the fused/unfused discriminator")


def pin_exact_dyadic_chain(impl, dtype, n=2000, seed=5, dot_rel_tol=0.0):
    """s = -0.75 and inputs with few significant bits: every elementwise step of
    the chain copy -> scale -> add -> triad is exact, so the arrays equal exact
    rational arithmetic with no rounding anywhere; the closing dot is compared
    with the exact rational sum (dot_rel_tol = 0: it must be that sum correctly
    rounded to double)."""
    bits = 20 if np.dtype(dtype) == np.float64 else 8
    s = -0.75
    a, b, c = (oi.short_mantissa_array(seed, k, n, dtype, bits=bits) for k in range(3))
    fa = [Fraction(float(x)) for x in a]
    fs = Fraction(s)

    impl.copy(a, c)                     # c = a
    fc = list(fa)
    impl.scale(b, c, s)                 # b = s*c
    fb = [fs * x for x in fc]
    impl.add(a, b, c)                   # c = a + b
    fc = [x + y for x, y in zip(fa, fb)]
    impl.triad(a, b, c, s)              # a = b + s*c
    fa = [y + fs * x for x, y in zip(fc, fb)]
    for name, arr, fr in (("a", a, fa), ("b", b, fb), ("c", c, fc)):
        want = np.array([float(x) for x in fr], dtype)
        if any(Fraction(float(w)) != x for w, x in zip(want, fr)):
            raise PinFailure("chain is not exact in %s: test construction error" % dtype)
        _require_same_bits(arr, want, "exact chain, array " + name)
    r = impl.dot(a, b)
    exact = sum(x * y for x, y in zip(fa, fb))
    want = exact.numerator / exact.denominator      # correctly rounded
    if dot_rel_tol == 0.0:
        if r != want:
            raise PinFailure("exact chain dot: got %r want %r" % (r, want))
    elif abs(Fraction(r) - exact) > Fraction(dot_rel_tol) * abs(exact):
        raise PinFailure("exact chain dot: got %r want %r (tol %g)" % (r, want, dot_rel_tol))


# -------------------------------------------------------------------------- dot

def pin_dot_closed_forms(impl, dtype, ns):
    """Integer-valued data: every partial sum in every summation order is an
    integer below 2**24 (fp32) / 2**53 (fp64), so the result is exact and must
    match the closed form bit for bit."""
    is64 = np.dtype(dtype) == np.float64
    for n in ns:
        # constants: n * a0 * b0 (kept below 2**24 for fp32 so fp32 partial sums stay exact)
        a0, b0 = (1.5, 2.0) if (is64 or 3 * n < (1 << 24)) else (2.0 ** -6, 2.0 ** -3)
        r = impl.dot(oi.constant_array(n, dtype, a0), oi.constant_array(n, dtype, b0))
        if r != n * a0 * b0:
            raise PinFailure("dot of constants, n=%d: got %r want %r" % (n, r, n * a0 * b0))
        # ramp (i mod m) . 1  and  (i mod m) . (i mod 7)
        m = 1024 if is64 else 8
        if not is64 and n * m * 7 >= (1 << 24):
            continue
        i = np.arange(n, dtype=np.int64)
        x, y = i % m, i % 7
        r1 = impl.dot(x.astype(dtype), np.ones(n, dtype))
        if r1 != float(int(x.sum())):
            raise PinFailure("dot ramp.1, n=%d: got %r want %r" % (n, r1, int(x.sum())))
        r2 = impl.dot(x.astype(dtype), y.astype(dtype))
        want = int((x * y).sum())
        if r2 != float(want):
            raise PinFailure("dot ramp.ramp7, n=%d: got %r want %r" % (n, r2, want))


def exact_dot(a, b):
    """sum a[i]*b[i] as an exact rational."""
    total = Fraction(0)
    for x, y in zip(a.tolist(), b.tolist()):
        total += Fraction(x) * Fraction(y)
    return total


def pin_dot_exact_rational(impl, dtype, n, rel_tol, seed=9, lo=-1.0, hi=1.0):
    """Random (sign-mixed by default) data against the exact rational sum."""
    a = oi.uniform_array(seed, 0, n, dtype, lo, hi)
    b = oi.uniform_array(seed, 1, n, dtype, lo, hi)
    exact = exact_dot(a, b)
    r = impl.dot(a, b)
    err = abs(Fraction(r) - exact)
    if exact == 0:
        raise PinFailure("degenerate test data: exact dot is zero")
    if err > Fraction(rel_tol) * abs(exact):
        raise PinFailure("dot vs exact rational, n=%d: got %r exact %r rel err %.3e > %.1e"
                         % (n, r, float(exact), float(err / abs(exact)), rel_tol))
    return float(err / abs(exact))
