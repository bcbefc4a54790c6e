"""Seeded synthetic inputs for the streaming vector kernels.

This module only produces bytes: three dense 1-D arrays a, b, c and the
workload table (length, element type, value range, scalar, misalignment).  It
holds none of the kernels' arithmetic and is the one module both the CPU
oracle's tests and the GPU library's tests draw their inputs from, so that
both sides see identical bits.

Generator: SplitMix64 (Steele, Lea, Flood, "Fast splittable pseudorandom
number generators", OOPSLA 2014) used counter-style.  With gamma =
0x9E3779B97F4A7C15 and mix() the published 64-bit finaliser, the j-th output
(j = 0, 1, ...) of a SplitMix64 stream seeded with S is mix(S + (j+1)*gamma).
Array k (0 = a, 1 = b, 2 = c) of a workload with seed sigma uses the stream
whose seed is the k-th output of the stream seeded with sigma; element i of the
array is built from the i-th output z of that stream:

    fp64: u = (z >> 11) * 2**-53        fp32: u = float32((z >> 40) * 2**-24)
    x = lo + (hi - lo) * u              evaluated in the array's own type

so any element can be produced independently of all others, in any order, and
the arrays do not depend on n (a longer array extends a shorter one).
"""
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

GAMMA = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_MASK = (1 << 64) - 1

_CHUNK = 1 << 21  # elements generated per numpy pass (16 MiB of uint64)


def mix64(z: int) -> int:
    """SplitMix64 output function on a Python int (reference form, used for stream seeds)."""
    z &= _MASK
    z = ((z ^ (z >> 30)) * _M1) & _MASK
    z = ((z ^ (z >> 27)) * _M2) & _MASK
    return z ^ (z >> 31)


def splitmix64_output(seed: int, j: int) -> int:
    """j-th output (0-based) of the SplitMix64 stream seeded with `seed`."""
    return mix64(seed + (j + 1) * GAMMA)


def _mix64_np(z: np.ndarray) -> np.ndarray:
    """Vectorised mix64 on a uint64 array (in place; wraps modulo 2**64)."""
    z ^= z >> np.uint64(30)
    z *= np.uint64(_M1)
    z ^= z >> np.uint64(27)
    z *= np.uint64(_M2)
    z ^= z >> np.uint64(31)
    return z


def raw_u64(stream_seed: int, start: int, count: int) -> np.ndarray:
    """Outputs start .. start+count-1 of the stream, as uint64."""
    j = np.arange(start + 1, start + count + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        j *= np.uint64(GAMMA)
        j += np.uint64(stream_seed & _MASK)
        return _mix64_np(j)


def _fill(out: np.ndarray, stream_seed: int, start: int, lo: float, hi: float) -> None:
    z = raw_u64(stream_seed, start, out.shape[0])
    if out.dtype == np.float64:
        u = (z >> np.uint64(11)).astype(np.float64)
        u *= 2.0 ** -53
        u *= np.float64(hi - lo)
        u += np.float64(lo)
        out[:] = u
    elif out.dtype == np.float32:
        u = (z >> np.uint64(40)).astype(np.float32)  # < 2**24: exact
        u *= np.float32(2.0 ** -24)
        u *= np.float32(hi - lo)
        u += np.float32(lo)
        out[:] = u
    else:
        raise TypeError("float64 or float32 only")


def uniform_array(seed: int, k: int, n: int, dtype, lo: float, hi: float,
                  out: np.ndarray = None, threads: int = 8) -> np.ndarray:
    """Array k (0=a, 1=b, 2=c) of the workload seeded with `seed`: n iid uniform [lo, hi) values."""
    dtype = np.dtype(dtype)
    if out is None:
        out = np.empty(n, dtype=dtype)
    if out.shape != (n,) or out.dtype != dtype:
        raise ValueError("out must be a 1-D array of n elements of dtype")
    stream_seed = splitmix64_output(seed, k)
    starts = range(0, n, _CHUNK)
    if n <= _CHUNK or threads <= 1:
        for st in starts:
            _fill(out[st:st + _CHUNK], stream_seed, st, lo, hi)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(lambda st: _fill(out[st:st + _CHUNK], stream_seed, st, lo, hi), starts))
    return out


@dataclass(frozen=True)
class Workload:
    """One synthetic workload: three arrays of n elements and a scalar."""
    name: str
    n: int
    dtype: str            # "f64" or "f32"
    lo: float
    hi: float
    s: float
    seed: int = 42
    offset_elems: int = 0  # every array starts this many elements past a 256-byte-aligned base
    iters: int = 1         # timed launches per kernel

    @property
    def np_dtype(self):
        return np.dtype(np.float64 if self.dtype == "f64" else np.float32)

    @property
    def itemsize(self) -> int:
        return 8 if self.dtype == "f64" else 4


# The five workloads, in order: a small parity case, a cache-straddling case, the
# headline roofline case, its fp32 twin, and a prime-length, misaligned,
# sign-mixed case.
WORKLOADS = (
    Workload("n2p20_f64", 1 << 20, "f64", 0.5, 1.5, 0.4, iters=1),
    Workload("n2p25_f64", 1 << 25, "f64", 0.5, 1.5, 0.4, iters=100),
    Workload("n2p28_f64", 1 << 28, "f64", 0.5, 1.5, 0.4, iters=100),
    Workload("n2p28_f32", 1 << 28, "f32", 0.5, 1.5, 0.4, iters=100),
    Workload("n300000007_f64_off1", 300000007, "f64", -1.0, 1.0, -0.75, offset_elems=1, iters=100),
)


def workload(name_or_index) -> Workload:
    if isinstance(name_or_index, int):
        return WORKLOADS[name_or_index]
    for w in WORKLOADS:
        if w.name == name_or_index:
            return w
    raise KeyError(name_or_index)


def make_arrays(w: Workload, n: int = None, threads: int = 8):
    """Host arrays (a, b, c) of workload w; n overrides the length (a prefix of the full arrays)."""
    n = w.n if n is None else n
    return tuple(uniform_array(w.seed, k, n, w.np_dtype, w.lo, w.hi, threads=threads) for k in range(3))


# Alternative deterministic fills used by the parity pins -------------------------------------

def constant_array(n: int, dtype, value: float) -> np.ndarray:
    return np.full(n, value, dtype=np.dtype(dtype))


def ramp_array(n: int, dtype, modulus: int = 0) -> np.ndarray:
    """x[i] = i (or i mod modulus); exact while the values stay below 2**53 (fp64) / 2**24 (fp32)."""
    i = np.arange(n, dtype=np.uint64)
    if modulus:
        i %= np.uint64(modulus)
    return i.astype(np.dtype(dtype))


def short_mantissa_array(seed: int, k: int, n: int, dtype, bits: int = 20, signed: bool = True) -> np.ndarray:
    """Values m * 2**-bits with odd integer |m| < 2**bits (never zero, so no signed-zero
    cases): products and sums of a few of them are exact."""
    z = raw_u64(splitmix64_output(seed, k), 0, n)
    m = (z >> np.uint64(64 - bits)).astype(np.int64) | 1
    if signed:
        sign = ((z >> np.uint64(7)) & np.uint64(1)).astype(np.int64) * 2 - 1
        m = m * sign
    return (m.astype(np.float64) * 2.0 ** -bits).astype(np.dtype(dtype))
