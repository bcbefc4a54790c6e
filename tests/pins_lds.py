"""Pins for the LDS streaming microkernel (tile-wise: rep rounds of "rotate by one 16-byte
vector and add c").  `impl` has lds_stream(inp, out, c, rep) on 1-D numpy arrays.  Expected
values come from index arithmetic and numpy scalar adds only."""
import numpy as np

from pins import PinFailure, _require_same_bits

TILE_VECTORS = 1024


def per_vec(dtype):
    return 16 // np.dtype(dtype).itemsize


def tile_elems(dtype):
    return TILE_VECTORS * per_vec(dtype)


def rotated(x, rep):
    """Each tile of x rotated down by rep vectors: out[vector j] = x[vector (j + rep) mod 1024]."""
    pv = per_vec(x.dtype)
    t = x.reshape(-1, TILE_VECTORS, pv)
    return np.roll(t, -(rep % TILE_VECTORS), axis=1).reshape(-1).copy()


def add_repeatedly(x, c, rep):
    c = x.dtype.type(c)
    y = x.copy()
    for _ in range(rep):
        y = y + c                       # one IEEE add per round, never fused or reassociated
    return y


def pin_lds_copy_and_pure_rotation(impl, dtype, tiles=3):
    n = tiles * tile_elems(dtype)
    x = (np.arange(n, dtype=np.int64) % (1 << 20)).astype(dtype)       # a ramp: every position distinct within reach
    out = np.full(n, -1, dtype)
    impl.lds_stream(x.copy(), out, 0.7, 0)
    _require_same_bits(out, x, "rep = 0 copies")
    for rep in (1, 2, 5, 1023, 1024, 1025, 2500):
        out = np.full(n, -1, dtype)
        impl.lds_stream(x.copy(), out, 0.0, rep)
        _require_same_bits(out, rotated(x, rep), "c = 0, rep = %d is a pure rotation inside each tile" % rep)
    out = np.full(n, -1, dtype)
    src = x.copy()
    impl.lds_stream(src, out, 0.0, 7)
    _require_same_bits(src, x, "input left alone")


def pin_lds_constant_fill(impl, dtype, tiles=2):
    n = tiles * tile_elems(dtype)
    for v0, c, rep in ((0.3, 0.1, 1), (0.3, 0.1, 37), (1.7, -0.4, 600)):
        x = np.full(n, v0, dtype)
        out = np.zeros(n, dtype)
        impl.lds_stream(x, out, c, rep)
        _require_same_bits(out, add_repeatedly(x, c, rep), "constant fill, c added %d times with a rounding each" % rep)


def pin_lds_exact_and_composition(impl, dtype, tiles=2):
    """c = 0.25 on small integers: every add is exact, so out = rotate(in) + rep/4, and two
    calls of r1 and r2 rounds equal one call of r1 + r2 rounds."""
    n = tiles * tile_elems(dtype)
    x = (np.arange(n, dtype=np.int64) * 7 % 1000).astype(dtype)
    for r1, r2 in ((3, 4), (600, 424), (1, 1023)):
        mid = np.zeros(n, dtype)
        impl.lds_stream(x.copy(), mid, 0.25, r1)
        _require_same_bits(mid, rotated(x, r1) + dtype(0.25 * r1), "exact: rotate(x, %d) + %d/4" % (r1, r1))
        two = np.zeros(n, dtype)
        impl.lds_stream(mid.copy(), two, 0.25, r2)
        one = np.zeros(n, dtype)
        impl.lds_stream(x.copy(), one, 0.25, r1 + r2)
        _require_same_bits(two, one, "f(%d) after f(%d) equals f(%d)" % (r2, r1, r1 + r2))


def pin_lds_random_values(impl, dtype, seed_array, c=0.1, rep=50):
    x = seed_array
    out = np.zeros_like(x)
    impl.lds_stream(x.copy(), out, c, rep)
    _require_same_bits(out, add_repeatedly(rotated(x, rep), c, rep), "random values: rotation and %d rounded adds" % rep)


def pin_lds_tiles_are_independent(impl, dtype):
    n = 3 * tile_elems(dtype)
    x = (np.arange(n, dtype=np.int64) % 5000).astype(dtype)
    base = np.zeros(n, dtype)
    impl.lds_stream(x.copy(), base, 0.5, 9)
    y = x.copy()
    y[:tile_elems(dtype)] += dtype(1000)            # disturb tile 0 only
    out = np.zeros(n, dtype)
    impl.lds_stream(y, out, 0.5, 9)
    te = tile_elems(dtype)
    _require_same_bits(out[te:], base[te:], "tiles 1.. do not see tile 0")
    if np.array_equal(out[:te], base[:te]):
        raise PinFailure("tile 0's output ignores tile 0's input")


def run_all(impl, dtype, random_array):
    pin_lds_copy_and_pure_rotation(impl, dtype)
    pin_lds_constant_fill(impl, dtype)
    pin_lds_exact_and_composition(impl, dtype)
    pin_lds_random_values(impl, dtype, random_array)
    pin_lds_tiles_are_independent(impl, dtype)
