"""The LDS-streaming microkernel on the GPU: bit-exact against the oracle and against the pins."""
import numpy as np
import pytest
import torch

import opal_inputs as oi
import paper_2510_00932_amd as opal

pytestmark = pytest.mark.gpu

DTYPES = [np.float64, np.float32]


class GpuLds:
    """opal_lds_stream behind the numpy interface of the pins (guarded device arrays)."""

    def __init__(self, stream=None):
        self.stream = stream

    def lds_stream(self, inp, out, c, rep):
        from gpu_harness import GuardedArray, opal_dtype
        n = inp.shape[0]
        di = GuardedArray(n, inp.dtype).upload(inp)
        do = GuardedArray(n, out.dtype).upload(out)
        torch.cuda.synchronize()
        opal.opal_lds_stream(di.ptr, do.ptr, c, n, rep, opal_dtype(inp.dtype), self.stream)
        torch.cuda.synchronize()
        assert di.guards_intact() and do.guards_intact()
        di.download(inp)
        do.download(out)


@pytest.fixture(scope="module")
def gpu():
    assert torch.cuda.is_available()
    opal.load()


@pytest.mark.parametrize("dtype", DTYPES)
def test_pins_hold_on_the_gpu(gpu, dtype):
    import pins_lds
    x = oi.uniform_array(11, 0, 2 * pins_lds.tile_elems(dtype), dtype, -1.0, 1.0)
    pins_lds.run_all(GpuLds(), dtype, x)


@pytest.mark.parametrize("dtype", DTYPES)
def test_bit_exact_against_the_oracle(gpu, dtype):
    import oracle
    import pins_lds
    te = pins_lds.tile_elems(dtype)
    impl = GpuLds()
    for tiles, rep, c in ((1, 1, 0.4), (7, 13, -0.75), (300, 600, 0.1), (2049, 3, 0.4), (64, 1500, 1e-3)):
        n = tiles * te
        x = oi.uniform_array(42, 2, n, dtype, -1.0, 1.0)
        want = np.zeros(n, dtype)
        oracle.lds_stream(x, want, c, rep)
        got = np.full(n, 7, dtype)
        impl.lds_stream(x.copy(), got, c, rep)
        bits = np.uint64 if dtype == np.float64 else np.uint32
        assert np.array_equal(got.view(bits), want.view(bits)), (tiles, rep, c)


def test_zero_length_and_errors(gpu):
    from gpu_harness import GuardedArray
    opal.opal_lds_stream(0, 0, 0.1, 0, 5, opal.OPAL_F64, None)          # n == 0: nothing happens
    a = GuardedArray(4096, np.float64).upload(np.ones(4096))
    b = GuardedArray(4096, np.float64).upload(np.zeros(4096))
    for args, status in (((a.ptr, b.ptr, 0.1, 2047, 1, opal.OPAL_F64, None), 6),
                         ((a.ptr + 8, b.ptr, 0.1, 2048, 1, opal.OPAL_F64, None), 3),
                         ((a.ptr, b.ptr, 0.1, 2048, 1, 9, None), 2),
                         ((0, b.ptr, 0.1, 2048, 1, opal.OPAL_F64, None), 1)):
        with pytest.raises(opal.OpalError) as e:
            opal.opal_lds_stream(*args)
        assert e.value.status == status
    torch.cuda.synchronize()
    assert (b.download() == 0).all()


def test_on_a_side_stream(gpu):
    import oracle
    n = 16 * 2048
    x = oi.uniform_array(5, 0, n, np.float64, 0.5, 1.5)
    want = np.zeros(n)
    oracle.lds_stream(x, want, 0.4, 77)
    got = np.zeros(n)
    GpuLds(torch.cuda.Stream()).lds_stream(x.copy(), got, 0.4, 77)
    assert np.array_equal(got.view(np.uint64), want.view(np.uint64))
