"""opal_dot_static (the entry point that allocates nothing: its partial sums live in a fixed
device array inside the library) against opal_dot with a caller workspace, through the C ABI.
Both run the same kernels, so for the same inputs the two results must have the same bits;
they are also held to opal_dot's own tolerance against the CPU oracle.  Two calls in a row, the
second on a smaller input, so that partial sums left behind by the first would show."""
import numpy as np
import pytest
import torch

import opal_inputs as oi
import paper_2510_00932_amd as opal

pytestmark = pytest.mark.gpu

TOL = {np.dtype(np.float64): 1e-12, np.dtype(np.float32): 1e-5}


def _both(da, db, n, dt, stream=None):
    """(result of opal_dot_static, result of opal_dot) on the same device arrays."""
    need = opal.opal_dot_workspace_bytes(n, dt)
    assert need <= opal.opal_dot_static_scratch_bytes()
    ws = torch.full((need // 8 + 1,), float("nan"), dtype=torch.float64, device="cuda:0")
    res = torch.full((2,), float("nan"), dtype=torch.float64, device="cuda:0")
    torch.cuda.synchronize()
    opal.opal_dot_static(da, db, n, dt, res.data_ptr(), stream)
    torch.cuda.synchronize()
    opal.opal_dot(da, db, n, dt, ws.data_ptr(), need, res.data_ptr() + 8, stream)
    torch.cuda.synchronize()
    out = res.cpu().numpy()
    return float(out[0]), float(out[1])


@pytest.mark.parametrize("np_dtype", [np.float64, np.float32])
def test_static_scratch_dot_equals_workspace_dot_twice_in_a_row(np_dtype, oracle):
    assert torch.cuda.is_available()
    opal.load()
    dt = opal.OPAL_F64 if np_dtype == np.float64 else opal.OPAL_F32
    # first a size at which every compute unit's workgroup writes a partial sum, then one
    # that uses only a few of those slots, then the empty and one-element cases
    for n in ((1 << 22) + 4099, 70001, 0, 1):
        print("opal_dot_static: %s n=%d" % (np.dtype(np_dtype).name, n), flush=True)
        ha = oi.uniform_array(7, 0, n, np_dtype, 0.5, 1.5)
        hb = oi.uniform_array(7, 1, n, np_dtype, 0.5, 1.5)
        da = torch.from_numpy(ha).cuda()
        db = torch.from_numpy(hb).cuda()
        pa = da.data_ptr() if n else 0
        pb = db.data_ptr() if n else 0
        got, want_gpu = _both(pa, pb, n, dt)
        assert np.float64(got).view(np.uint64) == np.float64(want_gpu).view(np.uint64), (n, got, want_gpu)
        ref = oracle.dot(ha, hb)
        if n == 0:
            assert got == 0.0 and ref == 0.0
        else:
            assert abs(got - ref) <= TOL[np.dtype(np_dtype)] * abs(ref), (n, got, ref)


def test_static_scratch_dot_on_a_side_stream_and_misaligned(oracle):
    opal.load()
    n = 300007
    ha = oi.uniform_array(11, 0, n + 1, np.float64, 0.5, 1.5)
    hb = oi.uniform_array(11, 1, n + 3, np.float64, 0.5, 1.5)
    da = torch.from_numpy(ha).cuda()
    db = torch.from_numpy(hb).cuda()
    stream = torch.cuda.Stream()
    got, want_gpu = _both(da.data_ptr() + 8, db.data_ptr() + 24, n, opal.OPAL_F64, stream)
    assert got == want_gpu
    ref = oracle.dot(ha[1:], hb[3:])
    assert abs(got - ref) <= 1e-12 * abs(ref)


def test_static_scratch_dot_on_the_paced_shape_then_a_small_one(oracle):
    """An array large enough for the paced shape (1024 partial sums), then a small one (a few)."""
    opal.load()
    opal.opal_set_pacing(2)
    for n in ((192 << 20) // 8 + 12345, 5000):
        print("opal_dot_static: paced-size check n=%d" % n, flush=True)
        ha = oi.uniform_array(13, 0, n, np.float64, 0.5, 1.5, threads=16)
        hb = oi.uniform_array(13, 1, n, np.float64, 0.5, 1.5, threads=16)
        da, db = torch.from_numpy(ha).cuda(), torch.from_numpy(hb).cuda()
        got, want_gpu = _both(da.data_ptr(), db.data_ptr(), n, opal.OPAL_F64)
        assert got == want_gpu, (n, got, want_gpu)
        ref = oracle.dot(ha, hb)
        assert abs(got - ref) <= 1e-12 * abs(ref), (n, got, ref)
    opal.opal_set_pacing(1)


def test_static_scratch_dot_argument_errors():
    A = 0x1000
    for args, status in (((0, A, 10, opal.OPAL_F64, A), 1), ((A, A, 10, opal.OPAL_F64, 0), 1),
                         ((A, A, 10, 7, A), 2), ((A, A + 4, 10, opal.OPAL_F64, A), 3),
                         ((A, A, 10, opal.OPAL_F64, A + 4), 3)):
        with pytest.raises(opal.OpalError) as e:
            opal.opal_dot_static(*args)
        assert e.value.status == status
