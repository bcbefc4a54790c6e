"""Helpers for the GPU parity tests: guarded device arrays and an adapter that
lets the GPU library be driven with numpy arrays (so that it can be put through
the same pins as the CPU oracle).  torch is used for device memory only."""
import numpy as np
import torch

import paper_2510_00932_amd as opal

GUARD_BYTES = 1024          # sentinel bytes before and after every array
SENTINEL = 0xA5
_TORCH = {np.dtype(np.float64): torch.float64, np.dtype(np.float32): torch.float32}


def opal_dtype(np_dtype):
    return opal.OPAL_F64 if np.dtype(np_dtype) == np.float64 else opal.OPAL_F32


class GuardedArray:
    """n elements of dtype in device memory, starting `offset_elems` elements past a
    256-byte-aligned address, with sentinel-filled guard bands on both sides."""

    def __init__(self, n, np_dtype, offset_elems=0, device="cuda:0"):
        self.n = n
        self.np_dtype = np.dtype(np_dtype)
        item = self.np_dtype.itemsize
        self.off = GUARD_BYTES + offset_elems * item
        nbytes = self.off + n * item + GUARD_BYTES + 256
        self.raw = torch.full((nbytes,), SENTINEL, dtype=torch.uint8, device=device)
        assert self.raw.data_ptr() % 256 == 0, "torch device allocations are expected to be 256-byte aligned"
        self.view = self.raw[self.off:self.off + n * item].view(_TORCH[self.np_dtype])
        assert n == 0 or self.view.data_ptr() == self.raw.data_ptr() + self.off

    @property
    def ptr(self):
        return self.raw.data_ptr() + self.off

    def upload(self, host):
        assert host.dtype == self.np_dtype and host.shape == (self.n,)
        self.view.copy_(torch.from_numpy(host))
        return self

    def download(self, out=None):
        host = self.view.cpu().numpy()
        if out is not None:
            out[:] = host
            return out
        return host

    def guards_intact(self):
        end = self.off + self.n * self.np_dtype.itemsize
        front = self.raw[:self.off]
        back = self.raw[end:]
        return bool((front == SENTINEL).all().item()) and bool((back == SENTINEL).all().item())


class GpuImpl:
    """The GPU library behind the numpy-array interface the pins expect.
    offsets = per-array misalignment in elements for (a-role, b-role, c-role)."""

    def __init__(self, offsets=(0, 0, 0), stream=None):
        self.offsets = offsets
        self.stream = stream

    def _dev(self, host, k):
        dev = GuardedArray(host.shape[0], host.dtype, self.offsets[k]).upload(host)
        if self.stream is not None:
            torch.cuda.synchronize()      # uploads ran on torch's stream, the kernel will not
        return dev

    def _finish(self, pairs):
        torch.cuda.synchronize()
        for host, dev in pairs:
            assert dev.guards_intact(), "a kernel wrote outside its array"
            dev.download(host)

    def copy(self, a, c):
        da, dc = self._dev(a, 0), self._dev(c, 2)
        opal.opal_copy(da.ptr, dc.ptr, a.shape[0], opal_dtype(a.dtype), self.stream)
        self._finish([(a, da), (c, dc)])

    def scale(self, b, c, s):
        db, dc = self._dev(b, 1), self._dev(c, 2)
        opal.opal_scale(db.ptr, dc.ptr, s, b.shape[0], opal_dtype(b.dtype), self.stream)
        self._finish([(b, db), (c, dc)])

    def add(self, a, b, c):
        da, db, dc = self._dev(a, 0), self._dev(b, 1), self._dev(c, 2)
        opal.opal_add(da.ptr, db.ptr, dc.ptr, a.shape[0], opal_dtype(a.dtype), self.stream)
        self._finish([(a, da), (b, db), (c, dc)])

    def triad(self, a, b, c, s):
        da, db, dc = self._dev(a, 0), self._dev(b, 1), self._dev(c, 2)
        opal.opal_triad(da.ptr, db.ptr, dc.ptr, s, a.shape[0], opal_dtype(a.dtype), self.stream)
        self._finish([(a, da), (b, db), (c, dc)])

    def dot(self, a, b):
        da, db = self._dev(a, 0), self._dev(b, 1)
        r = dot_device(da.ptr, db.ptr, a.shape[0], opal_dtype(a.dtype), self.stream)
        self._finish([(a, da), (b, db)])
        return r


def dot_device(a_ptr, b_ptr, n, dtype, stream=None):
    """opal_dot with a freshly allocated workspace and result; returns the fp64 result on the host."""
    nbytes = opal.opal_dot_workspace_bytes(n, dtype)
    ws = torch.full((nbytes // 8 + 1,), float("nan"), dtype=torch.float64, device="cuda:0")
    res = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda:0")
    if stream is not None:
        torch.cuda.synchronize()      # the fills ran on torch's stream, the kernels will not
    opal.opal_dot(a_ptr, b_ptr, n, dtype, ws.data_ptr(), nbytes, res.data_ptr(), stream)
    torch.cuda.synchronize()
    return float(res.item())
