"""ctypes binding for libopal.so: argument marshalling only.

Every function mirrors one C entry point of include/opal.h (same name, same
argument order).  Array arguments are either integers (device addresses) or
torch tensors on a GPU; a tensor contributes its data_ptr() and, when `dtype`
is None, its element type.  A non-zero status raises OpalError.
"""
import ctypes
import os

from . import build as _build

OPAL_F64 = 0
OPAL_F32 = 1

_STATUS_NAMES = {0: "OPAL_OK", 1: "OPAL_ERR_NULL", 2: "OPAL_ERR_DTYPE", 3: "OPAL_ERR_ALIGN",
                 4: "OPAL_ERR_WORKSPACE", 5: "OPAL_ERR_LAUNCH", 6: "OPAL_ERR_SIZE"}

_LIB = None


class OpalError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("%s (%d): %s" % (_STATUS_NAMES.get(status, "?"), status, message))
        self.status = status


def lib_path() -> str:
    return _build.LIB


def load():
    """Load libopal.so (building it first only if no built library exists; refusing a library that was
    built from other sources than the present ones). Never falls back."""
    global _LIB
    if _LIB is not None:
        return _LIB
    # torch ships its own copy of the HIP runtime.  Importing it first makes the
    # dynamic linker bind libopal.so to that same copy, so that streams and device
    # pointers created by torch are the runtime's own when the library sees them.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    path = _build.LIB
    if not os.path.exists(path):
        _build.build(force=True)
    elif _build.is_stale():
        raise RuntimeError("libopal.so was built from other sources than the ones in this tree (built %s, sources %s): "
                           "rebuild it with `python paper_2510_00932_amd/build.py`"
                           % (_build.built_digest(), _build.source_digest()))
    lib = ctypes.CDLL(path)
    vp, sz, it, dbl = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_double
    lib.opal_copy.argtypes = [vp, vp, sz, it, vp]
    lib.opal_scale.argtypes = [vp, vp, dbl, sz, it, vp]
    lib.opal_add.argtypes = [vp, vp, vp, sz, it, vp]
    lib.opal_triad.argtypes = [vp, vp, vp, dbl, sz, it, vp]
    lib.opal_dot.argtypes = [vp, vp, sz, it, vp, sz, vp, vp]
    for name in ("opal_copy", "opal_scale", "opal_add", "opal_triad", "opal_dot"):
        getattr(lib, name).restype = it
    lib.opal_dot_static.argtypes = [vp, vp, sz, it, vp, vp]
    lib.opal_dot_static.restype = it
    lib.opal_dot_static_scratch_bytes.argtypes = []
    lib.opal_dot_static_scratch_bytes.restype = sz
    lib.opal_set_pacing.argtypes = [it]
    lib.opal_set_pacing.restype = None
    lib.opal_set_matched_order.argtypes = [it]
    lib.opal_set_matched_order.restype = None
    lib.opal_matched_order_state.argtypes = [vp, vp, vp, sz, it, ctypes.POINTER(ctypes.c_uint)]
    lib.opal_matched_order_state.restype = it
    lib.opal_get_pacing.argtypes = []
    lib.opal_get_pacing.restype = it
    lib.opal_pacing_configure.argtypes = [it, dbl, dbl, dbl, dbl, ctypes.c_uint, it, ctypes.c_uint]
    lib.opal_pacing_configure.restype = it
    lib.opal_dot_workspace_bytes.argtypes = [sz, it]
    lib.opal_dot_workspace_bytes.restype = sz
    lib.opal_status_string.argtypes = [it]
    lib.opal_status_string.restype = ctypes.c_char_p
    lib.opal_lds_tile_elements.argtypes = [it]
    lib.opal_lds_tile_elements.restype = sz
    lib.opal_lds_stream.argtypes = [vp, vp, dbl, sz, ctypes.c_uint, it, vp]
    lib.opal_lds_stream.restype = it
    lib.opal_last_hip_error.argtypes = []
    lib.opal_last_hip_error.restype = ctypes.c_char_p
    lib.opal_bytes_per_element.argtypes = [it, it]
    lib.opal_bytes_per_element.restype = sz
    _LIB = lib
    return lib


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        if not x.is_cuda:
            raise TypeError("libopal takes device memory; got a tensor on %s" % x.device)
        if not x.is_contiguous():
            raise ValueError("libopal takes dense, contiguous arrays")
        return x.data_ptr()
    raise TypeError("expected a device address (int) or a torch GPU tensor, got %r" % type(x))


def _stream(stream):
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream        # torch.cuda.Stream


def _dtype_of(x, dtype):
    if dtype is not None:
        return dtype
    if hasattr(x, "dtype"):
        name = str(x.dtype)
        if name.endswith("float64"):
            return OPAL_F64
        if name.endswith("float32"):
            return OPAL_F32
        raise TypeError("libopal supports float64 and float32 arrays, got %s" % name)
    raise TypeError("dtype must be given when arrays are passed as addresses")


def _check(status):
    if status != 0:
        detail = opal_status_string(status)
        if status == 5:
            detail += " [%s]" % load().opal_last_hip_error().decode()
        raise OpalError(status, detail)


def opal_status_string(status: int) -> str:
    return load().opal_status_string(int(status)).decode()


def opal_bytes_per_element(kernel: int, dtype: int) -> int:
    return int(load().opal_bytes_per_element(int(kernel), int(dtype)))


def opal_copy(a, c, n, dtype=None, stream=None):
    """c[i] = a[i]."""
    _check(load().opal_copy(_ptr(a), _ptr(c), n, _dtype_of(a, dtype), _stream(stream)))


def opal_scale(b, c, s, n, dtype=None, stream=None):
    """b[i] = s * c[i]."""
    _check(load().opal_scale(_ptr(b), _ptr(c), float(s), n, _dtype_of(c, dtype), _stream(stream)))


def opal_add(a, b, c, n, dtype=None, stream=None):
    """c[i] = a[i] + b[i]."""
    _check(load().opal_add(_ptr(a), _ptr(b), _ptr(c), n, _dtype_of(a, dtype), _stream(stream)))


def opal_triad(a, b, c, s, n, dtype=None, stream=None):
    """a[i] = b[i] + s * c[i]."""
    _check(load().opal_triad(_ptr(a), _ptr(b), _ptr(c), float(s), n, _dtype_of(b, dtype), _stream(stream)))


def opal_dot_workspace_bytes(n, dtype) -> int:
    return int(load().opal_dot_workspace_bytes(n, int(dtype)))


def opal_dot(a, b, n, dtype, workspace, workspace_bytes, result, stream=None):
    """result[0] = sum a[i]*b[i] (result: one fp64 in device memory)."""
    _check(load().opal_dot(_ptr(a), _ptr(b), n, _dtype_of(a, dtype), _ptr(workspace), workspace_bytes,
                           _ptr(result), _stream(stream)))


def opal_dot_static_scratch_bytes() -> int:
    return int(load().opal_dot_static_scratch_bytes())


def opal_dot_static(a, b, n, dtype, result, stream=None):
    """opal_dot with the partial sums in the library's own fixed device array (no workspace argument)."""
    _check(load().opal_dot_static(_ptr(a), _ptr(b), n, _dtype_of(a, dtype), _ptr(result), _stream(stream)))


def opal_set_pacing(mode) -> None:
    """0 / False: off; 1 / True: on from the library's size thresholds; 2: on wherever the shape fits."""
    load().opal_set_pacing(int(mode))


def opal_set_matched_order(on) -> None:
    """Paced Add and Triad: second input in one of the two class-matched orders, learnt per pair of inputs (default),
    in the first input's order (0), or learnt with the other of the two orders timed first (2).  Every call starts
    the learning afresh."""
    load().opal_set_matched_order(2 if on == 2 and on is not True else (1 if on else 0))


def opal_matched_order_state(out, in0, in1, n, dtype):
    """(launches so far, shortest ticks with order 0, with order 1, order of the next launch) for the inputs of a
    paced Add or Triad call with these arguments.  Waits for the default stream only: synchronise other streams first."""
    state = (ctypes.c_uint * 4)()
    _check(load().opal_matched_order_state(ctypes.c_void_p(out), ctypes.c_void_p(in0), ctypes.c_void_p(in1),
                                           ctypes.c_size_t(n), int(dtype), state))
    return tuple(int(v) for v in state)


def opal_get_pacing() -> int:
    return int(load().opal_get_pacing())


def opal_pacing_configure(kind, terabytes_per_second, store_at, second_input_at, gap, tolerance_ticks, feedback,
                          set_bit=3):
    _check(load().opal_pacing_configure(int(kind), float(terabytes_per_second), float(store_at),
                                        float(second_input_at), float(gap), int(tolerance_ticks),
                                        1 if feedback else 0, int(set_bit)))


def opal_lds_tile_elements(dtype) -> int:
    return int(load().opal_lds_tile_elements(int(dtype)))


def opal_lds_stream(inp, out, c, n, rep, dtype=None, stream=None):
    """Tile-wise: rotate by one 16-byte vector and add c, rep times, through the LDS."""
    _check(load().opal_lds_stream(_ptr(inp), _ptr(out), float(c), n, int(rep), _dtype_of(inp, dtype), _stream(stream)))
