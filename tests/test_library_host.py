"""Host-side checks of libopal that need no GPU: the library loads, exports every
function include/opal.h declares, and rejects bad arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

import paper_2510_00932_amd as opal

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "opal.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(opal_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_five_kernels():
    names = _declared_functions()
    for want in ("opal_copy", "opal_scale", "opal_add", "opal_triad", "opal_dot",
                 "opal_dot_workspace_bytes", "opal_status_string"):
        assert want in names


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(opal.lib_path())
    for name in _declared_functions():
        assert hasattr(lib, name), name


def test_status_strings():
    seen = set()
    for st in range(7):
        msg = opal.opal_status_string(st)
        assert msg and msg not in seen
        seen.add(msg)
    assert opal.opal_status_string(99) == "unknown status"


def test_bytes_per_element():
    assert [opal.opal_bytes_per_element(k, opal.OPAL_F64) for k in range(5)] == [16, 16, 24, 24, 16]
    assert [opal.opal_bytes_per_element(k, opal.OPAL_F32) for k in range(5)] == [8, 8, 12, 12, 8]
    assert opal.opal_bytes_per_element(5, opal.OPAL_F64) == 0
    assert opal.opal_bytes_per_element(0, 7) == 0


def test_dot_workspace_is_a_pure_bounded_function():
    for dt in (opal.OPAL_F64, opal.OPAL_F32):
        prev = 0
        for n in (0, 1, 1000, 1 << 20, 1 << 25, 1 << 28, 300000007, 1 << 40):
            w = opal.opal_dot_workspace_bytes(n, dt)
            assert 8 <= w <= 65536 and w % 8 == 0
            assert w >= prev
            prev = w
    assert opal.opal_dot_workspace_bytes(100, 9) == 0


def _status(fn, *args):
    try:
        fn(*args)
    except opal.OpalError as e:
        return e.status
    return 0


A = 0x1000  # fake, suitably aligned "device addresses": argument errors return before any GPU call


def test_argument_errors_are_found_on_the_host():
    f64 = opal.OPAL_F64
    assert _status(opal.opal_copy, 0, A, 10, f64) == 1
    assert _status(opal.opal_copy, A, 0, 10, f64) == 1
    assert _status(opal.opal_scale, A, 0, 0.4, 10, f64) == 1
    assert _status(opal.opal_add, A, 0, A, 10, f64) == 1
    assert _status(opal.opal_triad, A, A, 0, 0.4, 10, f64) == 1
    assert _status(opal.opal_copy, A, A, 10, 2) == 2
    assert _status(opal.opal_copy, A, A, 10, -1) == 2
    assert _status(opal.opal_copy, A + 4, A, 10, f64) == 3
    assert _status(opal.opal_add, A, A + 2, A, 10, opal.OPAL_F32) == 3
    assert _status(opal.opal_triad, A + 1, A, A, 0.4, 10, f64) == 3


def test_dot_argument_errors():
    f64 = opal.OPAL_F64
    need = opal.opal_dot_workspace_bytes(1 << 20, f64)
    assert _status(opal.opal_dot, 0, A, 1 << 20, f64, A, need, A) == 1
    assert _status(opal.opal_dot, A, A, 1 << 20, f64, 0, need, A) == 1
    assert _status(opal.opal_dot, A, A, 1 << 20, f64, A, need, 0) == 1
    assert _status(opal.opal_dot, A, A, 1 << 20, 5, A, need, A) == 2
    assert _status(opal.opal_dot, A, A + 4, 1 << 20, f64, A, need, A) == 3
    assert _status(opal.opal_dot, A, A, 1 << 20, f64, A + 4, need, A) == 3
    assert _status(opal.opal_dot, A, A, 1 << 20, f64, A, need, A + 4) == 3
    assert _status(opal.opal_dot, A, A, 1 << 20, f64, A, need - 8, A) == 4


def test_zero_length_elementwise_calls_do_nothing():
    # n == 0: valid, no launch, pointers are not even looked at
    assert _status(opal.opal_copy, 0, 0, 0, opal.OPAL_F64) == 0
    assert _status(opal.opal_triad, 0, 0, 0, 0.4, 0, opal.OPAL_F32) == 0


def test_binding_refuses_host_tensors():
    import torch
    t = torch.zeros(4, dtype=torch.float64)
    with pytest.raises(TypeError):
        opal.opal_copy(t, t, 4)


def _no_gpu():
    import torch
    return not torch.cuda.is_available()


@pytest.mark.skipif(not _no_gpu(), reason="with a GPU present these calls would launch on made-up addresses")
def test_runtime_failures_surface_as_err_launch_with_the_hip_error_name():
    """Without a usable GPU the first runtime query of a call fails: the call must return OPAL_ERR_LAUNCH
    (never crash, never report success) and opal_last_hip_error() must name the runtime's error."""
    lib = opal.load()
    n = 1 << 20
    assert _status(opal.opal_copy, A, A + (n << 4), n, opal.OPAL_F64) == 5
    name = lib.opal_last_hip_error().decode()
    assert name.startswith("hipError") and name != "hipSuccess", name
    need = opal.opal_dot_workspace_bytes(n, opal.OPAL_F64)
    assert _status(opal.opal_dot, A, A + (n << 4), n, opal.OPAL_F64, A, need, A) == 5
    assert _status(opal.opal_dot_static, A, A + (n << 4), n, opal.OPAL_F64, A) == 5
    try:
        opal.opal_copy(A, A + (n << 4), n, opal.OPAL_F64)
    except opal.OpalError as e:
        assert "hipError" in str(e)          # the binding appends the runtime's error name to status 5


def test_sizes_whose_byte_count_does_not_fit_are_refused_before_any_gpu_call():
    huge = 1 << 62
    assert _status(opal.opal_copy, A, A, huge, opal.OPAL_F64) == 6
    assert _status(opal.opal_triad, A, A, A, 0.4, huge, opal.OPAL_F64) == 6
    assert _status(opal.opal_copy, A, A, 1 << 63, opal.OPAL_F32) == 6
    need = opal.opal_dot_workspace_bytes(huge, opal.OPAL_F64)
    assert _status(opal.opal_dot, A, A, huge, opal.OPAL_F64, A, need, A) == 6


def test_dot_with_n_zero_still_needs_result_and_workspace():
    # the pointer checks of opal_dot do not depend on n (documented in opal.h)
    assert _status(opal.opal_dot, 0, 0, 0, opal.OPAL_F64, 0, 64, A) == 1
    assert _status(opal.opal_dot, 0, 0, 0, opal.OPAL_F64, A, 64, 0) == 1


def test_pacing_switch_and_tuning_hook_are_host_only():
    lib = opal.load()
    before = opal.opal_get_pacing()
    for mode in (0, 1, 2):
        opal.opal_set_pacing(mode)
        assert opal.opal_get_pacing() == mode
    opal.opal_set_pacing(before)
    assert lib.opal_pacing_configure(7, 7.0, 0.5, 0.0, 0.0, 100, 1, 3) == 6
    assert lib.opal_pacing_configure(0, 7.0, 0.5, 0.0, 0.0, 100, 1, 12) == 6


def test_matched_order_state_argument_errors_are_found_on_the_host():
    f64 = opal.OPAL_F64
    assert _status(opal.opal_matched_order_state, A, A, A, 1 << 27, 7) == 2
    assert _status(opal.opal_matched_order_state, 0, A, A, 1 << 27, f64) == 1
    assert _status(opal.opal_matched_order_state, A, 0, A, 1 << 27, f64) == 1
    assert _status(opal.opal_matched_order_state, A, A, 0, 1 << 27, f64) == 1
    lib = opal.load()
    assert lib.opal_matched_order_state(A, A, A, 1 << 27, f64, None) == 1
    # without a GPU the device words cannot be reached: a runtime failure, not a crash
    if _no_gpu():
        assert _status(opal.opal_matched_order_state, A, A, A, 1 << 27, f64) == 5
    for setting in (0, 2, 1):
        opal.opal_set_matched_order(setting)   # host only


def test_built_library_matches_the_sources():
    from paper_2510_00932_amd import build
    opal.load()
    assert not build.is_stale()
    assert build.built_digest() == build.source_digest()
