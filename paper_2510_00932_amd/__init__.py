"""Streaming vector kernels (Copy, Mul/scale, Add, Triad, Dot; Table 1 of the
paper) as hand-written HIP kernels for MI355X behind a C ABI (libopal.so).

    from paper_2510_00932_amd import opal_copy, opal_scale, opal_add, opal_triad, opal_dot

The functions have the names and argument order of the C entry points declared
in include/opal.h and only marshal arguments: device pointers may be given as
torch tensors (their data_ptr() is passed on) or as plain integers.  All
arithmetic runs in the library's kernels; there is no CPU fallback, and
importing a function that needs the library fails loudly if it is not built.
"""
from .binding import (  # noqa: F401
    OPAL_F32,
    OPAL_F64,
    OpalError,
    lib_path,
    load,
    opal_add,
    opal_bytes_per_element,
    opal_copy,
    opal_dot,
    opal_dot_static,
    opal_dot_static_scratch_bytes,
    opal_dot_workspace_bytes,
    opal_get_pacing,
    opal_pacing_configure,
    opal_set_pacing,
    opal_set_matched_order,
    opal_matched_order_state,
    opal_lds_stream,
    opal_lds_tile_elements,
    opal_scale,
    opal_status_string,
    opal_triad,
)
