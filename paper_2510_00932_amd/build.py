"""Compile libopal.so (HIP kernels + C ABI) for gfx950, in-tree, next to this file."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "opal.hip")
DEPS = [SRC] + [os.path.join(HERE, "csrc", f) for f in
                ("stream_kernels.hpp", "lds_kernel.hpp", "launch_shapes.hpp", "launch_plan.hpp", "pacing.hpp")] + \
    [os.path.join(os.path.dirname(HERE), "include", "opal.h")]
LIB = os.path.join(HERE, "libopal.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -ffp-contract=off     : Triad keeps a rounded multiply followed by a rounded add.
# -packed-fp32-ops off  : fp32 vector math is emitted as scalar-lane VALU ops, never v_pk_*_f32.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-fPIC", "-shared", "-Wall", "-Wextra", "-Wno-unused-command-line-argument"]


STUDY_SRC = os.path.join(HERE, "csrc", "shape_study.hip")
STUDY_BIN = os.path.join(HERE, "shape_study")


def build_shape_study() -> str:
    """The stand-alone program that runs the alternative launch shapes side by side (for rocprofv3)."""
    flags = [f for f in FLAGS if f not in ("-fPIC", "-shared")]
    tmp = STUDY_BIN + ".tmp.%d" % os.getpid()
    subprocess.run([HIPCC, *flags, STUDY_SRC, "-o", tmp], check=True)
    os.replace(tmp, STUDY_BIN)
    return STUDY_BIN


def is_stale() -> bool:
    return (not os.path.exists(LIB)) or any(os.path.getmtime(d) > os.path.getmtime(LIB) for d in DEPS)


def build(force: bool = True) -> str:
    if not force and not is_stale():
        return LIB
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.run([HIPCC, *FLAGS, SRC, "-o", tmp], check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    print(build_shape_study())
