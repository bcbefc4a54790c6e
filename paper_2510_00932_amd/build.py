"""Compile libopal.so (HIP kernels + C ABI) for gfx950, in-tree, next to this file."""
import hashlib
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "opal.hip")
DEPS = [SRC] + [os.path.join(HERE, "csrc", f) for f in
                ("stream_kernels.hpp", "lds_kernel.hpp", "launch_shapes.hpp", "launch_plan.hpp", "pacing.hpp")] + \
    [os.path.join(os.path.dirname(HERE), "include", "opal.h")]
LIB = os.path.join(HERE, "libopal.so")
STAMP = os.path.join(HERE, "libopal.build_digest")   # digest of the sources the built library came from

# Everything that decides what the GPU executes for a call: kernels, launch shapes, work
# decomposition, timetable and the host code that picks between them.
KERNEL_SOURCES = [os.path.join(HERE, "csrc", f) for f in
                  ("stream_kernels.hpp", "launch_shapes.hpp", "launch_plan.hpp", "pacing.hpp", "opal.hip")]


def _digest(paths) -> str:
    h = hashlib.sha256()
    for path in paths:
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def kernel_source_digest() -> str:
    """Ties measured figures (HBM traffic per launch) to the sources they were measured on."""
    return _digest(KERNEL_SOURCES)


def source_digest() -> str:
    """Digest of every file libopal.so is built from."""
    return _digest(sorted(DEPS))


def built_digest():
    """Digest recorded when libopal.so was built, or None if there is no record."""
    if not (os.path.exists(LIB) and os.path.exists(STAMP)):
        return None
    with open(STAMP) as f:
        return f.read().strip()

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
    """True if there is no built library or it was built from other sources than the present ones
    (by content, not by file time: the built library travels between machines)."""
    return built_digest() != source_digest()


def build(force: bool = True) -> str:
    if not force and not is_stale():
        return LIB
    tmp = LIB + ".tmp.%d" % os.getpid()
    digest = source_digest()
    subprocess.run([HIPCC, *FLAGS, SRC, "-o", tmp], check=True)
    os.replace(tmp, LIB)
    with open(STAMP, "w") as f:
        f.write(digest + "\n")
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    print(build_shape_study())
