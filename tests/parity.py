"""GPU library vs CPU oracle on identical seeded inputs: the chained sequence
copy -> scale -> add -> triad -> dot (state carried from kernel to kernel on both
sides) and the same five kernels each on fresh inputs."""
import numpy as np
import torch

import opal_inputs as oi
import oracle
import paper_2510_00932_amd as opal
from gpu_harness import GuardedArray, dot_device, opal_dtype

DOT_REL_TOL = {np.dtype(np.float64): 1e-12, np.dtype(np.float32): 1e-5}


def _bits(x):
    return x.view(np.uint64 if x.dtype == np.float64 else np.uint32)


def assert_same_bits(dev: GuardedArray, host: np.ndarray, what: str):
    got = dev.download()
    if not np.array_equal(_bits(got), _bits(host)):
        bad = np.nonzero(_bits(got) != _bits(host))[0]
        i = int(bad[0])
        raise AssertionError("%s: %d of %d elements differ from the oracle, first at i=%d: gpu %r oracle %r"
                             % (what, bad.size, host.size, i, got[i], host[i]))


def check_dot(r_gpu, ha, hb, what):
    """|gpu - oracle| / |oracle| against the tolerance for the element type; returns (rel, kappa)."""
    r_ref = oracle.dot(ha, hb)
    s_abs = oracle.dot_abs(ha, hb)
    tol = DOT_REL_TOL[ha.dtype]
    if r_ref == 0.0:
        assert abs(r_gpu) <= tol * max(s_abs, 1e-300), "%s: gpu %r oracle 0" % (what, r_gpu)
        return 0.0, float("inf")
    rel = abs(r_gpu - r_ref) / abs(r_ref)
    kappa = s_abs / abs(r_ref)
    assert rel <= tol, "%s: gpu %r oracle %r rel err %.3e > %.1e (condition number %.3e)" % (
        what, r_gpu, r_ref, rel, tol, kappa)
    return rel, kappa


def run_chain(host_abc, s, offsets=(0, 0, 0), stream=None, check_all_arrays_each_step=True, iters=1):
    """Chained sequence on both sides; bitwise comparison after every elementwise step.
    `iters` > 1 launches each kernel that many times (all five are idempotent)."""
    ha, hb, hc = (x.copy() for x in host_abc)
    n, dt = ha.shape[0], opal_dtype(ha.dtype)
    da, db, dc = (GuardedArray(n, x.dtype, off).upload(x) for x, off in zip((ha, hb, hc), offsets))
    torch.cuda.synchronize()
    devs = {"a": da, "b": db, "c": dc}
    hosts = {"a": ha, "b": hb, "c": hc}

    def compare(step, written):
        torch.cuda.synchronize()
        names = "abc" if check_all_arrays_each_step else written
        for name in names:
            assert_same_bits(devs[name], hosts[name], "%s, array %s (n=%d, offsets=%s)" % (step, name, n, offsets))

    oracle.copy(ha, hc)
    for _ in range(iters):
        opal.opal_copy(da.ptr, dc.ptr, n, dt, stream)
    compare("copy", "c")
    oracle.scale(hb, hc, s)
    for _ in range(iters):
        opal.opal_scale(db.ptr, dc.ptr, s, n, dt, stream)
    compare("scale", "b")
    oracle.add(ha, hb, hc)
    for _ in range(iters):
        opal.opal_add(da.ptr, db.ptr, dc.ptr, n, dt, stream)
    compare("add", "c")
    oracle.triad(ha, hb, hc, s)
    for _ in range(iters):
        opal.opal_triad(da.ptr, db.ptr, dc.ptr, s, n, dt, stream)
    compare("triad", "a")
    r = None
    for _ in range(iters):
        r2 = dot_device(da.ptr, db.ptr, n, dt, stream)
        assert r is None or r2 == r, "dot is not reproducible from launch to launch"
        r = r2
    stats = check_dot(r, ha, hb, "chained dot (n=%d, offsets=%s)" % (n, offsets)) if n else (0.0, 0.0)
    if n == 0:
        assert r == 0.0
    compare("after dot", "abc")
    for name in "abc":
        assert devs[name].guards_intact(), "guard band of %s overwritten" % name
    return stats


def run_fresh(host_abc, s, offsets=(0, 0, 0), stream=None):
    """Each kernel on the original inputs (restored between kernels)."""
    n, dt = host_abc[0].shape[0], opal_dtype(host_abc[0].dtype)
    devs = [GuardedArray(n, x.dtype, off).upload(x) for x, off in zip(host_abc, offsets)]
    keep = [d.view.clone() for d in devs]
    da, db, dc = devs

    def restore():
        for d, k in zip(devs, keep):
            d.view.copy_(k)
        torch.cuda.synchronize()

    def expect(fn):
        ha, hb, hc = (x.copy() for x in host_abc)
        fn(ha, hb, hc)
        torch.cuda.synchronize()
        for name, d, h in zip("abc", devs, (ha, hb, hc)):
            assert_same_bits(d, h, "fresh %s, array %s (n=%d, offsets=%s)" % (fn.__name__, name, n, offsets))
            assert d.guards_intact()

    def scale(ha, hb, hc):
        oracle.scale(hb, hc, s)

    def add(ha, hb, hc):
        oracle.add(ha, hb, hc)

    def triad(ha, hb, hc):
        oracle.triad(ha, hb, hc, s)

    torch.cuda.synchronize()
    opal.opal_scale(db.ptr, dc.ptr, s, n, dt, stream)
    expect(scale)
    restore()
    opal.opal_add(da.ptr, db.ptr, dc.ptr, n, dt, stream)
    expect(add)
    restore()
    opal.opal_triad(da.ptr, db.ptr, dc.ptr, s, n, dt, stream)
    expect(triad)
    restore()
    r = dot_device(da.ptr, db.ptr, n, dt, stream)
    return check_dot(r, host_abc[0], host_abc[1], "fresh dot (n=%d, offsets=%s)" % (n, offsets)) if n else (0.0, 0.0)


def workload_arrays(w: oi.Workload, n=None):
    return oi.make_arrays(w, n=n)
