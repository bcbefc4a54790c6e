#!/usr/bin/env python3
"""Benchmark of the five streaming vector kernels (Copy, Mul/scale, Add, Triad, Dot;
Table 1 of the paper) on one MI355X.

A step is one pass copy -> scale -> add -> triad -> dot over the three resident
arrays of one synthetic workload, every kernel launched through the C ABI on one
HIP stream.  Prints ONE JSON line:

  value / ms_per_step : bytes of all five kernels per step / wall time per step, K steps
                        bracketed by device synchronisation (inputs already in HBM)
  kernels             : per kernel, from HIP events recorded on the launch stream around
                        every launch of the timed region: average / min / median time,
                        GB/s of algorithmic bytes and the fraction of the 8 TB/s HBM peak
  roofline            : the same for the kernel that takes the largest share of the step
  cpu_baseline        : the CPU oracle timed on this machine's host cores on the same
                        workload (also used to check the GPU results of this run)

Algorithmic bytes: every input element read once and every output element written once
(16, 16, 24, 24, 16 bytes per element in fp64; half that in fp32).
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak
KERNELS = ("copy", "scale", "add", "triad", "dot")


def kernel_source_digest():
    from paper_2510_00932_amd.build import kernel_source_digest as digest
    return digest()


def measured_traffic(workload_name, kernel):
    """HBM bytes per launch from the stored rocprofv3 counter runs, or None when there are
    none for this workload/kernel or the kernel sources have changed since they were taken."""
    path = os.path.join(ROOT, "paper_2510_00932_amd", "measured_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        rec = json.load(f)
    if rec.get("source_digest") != kernel_source_digest():
        return None
    return rec.get("workloads", {}).get(workload_name, {}).get(kernel)


def paper_shapes(args):
    """The paper's own workload shapes for these kernels (Table 1: ARRAY_SIZE in {2000896, 4000768,
    6000640}, num_times in {100, 200, 300}): 16-48 MB arrays that sit in the 256 MB Infinity Cache, where a
    kernel lasts a few microseconds and the launch path decides the run time (the regime of the paper's
    Section 6.4 finding).  One iteration = copy, scale, add, triad, dot.  Three ways to issue the
    iterations through the same C ABI are timed wall-clock, synchronisation to synchronisation:
      eager     : num_times x 5 asynchronous calls, one synchronisation at the end
      graph     : one iteration captured into a HIP graph, replayed num_times
      graph_all : all num_times iterations captured into one HIP graph, launched once
    Prints one JSON line."""
    import numpy as np
    import torch

    import opal_inputs as oi
    import paper_2510_00932_amd as opal

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the kernels have no CPU fallback", file=sys.stderr)
        sys.exit(2)
    opal.load()
    dev = torch.device("cuda:0")
    wl = oi.workload(0)
    s = wl.s
    results = []
    checks = []
    cases = [(n, dtype_name) for dtype_name in ("f64", "f32") for n in (2000896, 4000768, 6000640)]
    for n, dtype_name in cases:
        dt, tdt, item, npdt = (opal.OPAL_F64, torch.float64, 8, np.float64) if dtype_name == "f64" else \
            (opal.OPAL_F32, torch.float32, 4, np.float32)
        bits = np.uint64 if dtype_name == "f64" else np.uint32
        host = [oi.uniform_array(wl.seed, k, n, npdt, wl.lo, wl.hi) for k in range(3)]
        pitch = (n * item + 255) // 256 * 256 + args.skew_bytes
        pool = torch.empty(3 * pitch + 256, dtype=torch.uint8, device=dev)
        a, b, c = (pool[k * pitch:k * pitch + n * item].view(tdt) for k in range(3))
        ws_bytes = opal.opal_dot_workspace_bytes(n, dt)
        ws = torch.empty(ws_bytes // 8, dtype=torch.float64, device=dev)
        res = torch.empty(1, dtype=torch.float64, device=dev)
        stream = torch.cuda.Stream()
        pa, pb, pc, pws, pres = a.data_ptr(), b.data_ptr(), c.data_ptr(), ws.data_ptr(), res.data_ptr()

        def reset():
            for d, h in zip((a, b, c), host):
                d.copy_(torch.from_numpy(h))
            torch.cuda.synchronize()

        def iteration(st):
            opal.opal_copy(pa, pc, n, dt, st)
            opal.opal_scale(pb, pc, s, n, dt, st)
            opal.opal_add(pa, pb, pc, n, dt, st)
            opal.opal_triad(pa, pb, pc, s, n, dt, st)
            opal.opal_dot(pa, pb, n, dt, pws, ws_bytes, pres, st)

        reset()
        iteration(stream)
        stream.synchronize()
        g1 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g1, stream=stream):
            iteration(torch.cuda.current_stream())
        bytes_per_iter = 12 * item * n
        for num_times in (100, 200, 300):
            row = {"array_size": n, "dtype": dtype_name, "num_times": num_times}
            # eager
            reset()
            t0 = time.perf_counter()
            for _ in range(num_times):
                iteration(stream)
            stream.synchronize()
            t = time.perf_counter() - t0
            row["eager_us_per_iter"] = round(t / num_times * 1e6, 2)
            final_eager = (a.cpu().numpy(), b.cpu().numpy(), c.cpu().numpy(), float(res.item()))
            # graph of one iteration, replayed
            reset()
            t0 = time.perf_counter()
            for _ in range(num_times):
                g1.replay()
            torch.cuda.synchronize()
            t = time.perf_counter() - t0
            row["graph_us_per_iter"] = round(t / num_times * 1e6, 2)
            final_graph = (a.cpu().numpy(), b.cpu().numpy(), c.cpu().numpy(), float(res.item()))
            # one graph holding every iteration
            gall = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gall, stream=stream):
                for _ in range(num_times):
                    iteration(torch.cuda.current_stream())
            reset()
            t0 = time.perf_counter()
            gall.replay()
            torch.cuda.synchronize()
            t = time.perf_counter() - t0
            row["graph_all_us_per_iter"] = round(t / num_times * 1e6, 2)
            final_all = (a.cpu().numpy(), b.cpu().numpy(), c.cpu().numpy(), float(res.item()))
            del gall
            best = min(row["eager_us_per_iter"], row["graph_us_per_iter"], row["graph_all_us_per_iter"])
            row["best_GBps"] = round(bytes_per_iter / best / 1e3, 1)
            same = all(np.array_equal(x.view(bits), y.view(bits)) and np.array_equal(x.view(bits), z.view(bits))
                       for x, y, z in zip(final_eager[:3], final_graph[:3], final_all[:3]))
            row["three_ways_bit_identical"] = bool(same and final_eager[3] == final_graph[3] == final_all[3])
            if num_times == 100 and not args.no_cpu_baseline:
                import oracle
                xa, xb, xc = (h.copy() for h in host)
                r = 0.0
                for _ in range(num_times):
                    oracle.copy(xa, xc)
                    oracle.scale(xb, xc, s)
                    oracle.add(xa, xb, xc)
                    oracle.triad(xa, xb, xc, s)
                    r = oracle.dot(xa, xb)
                exact = all(np.array_equal(x.view(bits), y.view(bits)) for x, y in zip(final_eager[:3], (xa, xb, xc)))
                rel = abs(final_eager[3] - r) / abs(r)
                checks.append({"array_size": n, "dtype": dtype_name, "num_times": num_times,
                               "elementwise_bit_exact": bool(exact), "dot_rel_err": float("%.3e" % rel),
                               "dot_tolerance": 1e-12 if dtype_name == "f64" else 1e-5})
            results.append(row)
        del g1
    out = {"metric": "time per iteration (copy, scale, add, triad, dot) at the paper's array sizes, 1 GPU",
           "unit": "us", "dtype": "f64 and f32", "data": "synthetic", "bytes_per_iteration": "12 * element size * array_size",
           "results": results, "check_vs_oracle": checks}
    print(json.dumps(out))
    bad = [r for r in results if not r["three_ways_bit_identical"]] + \
        [c for c in checks if not (c["elementwise_bit_exact"] and c["dot_rel_err"] <= c["dot_tolerance"])]
    if bad:
        print("bench.py: paper-shape results differ", file=sys.stderr)
        sys.exit(1)


def call_overhead(args):
    """Host cost of one call through the C ABI, in the regime where a kernel lasts microseconds (the paper's
    Section 6.4 finding was a host-side cost per launch): `calls` back-to-back calls on arrays of 64 elements.
      enqueue_us : host time per call while the queue still has room (the call itself: argument checks, the
                   device query of opal_dot, one or two hipLaunchKernel)
      drain_us   : wall time per call including the final synchronisation (what the GPU front end sustains)
    Prints one JSON line."""
    import torch

    import paper_2510_00932_amd as opal

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the kernels have no CPU fallback", file=sys.stderr)
        sys.exit(2)
    lib = opal.load()
    n = 64
    a = torch.ones(n, dtype=torch.float64, device="cuda:0")
    b = torch.ones(n, dtype=torch.float64, device="cuda:0")
    c = torch.zeros(n, dtype=torch.float64, device="cuda:0")
    ws = torch.zeros(16, dtype=torch.float64, device="cuda:0")
    res = torch.zeros(1, dtype=torch.float64, device="cuda:0")
    stream = torch.cuda.Stream()
    hs = stream.cuda_stream
    pa, pb, pc, pws, pres = a.data_ptr(), b.data_ptr(), c.data_ptr(), ws.data_ptr(), res.data_ptr()
    # the raw ctypes entry points: no Python-side marshalling beyond ctypes' own
    cases = (("opal_copy", lambda: lib.opal_copy(pa, pc, n, 0, hs), 1),
             ("opal_triad", lambda: lib.opal_triad(pa, pb, pc, 0.4, n, 0, hs), 1),
             ("opal_dot", lambda: lib.opal_dot(pa, pb, n, 0, pws, 128, pres, hs), 2),
             ("opal_dot_static", lambda: lib.opal_dot_static(pa, pb, n, 0, pres, hs), 2),
             ("opal_dot_workspace_bytes (no GPU work)", lambda: lib.opal_dot_workspace_bytes(n, 0), 0))
    calls = 20000
    results = []
    for name, fn, launches in cases:
        for _ in range(200):
            fn()
        stream.synchronize()
        t0 = time.perf_counter()
        for _ in range(256):              # short enough that the hardware queue never fills
            fn()
        t_enq = (time.perf_counter() - t0) / 256
        stream.synchronize()
        t0 = time.perf_counter()
        for _ in range(calls):
            fn()
        stream.synchronize()
        t_all = (time.perf_counter() - t0) / calls
        results.append({"call": name, "kernel_launches": launches, "enqueue_us": round(t_enq * 1e6, 2),
                        "drain_us": round(t_all * 1e6, 2)})
    print(json.dumps({"metric": "host cost per call through the C ABI (ctypes), arrays of 64 elements, 1 GPU",
                      "unit": "us", "calls": calls, "results": results}))


def placement_scan(args):
    """How the two launch shapes of the elementwise kernels depend on where the three arrays lie relative to each
    other.  The arrays (2^28 fp64 by default, random values: zero-filled arrays hide the effect) are carved out of
    one allocation at base + k * (array bytes + skew), k = 0, 1, 2, for a list of skews; copy (a -> c), add and triad
    are timed with the paced shapes on, on with the matched order of the second input starting from the opposite
    assumption about the address bits above a page, on without the matched order, and off (average of `--steps`
    launches each, percent of the HBM peak).
    Prints one JSON line."""
    import torch

    import opal_inputs as oi
    import paper_2510_00932_amd as opal

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the kernels have no CPU fallback", file=sys.stderr)
        sys.exit(2)
    opal.load()
    wl = oi.workload(args.workload)
    n = args.n if args.n is not None else wl.n
    dt, tdt, item = (opal.OPAL_F64, torch.float64, 8) if wl.dtype == "f64" else (opal.OPAL_F32, torch.float32, 4)
    skews = [int(v) for v in args.placement_scan.split(",")]
    if any(v < 0 or v % 256 for v in skews):
        print("bench.py: skews must be non-negative multiples of 256", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    nbytes = n * item
    pool = torch.empty(3 * (nbytes + max(skews)) + 256, dtype=torch.uint8, device=dev)
    src = [torch.from_numpy(x).to(dev) for x in oi.make_arrays(wl, n=n, threads=min(16, os.cpu_count() or 1))]
    stream = torch.cuda.Stream()
    steps = max(3, min(args.steps, 20))
    rows = []
    mode0 = opal.opal_get_pacing()
    try:
        for skew in skews:
            pitch = nbytes + skew
            a, b, c = (pool[k * pitch:k * pitch + nbytes].view(tdt) for k in range(3))
            for d, h in zip((a, b, c), src):
                d.copy_(h)
            torch.cuda.synchronize()
            pa, pb, pc = a.data_ptr(), b.data_ptr(), c.data_ptr()
            row = {"skew_bytes": skew}
            for mode, label in ((1, "paced"), (1, "paced_other_start"), (1, "paced_same_order"), (0, "ordered")):
                opal.opal_set_pacing(mode)
                opal.opal_set_matched_order({"paced_same_order": 0, "paced_other_start": 2}.get(label, 1))
                for name, launch, moved in (("copy", lambda: opal.opal_copy(pa, pc, n, dt, stream), 2 * nbytes),
                                            ("add", lambda: opal.opal_add(pa, pb, pc, n, dt, stream), 3 * nbytes),
                                            ("triad", lambda: opal.opal_triad(pa, pb, pc, wl.s, n, dt, stream), 3 * nbytes)):
                    for _ in range(4):   # the launches in which the library times both orders of the second input
                        launch()
                    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
                    for e0, e1 in ev:
                        e0.record(stream)
                        launch()
                        e1.record(stream)
                    stream.synchronize()
                    avg_ms = sum(e0.elapsed_time(e1) for e0, e1 in ev) / steps
                    row["%s_%s" % (name, label)] = round(100 * moved / (avg_ms * 1e-3) / (HBM_PEAK_GBS * 1e9), 1)
            rows.append(row)
            print("bench.py: skew %d done" % skew, file=sys.stderr, flush=True)
    finally:
        opal.opal_set_pacing(mode0)
        opal.opal_set_matched_order(True)
    print(json.dumps({"metric": "percent of the HBM peak against the relative placement of the arrays, 1 GPU", "unit": "%",
                      "config": {"workload": wl.name, "n": n}, "dtype": wl.dtype, "data": "synthetic",
                      "launches_per_figure": steps, "results": rows}))


def lds_bench(args):
    """LDS-streaming microkernel (the analogue of the shared-memory benchmark subject of the paper's
    Table 1, rep = 300..1500, default 600): achieved LDS bandwidth = 32 bytes per 16-byte vector per
    round / time.  Peak used: 256 compute units x 128 bytes per clock x 2.4 GHz = 78.6 TB/s (derived
    from unit counts and clock, not a published figure).  Prints one JSON line."""
    import numpy as np
    import torch

    import opal_inputs as oi
    import paper_2510_00932_amd as opal

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the kernels have no CPU fallback", file=sys.stderr)
        sys.exit(2)
    opal.load()
    per_clk_cu = 256 * 2.4e9                 # bytes per second of one byte per clock per compute unit at 2.4 GHz
    results = []
    checks = []
    stream = torch.cuda.Stream()
    for dtype_name, dt, tdt, npdt in (("f32", opal.OPAL_F32, torch.float32, np.float32),
                                      ("f64", opal.OPAL_F64, torch.float64, np.float64)):
        te = opal.opal_lds_tile_elements(dt)
        tiles = 256 * 5 * 8                     # eight full waves of resident workgroups (5 per compute unit)
        n = tiles * te
        host = oi.uniform_array(42, 0, n, npdt, 0.5, 1.5)
        x = torch.from_numpy(host).cuda()
        y = torch.empty_like(x)
        torch.cuda.synchronize()
        for rep in ((args.lds_rep,) if args.lds_rep else (300, 600, 900, 1200, 1500)):
            for _ in range(2):
                opal.opal_lds_stream(x, y, 0.4, n, rep, dt, stream)
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
            for e0, e1 in ev:
                e0.record(stream)
                opal.opal_lds_stream(x, y, 0.4, n, rep, dt, stream)
                e1.record(stream)
            stream.synchronize()
            ms = sorted(e0.elapsed_time(e1) for e0, e1 in ev)
            avg = sum(ms) / len(ms)
            lds_bytes = 32.0 * (n * x.element_size() / 16) * rep
            results.append({"dtype": dtype_name, "n": n, "rep": rep, "avg_us": round(avg * 1e3, 1),
                            "min_us": round(ms[0] * 1e3, 1), "lds_GBps_avg": round(lds_bytes / avg / 1e6, 0),
                            "lds_bytes_per_clk_per_cu": round(lds_bytes / (avg * 1e-3) / per_clk_cu, 1)})
        if not args.no_cpu_baseline:
            import oracle
            m = 64 * te
            want = np.zeros(m, npdt)
            t0 = time.perf_counter()
            oracle.lds_stream(host[:m].copy(), want, 0.4, 600)
            t_cpu = time.perf_counter() - t0
            got = torch.empty(m, dtype=tdt, device="cuda")
            opal.opal_lds_stream(x[:m], got, 0.4, m, 600, dt, stream)
            stream.synchronize()
            bits = np.uint64 if dtype_name == "f64" else np.uint32
            checks.append({"dtype": dtype_name, "n": m, "rep": 600,
                           "bit_exact": bool(np.array_equal(got.cpu().numpy().view(bits), want.view(bits))),
                           "oracle_GBps": round(32.0 * (m * host.itemsize / 16) * 600 / t_cpu / 1e9, 2)})
    out = {"metric": "achieved LDS GB/s of the LDS-streaming microkernel, 1 GPU", "unit": "GB/s", "n_gpus": 1,
           "steps": args.steps, "data": "synthetic",
           # No fraction: the only published LDS figure of this chip is for reads (256 bytes per clock per compute
           # unit); what a half-read, half-write round can reach is measured by shape_study's read-only and
           # write-only variants of this kernel (group lds), not assumed.
           "roofline": {"bound": "lds", "peak": None, "unit": "GB/s",
                        "achieved": max(r["lds_GBps_avg"] for r in results), "frac": None,
                        "bytes_per_clk_per_cu_at_2.4GHz": max(r["lds_bytes_per_clk_per_cu"] for r in results)},
           "results": results, "cpu_baseline": {"kind": "oracle", "cores": 1, "checks": checks}}
    print(json.dumps(out))
    if any(not c["bit_exact"] for c in checks):
        print("bench.py: LDS kernel differs from the oracle", file=sys.stderr)
        sys.exit(1)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="n2p28_f64", help="name or index of a workload in opal_inputs.WORKLOADS")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing and the result check")
    ap.add_argument("--cpu-steps", type=int, default=2, help="oracle passes to time (the minimum is reported)")
    ap.add_argument("--n", type=int, default=None, help="override the workload's element count")
    ap.add_argument("--offset-elems", type=str, default=None,
                    help="override the workload's misalignment (elements past a 256-byte boundary): one number "
                         "for all three arrays, or a,b,c for one each")
    ap.add_argument("--skew-bytes", type=int, default=1024,
                    help="extra bytes between the starts of consecutive arrays beyond the array size (the arrays "
                         "are carved out of one allocation at base + k * (array bytes + skew), k = 0, 1, 2)")
    ap.add_argument("--paper-shapes", action="store_true",
                    help="instead of the roofline benchmark, time the paper's own (small, cache-resident) array "
                         "sizes and repetition counts issued eagerly and through HIP graphs")
    ap.add_argument("--placement-scan", default=None, metavar="SKEW[,SKEW...]",
                    help="instead of the roofline benchmark, time copy, add and triad with the paced shapes on and off "
                         "for each of these skews (bytes between consecutive arrays beyond the array size)")
    ap.add_argument("--lds-rep", type=int, default=0,
                    help="with --lds: time this repetition count only (default: the paper's five, 300..1500)")
    ap.add_argument("--call-overhead", action="store_true",
                    help="instead of the roofline benchmark, time the host cost of one call through the C ABI")
    ap.add_argument("--lds", action="store_true",
                    help="instead of the roofline benchmark, time the LDS-streaming microkernel (rep = 300..1500)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain torch copy of 1 GiB (a kernel of known traffic, for scaling "
                         "FETCH_SIZE / WRITE_SIZE counter readings)")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path is single-GPU by construction (no sharding, no collectives); "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.paper_shapes:
        paper_shapes(args)
        return
    if args.lds:
        lds_bench(args)
        return
    if args.call_overhead:
        call_overhead(args)
        return
    if args.placement_scan:
        placement_scan(args)
        return

    import numpy as np
    import torch

    import opal_inputs as oi
    import paper_2510_00932_amd as opal

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the kernels have no CPU fallback", file=sys.stderr)
        sys.exit(2)
    opal.load()
    from paper_2510_00932_amd import build as lib_build
    assert not lib_build.is_stale(), "libopal.so does not match the sources in this tree"

    wl = oi.workload(int(args.workload) if args.workload.isdigit() else args.workload)
    offsets = None
    if args.offset_elems is not None:
        offsets = [int(x) for x in args.offset_elems.split(",")]
        offsets = offsets * 3 if len(offsets) == 1 else offsets
        if len(offsets) != 3 or min(offsets) < 0:
            print("bench.py: --offset-elems takes one or three non-negative integers", file=sys.stderr)
            sys.exit(2)
    if args.n is not None or offsets is not None:
        import dataclasses
        wl = dataclasses.replace(wl, name=wl.name + "_custom", n=wl.n if args.n is None else args.n,
                                 offset_elems=wl.offset_elems if offsets is None else max(offsets))
    if offsets is None:
        offsets = [wl.offset_elems] * 3
    n, item = wl.n, wl.itemsize
    dt = opal.OPAL_F64 if wl.dtype == "f64" else opal.OPAL_F32
    tdt = torch.float64 if wl.dtype == "f64" else torch.float32
    dev = torch.device("cuda:0")

    # Inputs: generated on the host, copied once into HBM before anything is timed.
    host = oi.make_arrays(wl, threads=min(16, os.cpu_count() or 1))
    off = wl.offset_elems
    if args.skew_bytes % 256 != 0 or args.skew_bytes < 0:
        print("bench.py: --skew-bytes must be a non-negative multiple of 256", file=sys.stderr)
        sys.exit(2)
    pitch = ((n + off) * item + 255) // 256 * 256 + args.skew_bytes      # bytes from one array's base to the next
    pool = torch.empty(3 * pitch + 256, dtype=torch.uint8, device=dev)
    assert pool.data_ptr() % 256 == 0
    a, b, c = (pool[k * pitch + o * item:k * pitch + (o + n) * item].view(tdt) for k, o in zip(range(3), offsets))
    for d, h in zip((a, b, c), host):
        d.copy_(torch.from_numpy(h))
    ws_bytes = opal.opal_dot_workspace_bytes(n, dt)
    ws = torch.empty(ws_bytes // 8, dtype=torch.float64, device=dev)
    res = torch.empty(1, dtype=torch.float64, device=dev)
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()

    pa, pb, pc = a.data_ptr(), b.data_ptr(), c.data_ptr()
    pws, pres = ws.data_ptr(), res.data_ptr()
    s = wl.s

    launches = (
        lambda: opal.opal_copy(pa, pc, n, dt, stream),
        lambda: opal.opal_scale(pb, pc, s, n, dt, stream),
        lambda: opal.opal_add(pa, pb, pc, n, dt, stream),
        lambda: opal.opal_triad(pa, pb, pc, s, n, dt, stream),
        lambda: opal.opal_dot(pa, pb, n, dt, pws, ws_bytes, pres, stream),
    )

    def step(events=None):
        for k, launch in enumerate(launches):
            if events is not None:
                events[k][0].record(stream)
            launch()
            if events is not None:
                events[k][1].record(stream)

    # First step on the pristine inputs: its results are what the oracle check compares.
    step()
    stream.synchronize()
    first = {"a": a.cpu().numpy(), "b": b.cpu().numpy(), "c": c.cpu().numpy(), "dot": float(res.item())} \
        if not args.no_cpu_baseline else None

    for _ in range(max(0, args.warmup - 1)):
        step()
    stream.synchronize()
    torch.cuda.synchronize()

    K = args.steps
    events = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in KERNELS]
              for _ in range(K)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        step(events[i])
    stream.synchronize()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K

    if args.calibration_copy:
        src = torch.empty(1 << 27, dtype=torch.float64, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    bpe = [opal.opal_bytes_per_element(k, dt) for k in range(5)]
    step_bytes = sum(bpe) * n
    kernels = {}
    for k, name in enumerate(KERNELS):
        ms = [events[i][k][0].elapsed_time(events[i][k][1]) for i in range(K)]
        nbytes = bpe[k] * n
        avg, mn, med = sum(ms) / K, min(ms), statistics.median(ms)
        kernels[name] = {
            "bytes": nbytes, "avg_us": round(avg * 1e3, 2), "min_us": round(mn * 1e3, 2),
            "median_us": round(med * 1e3, 2),
            "GBps_avg": round(nbytes / avg / 1e6, 1), "GBps_best": round(nbytes / mn / 1e6, 1),
            "GBps_median": round(nbytes / med / 1e6, 1),
            "frac_of_peak_avg": round(nbytes / avg / 1e6 / HBM_PEAK_GBS, 4),
            "launches_over_1.03x_median": sum(1 for t in ms if t > 1.03 * med),
        }
    # The kernel with the largest share of the step; add and triad move the same bytes and tie to
    # within noise, so a tie (1 %) goes to triad, which also does the most arithmetic.
    longest = max(kernels[name]["avg_us"] for name in KERNELS)
    dominant = "triad" if kernels["triad"]["avg_us"] >= 0.99 * longest else \
        max(KERNELS, key=lambda name: kernels[name]["avg_us"])
    dk = kernels[dominant]
    roofline = {
        "kernel": dominant, "bound": "hbm", "achieved": dk["GBps_avg"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(dk["GBps_avg"] / HBM_PEAK_GBS, 4),
        "traffic": measured_traffic(wl.name, dominant),
        "algorithmic_bytes_per_launch": dk["bytes"], "avg_launch_us": dk["avg_us"],
    }

    out = {
        "metric": "achieved HBM GB/s per kernel (copy/scale/add/triad/dot) and % of peak, 1 GPU",
        "value": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "unit": "GB/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "n": n, "elem_bytes": item, "scalar": s,
                   "offset_elems": offsets, "array_pitch_bytes": pitch, "seed": wl.seed, "value_range": [wl.lo, wl.hi],
                   "step": "copy,scale,add,triad,dot once each", "bytes_per_step": step_bytes},
        "frac_of_hbm_peak": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "kernels": kernels,
        "roofline": roofline,
        "library": {"source_digest": lib_build.source_digest(), "kernel_source_digest": kernel_source_digest(),
                    "pacing_mode": opal.opal_get_pacing()},
    }

    if not args.no_cpu_baseline:
        import oracle
        ha, hb, hc = host
        times = []
        state = None
        for rep in range(max(1, args.cpu_steps)):
            xa, xb, xc = ha.copy(), hb.copy(), hc.copy()
            t0 = time.perf_counter()
            oracle.copy(xa, xc)
            oracle.scale(xb, xc, s)
            oracle.add(xa, xb, xc)
            oracle.triad(xa, xb, xc, s)
            r = oracle.dot(xa, xb)
            times.append(time.perf_counter() - t0)
            state = (xa, xb, xc, r)
        best = min(times)
        out["cpu_baseline"] = {
            "value": round(step_bytes / best / 1e9, 2), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "the full workload (n=%d), one step = the same five kernels, best of %d passes, "
                      "single thread; host has %d logical cores" % (n, len(times), os.cpu_count() or 0),
            "ms_per_step": round(best * 1e3, 1),
        }
        xa, xb, xc, r = state
        bits = np.uint64 if wl.dtype == "f64" else np.uint32
        exact = all(np.array_equal(first[k].view(bits), x.view(bits)) for k, x in (("a", xa), ("b", xb), ("c", xc)))
        rel = abs(first["dot"] - r) / abs(r) if r != 0 else abs(first["dot"])
        out["check_vs_oracle"] = {"elementwise_bit_exact": bool(exact), "dot_rel_err": float("%.3e" % rel),
                                  "dot_tolerance": 1e-12 if wl.dtype == "f64" else 1e-5}

    print(json.dumps(out))
    if "check_vs_oracle" in out:
        ok = out["check_vs_oracle"]["elementwise_bit_exact"] and \
            out["check_vs_oracle"]["dot_rel_err"] <= out["check_vs_oracle"]["dot_tolerance"]
        if not ok:
            print("bench.py: GPU results differ from the oracle", file=sys.stderr)
            sys.exit(1)


if __name__ == "__main__":
    main()
