#!/usr/bin/env python3
"""Roofline position of the streaming kernels from rocprofv3 output: observed against peak,
component by component, with the under-used components named.

This is the analytic half of the paper's AMD branch (Section 3.2.1: the vendor tools give only
numbers per memory level and operation type, so under-utilised components are found by comparing
observed and peak values), applied to this library's own kernels and without the LLM.

    python3 paper_2510_00932_amd/roofline_report.py <dir> [--n N] [--dtype f64|f32]

<dir> is searched recursively for rocprofv3 CSV files written with --output-format csv:
  *_kernel_stats.csv        from  rocprofv3 --kernel-trace --stats -- python3 bench.py ...
  *_counter_collection.csv  from  rocprofv3 --pmc <counters> -- python3 bench.py ... [--calibration-copy]
Any subset of counters may be present; lines whose counters are missing are left out.

Peaks (MI355X): HBM 8.0 TB/s and vector fp64 78.6 / fp32 157.3 TFLOP/s are published; the cache
levels are derived from unit counts, widths per clock and the 2.4 GHz peak clock: L2 = 8 XCDs x 16
channels x 128 B/clk = 39.3 TB/s; L1 (vector cache to L2 and to the compute unit) = 256 compute
units x 64 B/clk = 39.3 TB/s.  The LDS has a published figure for reads only (256 B/clk per compute
unit on CDNA 4, twice the 128 B/clk of CDNA 3, which was one figure for reads and writes); its lines are
given in bytes per clock per compute unit against that read figure and against the rates that read-only
and write-only variants of the same kernel reach (shape_study, group lds).
"""
import argparse
import csv
import glob
import os
import sys

HBM_PEAK = 8.0e12
VALU_PEAK = {"f64": 78.6e12, "f32": 157.3e12}
CLOCK_HZ = 2.4e9
L2_PEAK = 8 * 16 * 128 * CLOCK_HZ       # bytes per second
L1_PEAK = 256 * 64 * CLOCK_HZ
LDS_READ_PEAK_B_PER_CLK_CU = 256.0                       # published, CDNA 4, reads
# measured with shape_study's read-only and write-only variants of the LDS kernel (same tile, same launch)
LDS_MEASURED_B_PER_CLK_CU = {"read": 209.0, "write": 77.0}
CAL_KERNEL = "__amd_rocclr_copyBuffer"
CAL_BYTES = 1 << 30

# name, substrings of the kernel's symbol, algorithmic bytes per element in units of the element size, flops per
# element.  The elementwise kernels and dot's first pass exist in an index-ordered / tiled and a paced form; a run
# uses one of them per workload.
KERNELS = (
    ("copy", ("stream_kernel", "(opal::Op)0"), 2, 0),
    ("scale", ("stream_kernel", "(opal::Op)1"), 2, 1),
    ("add", ("stream_kernel", "(opal::Op)2"), 3, 1),
    ("triad", ("stream_kernel", "(opal::Op)3"), 3, 2),
    ("dot", ("dot_", "_kernel<"), 2, 2),
)
LDS_KERNEL = ("lds_stream_kernel",)


def find(root, suffix):
    return sorted(glob.glob(os.path.join(root, "**", "*" + suffix), recursive=True))


def read_kernel_stats(root):
    """{kernel symbol: (calls, average ns)} from every *_kernel_stats.csv under root (later files win)."""
    out = {}
    for path in find(root, "_kernel_stats.csv"):
        with open(path) as f:
            for row in csv.DictReader(f):
                out[row["Name"]] = (int(row["Calls"]), float(row["AverageNs"]))
    return out


def read_counters(root):
    """{counter: {kernel symbol: average value per dispatch}} from every *_counter_collection.csv under root."""
    acc = {}
    for path in find(root, "_counter_collection.csv"):
        with open(path) as f:
            for row in csv.DictReader(f):
                acc.setdefault(row["Counter_Name"], {}).setdefault(row["Kernel_Name"], []).append(float(row["Counter_Value"]))
    return {c: {k: sum(v) / len(v) for k, v in per.items()} for c, per in acc.items()}


def pick(table, needles):
    if isinstance(needles, str):
        needles = (needles,)
    hits = [v for k, v in table.items() if all(x in k for x in needles)]
    return hits[0] if len(hits) == 1 else None


def analyse(root, n, dtype):
    """Returns a list of (kernel name, {metric: value}) and a list of report lines."""
    width = 8 if dtype == "f64" else 4
    stats = read_kernel_stats(root)
    counters = read_counters(root)

    def ctr(name, needle):
        return pick(counters.get(name, {}), needle)

    fetch_unit = write_unit = None
    cal_f, cal_w = ctr("FETCH_SIZE", CAL_KERNEL), ctr("WRITE_SIZE", CAL_KERNEL)
    if cal_f:
        fetch_unit = CAL_BYTES / cal_f
    if cal_w:
        write_unit = CAL_BYTES / cal_w

    results, lines = [], []
    for name, needle, words, flops in KERNELS:
        m = {}
        st = pick(stats, needle)
        alg_bytes = words * width * n
        m["algorithmic_bytes"] = alg_bytes
        if st:
            calls, avg_ns = st
            t = avg_ns * 1e-9
            if name == "dot":
                final = pick(stats, "dot_final_kernel")
                if final:
                    t += final[1] * 1e-9
            m["seconds"] = t
            m["hbm_bytes_per_s"] = alg_bytes / t
            m["hbm_frac"] = alg_bytes / t / HBM_PEAK
            m["valu_frac"] = flops * n / t / VALU_PEAK[dtype]
            m["intensity"] = flops / (words * width)
        f, w = ctr("FETCH_SIZE", needle), ctr("WRITE_SIZE", needle)
        if f is not None and w is not None and fetch_unit and write_unit:
            m["hbm_traffic_bytes"] = f * fetch_unit + w * write_unit
            m["traffic_over_algorithmic"] = m["hbm_traffic_bytes"] / alg_bytes
        req, hit = ctr("TCC_REQ_sum", needle), ctr("TCC_HIT_sum", needle)
        if req and hit is not None:
            m["l2_hit_rate"] = hit / req
        busy = ctr("TCC_BUSY_sum", needle)
        for key, cname in (("ea_write_stall_frac", "TCC_EA0_WRREQ_STALL_sum"),
                           ("ea_read_credit_stall_frac", "TCC_EA0_RDREQ_DRAM_CREDIT_STALL_sum"),
                           ("l2_tag_stall_frac", "TCC_TAG_STALL_sum")):
            v = ctr(cname, needle)
            if v is not None and busy:
                m[key] = v / busy
        rd, rdlat = ctr("TCP_TCC_READ_REQ_sum", needle), ctr("TCP_TCC_READ_REQ_LATENCY_sum", needle)
        if rd and rdlat:
            m["read_latency_cycles"] = rdlat / rd
        wr, wrlat = ctr("TCP_TCC_WRITE_REQ_sum", needle), ctr("TCP_TCC_WRITE_REQ_LATENCY_sum", needle)
        if wr and wrlat:
            m["write_latency_cycles"] = wrlat / wr
        tlb_req, tlb_miss = ctr("TCP_UTCL1_REQUEST_sum", needle), ctr("TCP_UTCL1_TRANSLATION_MISS_sum", needle)
        if tlb_req and tlb_miss is not None:
            m["tlb_miss_rate"] = tlb_miss / tlb_req
        # traffic per cache level, from request counts (the request size is what the counters cannot tell: it is
        # inferred from the algorithmic bytes, which every level moves exactly once in these kernels)
        if "seconds" in m:
            l2req = ctr("TCC_REQ_sum", needle)
            if l2req:
                m["l2_bytes_per_request"] = alg_bytes / l2req
                m["l2_bytes_per_s"] = alg_bytes / m["seconds"]
                m["l2_frac"] = m["l2_bytes_per_s"] / L2_PEAK
            l1rd, l1wr = ctr("TCP_TCC_READ_REQ_sum", needle), ctr("TCP_TCC_WRITE_REQ_sum", needle)
            if l1rd is not None and l1wr is not None and (l1rd + l1wr) > 0:
                m["l1_l2_bytes_per_request"] = alg_bytes / (l1rd + l1wr)
                m["l1_bytes_per_s"] = alg_bytes / m["seconds"]
                m["l1_frac"] = m["l1_bytes_per_s"] / L1_PEAK
            acc, cacc = ctr("TCP_TOTAL_ACCESSES_sum", needle), ctr("TCP_TOTAL_CACHE_ACCESSES_sum", needle)
            if acc:
                m["l1_accesses"] = acc
                m["l1_bytes_per_access"] = alg_bytes / acc
            if cacc is not None:
                m["l1_cache_accesses"] = cacc
        waves, wave_cycles = ctr("SQ_WAVES", needle), ctr("SQ_WAVE_CYCLES", needle)
        if waves and wave_cycles:
            m["wave_lifetime_cycles"] = 4.0 * wave_cycles / waves     # the counter ticks once per four cycles
        results.append((name, m))

    lines.append("Roofline position, n = %d %s (peaks: HBM %.1f TB/s, vector %s %.1f TFLOP/s)"
                 % (n, dtype, HBM_PEAK / 1e12, dtype, VALU_PEAK[dtype] / 1e12))
    for name, m in results:
        lines.append("")
        lines.append("%s" % name)
        if "seconds" in m:
            lines.append("  time per launch %.1f us; algorithmic bytes %.0f -> %.0f GB/s = %.1f %% of the HBM peak"
                         % (m["seconds"] * 1e6, m["algorithmic_bytes"], m["hbm_bytes_per_s"] / 1e9, 100 * m["hbm_frac"]))
            ridge = VALU_PEAK[dtype] / HBM_PEAK
            lines.append("  arithmetic intensity %.3f flop/byte (ridge at %.1f): vector ALU at %.3f %% of its peak"
                         % (m["intensity"], ridge, 100 * m["valu_frac"]))
        if "traffic_over_algorithmic" in m:
            lines.append("  HBM traffic (FETCH_SIZE + WRITE_SIZE, calibrated) = %.4f x algorithmic bytes"
                         % m["traffic_over_algorithmic"])
        if "l2_frac" in m:
            lines.append("  L2: %.0f GB/s = %.1f %% of its %.1f TB/s peak (%.0f bytes per L2 request)"
                         % (m["l2_bytes_per_s"] / 1e9, 100 * m["l2_frac"], L2_PEAK / 1e12, m["l2_bytes_per_request"]))
        if "l1_frac" in m:
            lines.append("  L1 (vector cache to L2): %.0f GB/s = %.1f %% of its %.1f TB/s peak (%.0f bytes per request to L2)"
                         % (m["l1_bytes_per_s"] / 1e9, 100 * m["l1_frac"], L1_PEAK / 1e12, m["l1_l2_bytes_per_request"]))
        if "l1_bytes_per_access" in m:
            lines.append("  L1 accesses: %.0f per launch, %.0f algorithmic bytes each" % (m["l1_accesses"], m["l1_bytes_per_access"]))
        if "l2_hit_rate" in m:
            note = " (hits are the second 64-byte half of a freshly allocated write line)" if m["l2_hit_rate"] > 0.01 else ""
            lines.append("  L2 hit rate %.1f %%%s" % (100 * m["l2_hit_rate"], note))
        for key, text in (("ea_write_stall_frac", "L2-to-fabric write requests stalled (no DRAM credit)"),
                          ("ea_read_credit_stall_frac", "L2-to-fabric read requests stalled (no DRAM credit)"),
                          ("l2_tag_stall_frac", "L2 tag pipeline stalled")):
            if key in m:
                lines.append("  %s: %.1f %% of L2 channel-busy cycles" % (text, 100 * m[key]))
        if "read_latency_cycles" in m:
            lines.append("  mean L1-to-L2 read latency %.0f cycles (%.2f us)"
                         % (m["read_latency_cycles"], m["read_latency_cycles"] / CLOCK_HZ * 1e6))
        if "write_latency_cycles" in m:
            lines.append("  mean L1-to-L2 write latency %.0f cycles" % m["write_latency_cycles"])
        if "tlb_miss_rate" in m:
            lines.append("  L1 TLB miss rate %.4f %%" % (100 * m["tlb_miss_rate"]))
        if "wave_lifetime_cycles" in m:
            lines.append("  mean wavefront lifetime %.0f cycles" % m["wave_lifetime_cycles"])
        lines.extend("  => " + v for v in verdicts(m))
    return results, lines


def lds_composed_rate(read=None, write=None):
    """Bytes per clock per compute unit of a round that reads and writes the same number of bytes when reads run at
    `read` and writes at `write` bytes per clock and share one pipe (the times add)."""
    read = LDS_MEASURED_B_PER_CLK_CU["read"] if read is None else read
    write = LDS_MEASURED_B_PER_CLK_CU["write"] if write is None else write
    return 2.0 / (1.0 / read + 1.0 / write)


def analyse_lds(root, n, dtype, rep):
    """The LDS microkernel: observed LDS bandwidth (32 bytes per 16-byte vector per round, from the definition) per
    compute unit and clock, against the published read rate and the measured read-only and write-only rates."""
    stats = read_kernel_stats(root)
    counters = read_counters(root)
    width = 8 if dtype == "f64" else 4
    needle = LDS_KERNEL + (("double" if dtype == "f64" else "float"),)
    st = pick(stats, needle)
    if not st:
        return []
    t = st[1] * 1e-9
    lds_bytes = 32.0 * (n * width / 16) * rep
    rate = lds_bytes / t / 256 / CLOCK_HZ                      # bytes per clock per compute unit, read + written
    composed = lds_composed_rate()
    lines = ["", "lds_stream (n = %d %s, rep = %d)" % (n, dtype, rep),
             "  time per launch %.1f us; LDS traffic by definition %.3e bytes -> %.0f GB/s"
             % (t * 1e6, lds_bytes, lds_bytes / t / 1e9),
             "  per compute unit and clock at 2.4 GHz: %.1f bytes (%.1f read + %.1f written)" % (rate, rate / 2, rate / 2),
             "  reads alone: %.1f %% of the published %.0f B/clk/CU read rate" % (100 * rate / 2 / LDS_READ_PEAK_B_PER_CLK_CU,
                                                                              LDS_READ_PEAK_B_PER_CLK_CU),
             "  measured ceilings of the same kernel: read-only %.0f, write-only %.0f B/clk/CU; reads and writes share one "
             "pipe, so a round at those rates moves %.1f B/clk/CU: the kernel is at %.0f %% of that"
             % (LDS_MEASURED_B_PER_CLK_CU["read"], LDS_MEASURED_B_PER_CLK_CU["write"], composed, 100 * rate / composed)]
    conf, idx = pick(counters.get("SQ_LDS_BANK_CONFLICT", {}), needle), pick(counters.get("SQ_LDS_IDX_ACTIVE", {}), needle)
    insts = pick(counters.get("SQ_INSTS_LDS", {}), needle)
    if conf is not None and idx:
        lines.append("  LDS bank conflicts: %.2f %% of LDS-active cycles" % (100 * conf / idx))
    if idx:
        lines.append("  LDS index unit active %.0f %% of the kernel's cycles%s"
                     % (100 * idx / (256 * t * CLOCK_HZ),
                        (", %.1f cycles per LDS instruction (a 16-byte read and a 16-byte write per lane in turn)" % (idx / insts))
                        if insts else ""))
    frac = rate / composed
    lines.append("  => the LDS %s; its read path is under-used (%.0f %% of the published read rate) because the writes of "
                 "every round hold the pipe for %.0f %% of the time; HBM carries only one read and one write of the tile "
                 "(%.3f %% of its peak)"
                 % ("write rate is the binding component (the kernel runs at what the measured read-only and write-only "
                    "rates compose to)" if frac >= 0.9 else
                    "is under-used (%.0f %% of what the measured read-only and write-only rates compose to)" % (100 * frac),
                    100 * rate / 2 / LDS_READ_PEAK_B_PER_CLK_CU,
                    100 * (1.0 / LDS_MEASURED_B_PER_CLK_CU["write"]) /
                    (1.0 / LDS_MEASURED_B_PER_CLK_CU["write"] + 1.0 / LDS_MEASURED_B_PER_CLK_CU["read"]),
                    100 * 2 * n * width / t / HBM_PEAK))
    return lines


def verdicts(m):
    """Observed against peak, component by component: which one binds, which are under-used."""
    out = []
    if "hbm_frac" in m:
        if m["hbm_frac"] >= 0.80:
            out.append("HBM is the binding component (%.0f %% of peak); the vector ALU and LDS are idle by construction "
                       "(intensity far left of the ridge), so only fewer bytes or better DRAM efficiency can help"
                       % (100 * m["hbm_frac"]))
        else:
            out.append("HBM is under-used (%.0f %% of peak) although the kernel is memory-bound by intensity: "
                       "look at launch shape, in-flight requests and access order" % (100 * m["hbm_frac"]))
    for key, what in (("l2_frac", "L2"), ("l1_frac", "L1")):
        if key in m and m[key] < 0.5:
            out.append("%s is under-used (%.0f %% of its peak): every byte passes through it once, nothing is reused, "
                       "so it can only ever carry the HBM rate" % (what, 100 * m[key]))
    if m.get("traffic_over_algorithmic", 1.0) > 1.02:
        out.append("HBM moves %.1f %% more than the algorithm needs: re-reads or partial-line writes"
                   % (100 * (m["traffic_over_algorithmic"] - 1)))
    elif "traffic_over_algorithmic" in m:
        out.append("no wasted traffic: every byte moved is an algorithmic byte")
    if m.get("ea_write_stall_frac", 0.0) > 0.10:
        out.append("the write path is the tighter side: %.0f %% of L2 cycles wait for DRAM write credits"
                   % (100 * m["ea_write_stall_frac"]))
    if m.get("tlb_miss_rate", 0.0) > 0.01:
        out.append("address translation misses are frequent (%.2f %%): the access window is too wide" % (100 * m["tlb_miss_rate"]))
    return out


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("dir")
    ap.add_argument("--n", type=int, default=1 << 28)
    ap.add_argument("--dtype", choices=("f64", "f32"), default="f64")
    ap.add_argument("--lds-n", type=int, default=0, help="element count of the LDS microkernel launches in the run (0: none)")
    ap.add_argument("--lds-rep", type=int, default=600)
    args = ap.parse_args()
    _, lines = analyse(args.dir, args.n, args.dtype)
    if args.lds_n:
        lines += analyse_lds(args.dir, args.lds_n, args.dtype, args.lds_rep)
    print("\n".join(lines))


if __name__ == "__main__":
    sys.exit(main())
