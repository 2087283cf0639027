"""Turns the raw output of rocprofv3 runs of bench.py into the short text summaries kept under profiles/.

It runs nothing on the GPU: it reads the SQLite databases rocprofv3 wrote (`-d <dir>`), keeps the dispatches of the
MAIN phase of the bench run (set-up decode steps are cut off: bench.py polls the status word once between set-up and
warm-up, and the second `clear_status_kernel` dispatch of the process marks that point), attributes every library
kernel to its kernel class (the O and down projections share kernel instantiations and are told apart by what ran
before them in the layer), and prints

  * the kernel trace of the main phase (calls, total, average, min, max per kernel),
  * FETCH_SIZE / WRITE_SIZE per dispatch, scaled to bytes by the plain 256 MiB device copy of --copy-calibration,
  * any further counter passes (--pmc), averaged per kernel,
  * one `traffic <class> <fetched bytes> <written bytes>` line per kernel class: bench.py reads these for
    `roofline.traffic` (HBM bytes per launch of the class).

Typical use, one workload (every run from /tmp with TMPDIR=/tmp; W = workload name):
  rocprofv3 --kernel-trace --stats -d OUT/kt -o kt -- python3 bench.py --config W --no-sub --no-cpu-baseline
  rocprofv3 --pmc FETCH_SIZE -d OUT/fetch -o f -- python3 bench.py --config W --no-sub --no-cpu-baseline --steps 3 --warmup 1 --copy-calibration
  rocprofv3 --pmc WRITE_SIZE -d OUT/write -o w -- python3 bench.py --config W --no-sub --no-cpu-baseline --steps 3 --warmup 1 --copy-calibration
  python3 -m paper_2605_08862_amd.profile_summary --workload W --kt OUT/kt --fetch OUT/fetch --write OUT/write \\
          --bench-log OUT/kt.log > profiles/W_kernels.txt
"""
import argparse
import glob
import json
import re
import sqlite3
import sys

CLASS_ORDER = ["attention", "gemm_qkv", "gemm_o", "gemm_gate_up", "gemm_down", "lmhead"]
CALIBRATION_KIB = 262144.0          # the 256 MiB copy of bench.py --copy-calibration


def _db(directory):
    files = glob.glob(directory + "/**/*_results.db", recursive=True)
    if not files:
        sys.exit("profile_summary: no *_results.db under %s" % directory)
    return sqlite3.connect(files[0])


def classify(names):
    """names: kernel names in dispatch order -> list of classes (None: not a roofline class)."""
    out, marker = [], None
    for n in names:
        cls = None
        if "attn_mfma_kernel" in n or "attn_wide_kernel" in n or "attn_wide_merge_kernel" in n:
            cls, marker = "attention", "attention"
        elif "qkv_rope_kernel" in n:
            cls = "gemm_qkv"
        elif "gemm8_kernel" in n or "gemm_ring2_swiglu_kernel" in n or re.search(r"gemm_mfma_kernelILi\dELi\dELi2E", n):
            cls, marker = "gemm_gate_up", "gate_up"
        elif "gemm_resid_kernel" in n or re.search(r"gemm_mfma_kernelILi\dELi\dELi1E", n):
            cls = "gemm_down" if marker == "gate_up" else "gemm_o"
        elif re.search(r"gemm_mfma_kernelILi\dELi\dELi3E", n):
            cls = "gemm_qkv"                                   # unfused QKV projection (head sizes other than 128)
        elif re.search(r"lmhead_kernelILi\dELb1E", n):
            cls = "lmhead"
        out.append(cls)
    return out


def main_phase(rows, name_col):
    """Drops everything up to and including the second clear_status_kernel dispatch (context creation, then the
    poll between set-up and warm-up)."""
    seen = 0
    for i, r in enumerate(rows):
        if "clear_status_kernel" in r[name_col]:
            seen += 1
            if seen == 2:
                return rows[i + 1:]
    return rows


def short(name, width=100):
    return name if len(name) <= width else name[:width - 1] + "~"


def kernel_trace(directory, lines):
    c = _db(directory)
    rows = c.execute("select dispatch_id, name, (end - start) / 1e3 from kernels order by dispatch_id").fetchall()
    rows = main_phase(rows, 1)
    classes = classify([r[1] for r in rows])
    agg, per_class = {}, {}
    for (did, name, us), cls in zip(rows, classes):
        a = agg.setdefault(name, [0, 0.0, 1e30, 0.0, cls])
        a[0] += 1
        a[1] += us
        a[2] = min(a[2], us)
        a[3] = max(a[3], us)
        if cls:
            pc = per_class.setdefault(cls, {})
            k = pc.setdefault(name, [0, 0.0])
            k[0] += 1
            k[1] += us
    total = sum(a[1] for a in agg.values())
    lines.append("== kernel trace, main phase (warm-up, timed steps and the per-class event passes; durations in us) ==")
    lines.append("%-100s %-12s %7s %12s %9s %9s %9s %6s" % ("kernel", "class", "calls", "total_us", "avg_us", "min_us", "max_us", "pct"))
    for name, a in sorted(agg.items(), key=lambda kv: -kv[1][1])[:40]:
        if name.startswith("void at::") or "at::native" in name:
            continue                                             # torch's own kernels (state reset, event passes' copies)
        lines.append("%-100s %-12s %7d %12.1f %9.2f %9.2f %9.2f %6.2f" % (short(name), a[4] or "-", a[0], a[1], a[1] / a[0], a[2], a[3],
                                                                          100 * a[1] / total))
    return per_class


def counter_names(directory):
    return [r[0] for r in _db(directory).execute("select distinct counter_name from counters_collection order by counter_name")]


def counter_pass(directory, lines, title=None):
    c = _db(directory)
    rows = c.execute("select dispatch_id, kernel_name, counter_name, value from counters_collection order by dispatch_id").fetchall()
    # calibration copy: the first large plain copy of the process
    cal = {}
    for did, name, cn, v in rows:
        if "copyBuffer" in name and v > 60000 and cn not in cal:
            cal[cn] = v
    by_dispatch = {}
    for did, name, cn, v in rows:
        by_dispatch.setdefault(did, [name, {}])[1][cn] = v
    ordered = [(did, by_dispatch[did][0], by_dispatch[did][1]) for did in sorted(by_dispatch)]
    ordered = main_phase(ordered, 1)
    classes = classify([r[1] for r in ordered])
    agg, per_class = {}, {}
    for (did, name, vals), cls in zip(ordered, classes):
        a = agg.setdefault(name, [0, {}, cls])
        a[0] += 1
        for cn, v in vals.items():
            a[1][cn] = a[1].get(cn, 0.0) + v
        if cls:
            pc = per_class.setdefault(cls, [0, {}])
            pc[0] += 1
            for cn, v in vals.items():
                pc[1][cn] = pc[1].get(cn, 0.0) + v
    counters = sorted({cn for a in agg.values() for cn in a[1]})
    lines.append("")
    lines.append("== %s: average per dispatch, main phase ==" % (title or " ".join(counters)))
    lines.append("%-100s %-12s %7s " % ("kernel", "class", "calls") + " ".join("%18s" % cn[:18] for cn in counters))
    for name, a in sorted(agg.items(), key=lambda kv: -kv[1][0] * max(kv[1][1].values() or [0])):
        if name.startswith("void at::") or "at::native" in name:
            continue
        lines.append("%-100s %-12s %7d " % (short(name), a[2] or "-", a[0]) + " ".join("%18.1f" % (a[1].get(cn, 0.0) / a[0]) for cn in counters))
    derived_rates(c, ordered, classes, lines)
    return {cls: {cn: v / n for cn, v in vals.items()} for cls, (n, vals) in per_class.items()}, cal


N_XCD, N_CU, N_SIMD = 8, 256, 1024


def derived_rates(c, ordered, classes, lines):
    """Rates that follow from a pass which holds GRBM_GUI_ACTIVE (cycles with the GPU busy, summed over the 8 XCDs)
    next to unit-busy counters: shader clock = GUI_ACTIVE / 8 / dispatch duration, unit busy shares = busy cycles /
    (units x GUI_ACTIVE / 8)."""
    if not ordered or "GRBM_GUI_ACTIVE" not in ordered[0][2]:
        return
    dur = dict(c.execute("select dispatch_id, end - start from kernels").fetchall())
    agg = {}
    for (did, name, vals), cls in zip(ordered, classes):
        if not cls or did not in dur:
            continue
        a = agg.setdefault((name, cls), [cls, 0, 0.0, {}])
        a[1] += 1
        a[2] += dur[did]
        for cn, v in vals.items():
            a[3][cn] = a[3].get(cn, 0.0) + v
    lines.append("")
    lines.append("== derived per kernel (main phase): duration in this pass, shader clock = GRBM_GUI_ACTIVE / 8 / duration, busy shares ==")
    lines.append("%-60s %-12s %9s %9s %11s %9s %9s %12s" % ("kernel", "class", "avg_us", "clock_GHz", "MFMA_busy_%", "TA_busy_%", "L2_hit_%", "L2->L1_GB"))
    seen_cls = {}
    for (name, _), (cls, n, ns, v) in sorted(agg.items(), key=lambda kv: -kv[1][2]):
        if ns / n < 20e3:
            continue                                             # too short for the busy-cycle counter to mean a clock
        cyc = v["GRBM_GUI_ACTIVE"] / N_XCD
        f = lambda num, units: ("%.1f" % (100.0 * v[num] / (units * cyc))) if num in v and cyc else "-"
        hit = ("%.1f" % (100.0 * v["TCC_HIT_sum"] / (v["TCC_HIT_sum"] + v["TCC_MISS_sum"]))) if "TCC_HIT_sum" in v and "TCC_MISS_sum" in v else "-"
        l2l1 = ("%.3f" % (v["TCP_TCC_READ_REQ_sum"] * 128.0 / n / 1e9)) if "TCP_TCC_READ_REQ_sum" in v else "-"
        lines.append("%-60s %-12s %9.1f %9.2f %11s %9s %9s %12s" % (short(name, 60), cls, ns / n / 1e3, cyc / ns if ns else 0.0,
                                                                   f("SQ_VALU_MFMA_BUSY_CYCLES", N_SIMD), f("TA_TA_BUSY_sum", N_CU), hit, l2l1))
        if cls not in seen_cls and "SQ_VALU_MFMA_BUSY_CYCLES" in v:      # the longest kernel of the class; read by bench.py
            seen_cls[cls] = "derived %s %.3f %.4f" % (cls, cyc / ns, v["SQ_VALU_MFMA_BUSY_CYCLES"] / (N_SIMD * cyc))
    if seen_cls:
        lines.append("")
        lines.append("== per kernel class: shader clock (GHz) and matrix-unit busy share of its main kernel; read by bench.py ==")
        lines.extend(seen_cls[c] for c in CLASS_ORDER if c in seen_cls)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", required=True)
    ap.add_argument("--kt", help="directory of the --kernel-trace run")
    ap.add_argument("--fetch", help="directory of the --pmc FETCH_SIZE run (with --copy-calibration)")
    ap.add_argument("--write", help="directory of the --pmc WRITE_SIZE run (with --copy-calibration)")
    ap.add_argument("--pmc", action="append", default=[], help="directory of a further counter pass (repeatable)")
    ap.add_argument("--bench-log", help="stdout of the kernel-trace run (its JSON line is quoted)")
    ap.add_argument("--bench-args", default="", help="further bench.py arguments every pass was run with (e.g. '--layers 2')")
    ap.add_argument("--note", action="append", default=[], help="free text for the header (repeatable)")
    args = ap.parse_args()
    lines = ["rocprofv3 summary of bench.py --config %s (one MI355X), written by paper_2605_08862_amd/profile_summary.py." % args.workload,
             "Only the main phase of each run is counted (set-up steps are cut off).  Commands, each run from /tmp with",
             "TMPDIR=/tmp and bench.py given by its path in the checkout:"]
    b = "python3 bench.py --config %s --no-sub --no-cpu-baseline" % args.workload + (" " + args.bench_args if args.bench_args else "")
    if args.kt:
        lines.append("  rocprofv3 --kernel-trace --stats -d OUT/kt -o kt -- %s" % b)
    if args.fetch:
        lines.append("  rocprofv3 --pmc FETCH_SIZE -d OUT/fetch -o f -- %s --steps 3 --warmup 1 --copy-calibration" % b)
    if args.write:
        lines.append("  rocprofv3 --pmc WRITE_SIZE -d OUT/write -o w -- %s --steps 3 --warmup 1 --copy-calibration" % b)
    for directory in args.pmc:
        lines.append("  rocprofv3 --pmc %s -d OUT/pmc -o p -- %s --steps 3 --warmup 1" % (" ".join(counter_names(directory)), b))
    lines.append("  python3 -m paper_2605_08862_amd.profile_summary --workload %s ... (the directories above) > this file" % args.workload)
    lines += args.note
    bench = None
    if args.bench_log:
        for l in open(args.bench_log):
            if l.startswith('{"metric"'):
                bench = json.loads(l)
    if bench:
        ro = bench["roofline"]
        lines.append("")
        lines.append("Bench line of the kernel-trace run: %.3f ms per step (median %.3f), %.0f emitted tokens/s, %.1f rows per step;"
                     % (bench["ms_per_step"], bench["verify_step_latency_ms"], bench["value"], bench["config"]["rows_per_step"]))
        lines.append("dominant class %s: %.1f us per launch by HIP events, %.1f %% of the peak of %.0f %s (%s bound)."
                     % (ro["kernel"], ro["us_per_launch"], 100 * ro["frac"], ro["peak"], ro["unit"], ro["bound"]))
    per_class_kt = {}
    body = []
    if args.kt:
        per_class_kt = kernel_trace(args.kt, body)
    traffic = {}
    for directory, cn in ((args.fetch, "FETCH_SIZE"), (args.write, "WRITE_SIZE")):
        if not directory:
            continue
        per_class, cal = counter_pass(directory, body, cn + " (KiB as reported)")
        factor = CALIBRATION_KIB / cal[cn] if cn in cal else float("nan")
        lines.append("Calibration: the plain 256 MiB device copy (262144 KiB read and written) reports %s = %.0f, so bytes = %.3f x %s KiB."
                     % (cn, cal.get(cn, float("nan")), factor, cn))
        for cls, vals in per_class.items():
            traffic.setdefault(cls, {})[cn] = vals.get(cn, 0.0) * 1024.0 * factor
    for directory in args.pmc:
        counter_pass(directory, body)
    if bench and per_class_kt:
        lines.append("")
        lines.append("HIP-event duration per launch of every class (event-pair overhead %.1f us subtracted) next to the rocprofv3 average"
                     % ro["event_pair_overhead_us"])
        lines.append("of the same dispatches (a class with two kernels per launch, e.g. attention + its merge, lists both):")
        for cls in CLASS_ORDER:
            kc = bench["kernel_classes"].get(cls)
            if not kc or cls not in per_class_kt:
                continue
            prof = " + ".join("%.2f us %s" % (t / n, re.sub(r"^_Z\d+", "", nm)[:34]) for nm, (n, t) in
                              sorted(per_class_kt[cls].items(), key=lambda kv: -kv[1][1]))
            lines.append("  %-13s events %8.1f us (%s roofline fraction %.1f %%)   rocprofv3: %s"
                         % (cls, kc["us_per_launch"], kc["bound"], 100 * kc["frac_of_peak"], prof))
    out = lines + [""] + body
    if traffic:
        out.append("")
        out.append("== HBM traffic per launch of each kernel class (bytes; fetched, written); read by bench.py ==")
        for cls in CLASS_ORDER:
            if cls in traffic:
                # a class with several kernels per launch (attention + merge): counters are per dispatch, so scale
                # the per-dispatch average by the dispatches per launch
                n_per_launch = 1.0
                if cls in per_class_kt and bench and cls in bench["kernel_classes"]:
                    calls = sum(n for n, _ in per_class_kt[cls].values())
                    main_kernel_calls = max(n for n, _ in per_class_kt[cls].values())
                    n_per_launch = calls / main_kernel_calls
                out.append("traffic %s %.0f %.0f" % (cls, traffic[cls].get("FETCH_SIZE", 0.0) * n_per_launch,
                                                     traffic[cls].get("WRITE_SIZE", 0.0) * n_per_launch))
    print("\n".join(out))


if __name__ == "__main__":
    main()
