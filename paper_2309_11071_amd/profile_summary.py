"""Turns rocprofv3 output of bench.py runs into the short summaries kept under profiles/.

    python -m paper_2309_11071_amd.profile_summary --kernel 'k_agg_events<false, 32>' \
        [--stats DIR_OR_CSV] [--pmc DIR_OR_CSV ...] [--top-frac 0.5]

--stats : output of `rocprofv3 --kernel-trace --stats` (the *_kernel_stats.csv file or its folder);
          if the per-dispatch *_kernel_trace.csv lies there too, the durations of the LARGE launches
          (see below) are listed as well, and with --window W K those of K large launches after
          the first W alone (bench.py runs its warm-up steps, then its timed steps, then other
          legs: W = --warmup and K = --steps select the launches whose HIP-event average bench.py
          prints as avg_launch_ms)
--pmc   : output of `rocprofv3 --pmc ...` runs (*_counter_collection.csv or folders), any number

Prints markdown: the duration table of the kernels that match --kernel, then per counter the
median over the LARGE launches of that kernel (those within --top-frac of the largest value of the
counter: bench.py launches the same kernel for every layer, and the roofline is about the launches
of the largest layer; the median because single batches are several times heavier than the rest).  If the runs were made with `bench.py --calibration`, the byte counters FETCH_SIZE and
WRITE_SIZE are also given for the calibration kernels of known size (a 1 GiB elementwise copy and
gathers of 2^21 rows of 192 B / 512 B / 1 KiB from a 4 GiB table), with the factor
known bytes / counter bytes that scales them.
"""
import argparse
import collections
import csv
import glob
import os
import sys

KIB = 1024.0
CAL_COPY = "elementwise_kernel"          # torch.mul(a, 1.0, out=b): reads 1 GiB, writes 1 GiB
CAL_GATHER = "vectorized_gather_kernel"  # torch.index_select on [rows][width] tables
CAL_GATHER_ROWS = 1 << 21
CAL_WIDTHS = (48, 128, 256)              # floats per row, in launch order


def find(path, pattern):
    if os.path.isfile(path):
        return [path]
    return sorted(glob.glob(os.path.join(path, "**", pattern), recursive=True))


def load_stats(path):
    rows = []
    for f in find(path, "*kernel_stats.csv"):
        rows += list(csv.DictReader(open(f)))
    return rows


def load_pmc(path):
    rows = []
    for f in find(path, "*counter_collection.csv"):
        rows += list(csv.DictReader(open(f)))
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--kernel", required=True, help="substring of the kernel name")
    ap.add_argument("--stats", default=None)
    ap.add_argument("--pmc", nargs="*", default=[])
    ap.add_argument("--top-frac", type=float, default=0.2)
    ap.add_argument("--window", type=int, nargs=2, default=None, metavar=("SKIP", "COUNT"),
                    help="also average COUNT large launches of the kernel trace after the first SKIP")
    args = ap.parse_args()
    out = []
    if args.stats:
        out.append("| kernel | calls | total ms | average us | min us | max us |")
        out.append("|---|---|---|---|---|---|")
        for r in load_stats(args.stats):
            if args.kernel in r["Name"]:
                out.append("| `%s` | %s | %.3f | %.1f | %.1f | %.1f |" % (
                    r["Name"].split("(")[0][:90], r["Calls"], float(r["TotalDurationNs"]) / 1e6,
                    float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3))
        out.append("")
        durs = []
        for f in find(args.stats, "*kernel_trace.csv"):
            for r in csv.DictReader(open(f)):
                if args.kernel in r["Kernel_Name"]:
                    durs.append((int(r["Start_Timestamp"]), (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6))
        if durs:
            durs.sort()
            longest = max(d for _, d in durs)
            in_order = [d for _, d in durs if d >= args.top_frac * longest]
            big = sorted(in_order)
            out.append("large launches (at least %.2f of the longest): %d of %d; average %.3f ms, median %.3f ms, min %.3f ms, max %.3f ms"
                       % (args.top_frac, len(big), len(durs), sum(big) / len(big), big[len(big) // 2], big[0], big[-1]))
            if args.window:
                part = in_order[args.window[0]:args.window[0] + args.window[1]]
                if part:
                    out.append("large launches %d .. %d in launch order (the timed steps): average %.3f ms, median %.3f ms"
                               % (args.window[0] + 1, args.window[0] + len(part), sum(part) / len(part), sorted(part)[len(part) // 2]))
            out.append("")
    for path in args.pmc:
        rows = load_pmc(path)
        per = collections.defaultdict(list)              # counter -> values of the matching kernel
        cal = collections.defaultdict(list)              # (counter, kind) -> values of calibration kernels
        for r in rows:
            name, cn, v = r["Kernel_Name"], r["Counter_Name"], float(r["Counter_Value"])
            if args.kernel in name:
                per[cn].append(v)
            elif CAL_COPY in name and "MulFunctor" in name and int(r["Grid_Size"]) >= (1 << 26):
                cal[(cn, "copy")].append(v)
            elif CAL_GATHER in name:
                cal[(cn, "gather")].append(v)
        out.append("from `%s`:" % os.path.basename(os.path.normpath(path)))
        out.append("")
        out.append("| counter | launches of the kernel | large launches | median of the large launches | max |")
        out.append("|---|---|---|---|---|")
        for cn, vals in sorted(per.items()):
            top = max(vals)
            big = [v for v in vals if v >= args.top_frac * top] if top > 0 else vals
            out.append("| %s | %d | %d | %.6g | %.6g |" % (cn, len(vals), len(big), sorted(big)[len(big) // 2], top))
        out.append("")
        for (cn, kind), vals in sorted(cal.items()):
            if cn not in ("FETCH_SIZE", "WRITE_SIZE"):
                continue
            if kind == "copy":
                known = float(1 << 30)
                for v in vals[-1:]:
                    out.append("calibration, elementwise copy (1 GiB read, 1 GiB written): %s = %.0f KiB -> factor %.3f"
                               % (cn, v, known / (v * KIB) if v else float("nan")))
            else:
                for w, v in zip(CAL_WIDTHS, vals[:len(CAL_WIDTHS)]):      # the calibration gathers come first in a run
                    known = float(CAL_GATHER_ROWS * w * 4)
                    out.append("calibration, gather of 2^21 rows of %d B (%s side %.0f MiB known): %s = %.0f KiB -> factor %.3f"
                               % (w * 4, "read" if cn == "FETCH_SIZE" else "write", known / (1 << 20), cn, v,
                                  known / (v * KIB) if v else float("nan")))
        out.append("")
    print("\n".join(out))


if __name__ == "__main__":
    sys.exit(main())
