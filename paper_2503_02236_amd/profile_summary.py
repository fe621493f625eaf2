"""Turn rocprofv3 CSV output into the short text summaries kept under profiles/.

  python -m paper_2503_02236_amd.profile_summary stats <kernel_stats.csv> <out.md> --cmd "<command>" [--note "..."]
  python -m paper_2503_02236_amd.profile_summary traffic <fetch_counter_collection.csv> <write_counter_collection.csv>
         <out.md> --cmd "<command>" [--copy-bytes N]

  python -m paper_2503_02236_amd.profile_summary counters <out.md> <counter_collection.csv>... --kernel <substring>...
         --title "..." --cmd "<command>" [--note "..."]

`counters` writes, for every kernel whose name contains one of the substrings, the average per dispatch of every counter
found in the given files (one file per counter run).

`traffic` expects two counter runs of `bench.py --pmc-probe` (one with FETCH_SIZE, one with
WRITE_SIZE; both counters are in KiB per dispatch).  The probe run starts with plain copies of
a known size; the ratio counter / known bytes of those copies is the calibration factor every
other reading is divided by.  The per-launch figure is the sum over all gemv kernels of the
pass (main kernels + their reduction kernels) divided by the number of main-kernel dispatches.
"""
from __future__ import annotations

import argparse
import collections
import csv
import subprocess


def _short(name: str) -> str:
    try:
        name = subprocess.run(["c++filt", name], capture_output=True, text=True).stdout.strip() or name
    except OSError:
        pass
    return name.split("(")[0][-90:]


def stats(args):
    rows = list(csv.DictReader(open(args.src)))
    with open(args.out, "w") as f:
        f.write("# rocprofv3 kernel-trace summary\n\ncommand: `%s`\n\n%s\n\n" % (args.cmd, args.note))
        f.write("| kernel | calls | avg us | min us | max us | total ms | % |\n|---|---|---|---|---|---|---|\n")
        for r in rows:
            if float(r["Percentage"]) < 0.05:
                continue
            f.write("| %s | %s | %.2f | %.2f | %.2f | %.3f | %.2f |\n" % (
                _short(r["Name"]), r["Calls"], float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3,
                float(r["MaxNs"]) / 1e3, float(r["TotalDurationNs"]) / 1e6, float(r["Percentage"])))


def _per_kernel(path, counter):
    agg = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == counter:
            agg[_short(r["Kernel_Name"])].append(float(r["Counter_Value"]) * 1024.0)  # KiB -> bytes
    return agg


def traffic(args):
    fetch = _per_kernel(args.fetch, "FETCH_SIZE")
    write = _per_kernel(args.write, "WRITE_SIZE")
    copy_name = next(k for k in fetch if "probe_copy" in k)
    f_cal = sum(fetch[copy_name]) / len(fetch[copy_name]) / args.copy_bytes
    w_cal = sum(write[copy_name]) / len(write[copy_name]) / args.copy_bytes
    kernels = sorted(k for k in fetch if "gemv_packed" in k or "gemv_pipeline" in k)
    mains = [k for k in kernels if "finalize" not in k]         # one dispatch of these per launch of the stack
    n = sum(len(fetch[k]) for k in mains)
    rd = sum(sum(fetch[k]) for k in kernels) / n / f_cal
    wr = sum(sum(write[k]) for k in kernels) / n / w_cal
    with open(args.out, "w") as f:
        f.write("# HBM traffic of the vq_gemv launches of the C2 stack (rocprofv3 --pmc)\n\ncommands (one run per counter):\n`%s`\n\n"
                % args.cmd)
        f.write("Calibration on vq_probe_copy of %d bytes: FETCH_SIZE reads %.4f x, WRITE_SIZE %.4f x the known size.\n"
                "Readings below are divided by these factors.\n\n" % (args.copy_bytes, f_cal, w_cal))
        f.write("| kernel | dispatches | read bytes / dispatch | written bytes / dispatch |\n|---|---|---|---|\n")
        for k in kernels:
            f.write("| %s | %d | %.0f | %.0f |\n" % (k, len(fetch[k]), sum(fetch[k]) / len(fetch[k]) / f_cal,
                                                    sum(write[k]) / len(write[k]) / w_cal))
        f.write("\nper launch (main kernel + its share of the reduction kernels: a vq_gemv / vq_gemv_batch call, or with "
                "vq_gemv_pipeline the whole pass), average over the %d main-kernel launches of one pass over the "
                "32-block stack:\n\n" % n)
        f.write("read_bytes_per_launch: %.0f\nwritten_bytes_per_launch: %.0f\ntraffic_bytes_per_launch: %.0f\n"
                % (rd, wr, rd + wr))


def counters(args):
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for path in args.src:
        per = collections.defaultdict(lambda: collections.defaultdict(float))   # (kernel, dispatch) -> counter -> sum over units
        for r in csv.DictReader(open(path)):
            if any(k in r["Kernel_Name"] for k in args.kernel):
                per[(_short(r["Kernel_Name"]), r["Dispatch_Id"])][r["Counter_Name"]] += float(r["Counter_Value"])
        for (k, _), cs in per.items():
            for c, v in cs.items():
                agg[k][c].append(v)
    with open(args.out, "w") as f:
        f.write("# %s\n\ncommands (one run per counter set):\n`%s`\n\n%s\n\n" % (args.title, args.cmd, args.note))
        for k in sorted(agg):
            n = max(len(v) for v in agg[k].values())
            f.write("## %s (%d dispatches; average per dispatch, summed over the chip)\n\n| counter | value |\n|---|---|\n" % (k, n))
            for c in sorted(agg[k]):
                f.write("| %s | %.0f |\n" % (c, sum(agg[k][c]) / len(agg[k][c])))
            f.write("\n")


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="mode", required=True)
    a = sub.add_parser("stats")
    a.add_argument("src")
    a.add_argument("out")
    a.add_argument("--cmd", required=True)
    a.add_argument("--note", default="")
    a.set_defaults(fn=stats)
    b = sub.add_parser("traffic")
    b.add_argument("fetch")
    b.add_argument("write")
    b.add_argument("out")
    b.add_argument("--cmd", required=True)
    b.add_argument("--copy-bytes", type=int, default=256 << 20)
    b.set_defaults(fn=traffic)
    c = sub.add_parser("counters")
    c.add_argument("out")
    c.add_argument("src", nargs="+")
    c.add_argument("--kernel", required=True, nargs="+")
    c.add_argument("--title", required=True)
    c.add_argument("--cmd", required=True)
    c.add_argument("--note", default="")
    c.set_defaults(fn=counters)
    args = ap.parse_args()
    args.fn(args)


if __name__ == "__main__":
    main()
