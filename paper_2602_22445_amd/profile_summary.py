"""Short text summaries of rocprofv3 runs of bench.py.

  python -m paper_2602_22445_amd.profile_summary stats   <kernel_stats.csv> <out.txt> --command "<cmd>" [--bench-line FILE]
  python -m paper_2602_22445_amd.profile_summary traffic <fetch counter_collection.csv> <write counter_collection.csv> <out.txt>
                                                         --command "<cmd>" --copy-bytes N

`traffic` turns two counter runs (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch)
of `bench.py --calibrate-copy` into HBM bytes per launch of every kernel.  Each
counter is scaled by what it reads for the plain copy of N bytes that
--calibrate-copy adds to the run (the largest __amd_rocclr_copyBuffer dispatch).
The file ends with machine-readable `traffic` lines and the hash of the kernel
sources they were taken with; bench.py reports such a figure only while the
sources still have that hash.
"""
import argparse
import collections
import csv
import hashlib
import os
import re

HERE = os.path.dirname(os.path.abspath(__file__))


def source_hash():
    """sha256 over the HIP sources and headers of the library, in name order."""
    h = hashlib.sha256()
    d = os.path.join(HERE, "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".h", ".hip")):
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()


def short_name(kernel):
    k = kernel.replace("(anonymous namespace)::", "").replace("void ", "")
    m = re.match(r"([A-Za-z_0-9:]+)(<[^(]*>)?", k)
    name = m.group(1) if m else k
    return name.split("::")[-1]


def read_traffic(path):
    """{kernel: bytes per launch} and the source hash of a file written by `traffic`."""
    out, sha = {}, None
    for line in open(path):
        p = line.split()
        if len(p) >= 3 and p[0] == "traffic":
            out[p[1]] = float(dict(q.split("=") for q in p[2:])["hbm_bytes_per_launch"])
        if len(p) == 2 and p[0] == "source_sha256":
            sha = p[1]
    return out, sha


def _per_kernel(path, counter):
    agg = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] == counter:
            agg[short_name(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return agg


def cmd_traffic(a):
    fetch = _per_kernel(a.fetch_csv, "FETCH_SIZE")
    write = _per_kernel(a.write_csv, "WRITE_SIZE")
    copy = "__amd_rocclr_copyBuffer"
    f_fac = a.copy_bytes / (max(fetch[copy]) * 1024.0)
    w_fac = a.copy_bytes / (max(write[copy]) * 1024.0)
    with open(a.out, "w") as fh:
        fh.write("HBM traffic per kernel launch from rocprofv3 counters: allreduce P=16384 f=4 elems=8xf64 S=4096 "
                 "(bench.py workload), one MI355X\n")
        fh.write("commands (run from the repository root; cd /tmp && export TMPDIR=/tmp first), one counter per run:\n")
        for c in ("FETCH_SIZE", "WRITE_SIZE"):
            fh.write("  " + a.command.replace("COUNTER", c) + "\n")
        fh.write("source: counter_collection.csv of the two runs; KiB per dispatch, averaged over the dispatches of a kernel\n")
        fh.write("calibration: the plain copy of %d bytes (largest __amd_rocclr_copyBuffer dispatch) reads FETCH_SIZE = "
                 "%.1f KiB, WRITE_SIZE = %.1f KiB\n  => FETCH_SIZE x %.4f, WRITE_SIZE x %.4f give bytes\n\n"
                 % (a.copy_bytes, max(fetch[copy]), max(write[copy]), f_fac, w_fac))
        fh.write("%-22s %8s %16s %16s %18s\n" % ("kernel", "launches", "FETCH_SIZE KiB", "WRITE_SIZE KiB", "HBM bytes/launch"))
        lines = []
        for k in fetch:
            if k == copy or k not in write:
                continue
            fk = sum(fetch[k]) / len(fetch[k])
            wk = sum(write[k]) / len(write[k])
            total = fk * 1024.0 * f_fac + wk * 1024.0 * w_fac
            fh.write("%-22s %8d %16.1f %16.1f %18.0f\n" % (k, len(fetch[k]), fk, wk, total))
            lines.append("traffic %s hbm_bytes_per_launch=%.0f fetch_bytes=%.0f write_bytes=%.0f\n"
                         % (k, total, fk * 1024.0 * f_fac, wk * 1024.0 * w_fac))
        fh.write("\n")
        fh.writelines(lines)
        fh.write("source_sha256 %s\n" % source_hash())


def cmd_stats(a):
    rows = list(csv.DictReader(open(a.stats_csv)))
    with open(a.out, "w") as fh:
        fh.write("rocprofv3 kernel-trace summary: allreduce P=16384 f=4 elems=8xf64 S=4096 (bench.py workload), one MI355X\n")
        fh.write("command (run from the repository root; cd /tmp && export TMPDIR=/tmp first):\n  " + a.command + "\n")
        fh.write("source: kernel_stats.csv of that run (warm-up and timed steps together)\n\n")
        fh.write("%-46s %6s %14s %12s %7s\n" % ("kernel", "calls", "total_ns", "avg_ns", "pct"))
        for r in rows:
            name = r["Name"].replace("(anonymous namespace)::", "").split("(")[0].replace("void ", "")
            fh.write("%-46s %6s %14s %12.0f %7s\n" % (name[:46], r["Calls"], r["TotalDurationNs"], float(r["AverageNs"]),
                                                     r["Percentage"]))
        if a.bench_line:
            fh.write("\nbench.py line of the same build (HIP events inside bench.py, no profiler):\n"
                     + open(a.bench_line).read().strip() + "\n")


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="what", required=True)
    s = sub.add_parser("stats")
    s.add_argument("stats_csv")
    s.add_argument("out")
    s.add_argument("--command", required=True)
    s.add_argument("--bench-line")
    s.set_defaults(fn=cmd_stats)
    t = sub.add_parser("traffic")
    t.add_argument("fetch_csv")
    t.add_argument("write_csv")
    t.add_argument("out")
    t.add_argument("--command", required=True, help="the rocprofv3 command, with COUNTER for the counter name")
    t.add_argument("--copy-bytes", type=int, required=True)
    t.set_defaults(fn=cmd_traffic)
    a = ap.parse_args()
    a.fn(a)


if __name__ == "__main__":
    main()
