"""Summarise rocprofv3 CSV output of a bench.py run into the text kept under profiles/.

    python -m paper_2311_09431_amd.profsum [--kt DIR] [--fetch DIR] [--write DIR] [--sq DIR] [--prefix P]

Each DIR is the `-d` folder of one rocprofv3 run of `python bench.py ...` made with
`--output-format csv -o P`:
  --kt     `--kernel-trace --stats`              (P_kernel_stats.csv)
  --fetch  `--pmc FETCH_SIZE`                     (P_counter_collection.csv)
  --write  `--pmc WRITE_SIZE`
  --sq     `--pmc SQ_... GRBM_GUI_ACTIVE`         (any counters; listed per kernel)
Prints the per-kernel tables and, when both byte counters are there, one line per library
kernel that bench.py parses:
    TRAFFIC <kernel> read_GB=<x> written_GB=<y>
for the triangular-step instantiation of each matrix-core kernel.  FETCH_SIZE / WRITE_SIZE
are KiB per dispatch; they are scaled by what the same counters read for permute_kernel, a
plain copy that reads and writes its tensor once (bytes read = bytes written, and WRITE_SIZE
matches the tensor size on this hardware), so the fetch factor is WRITE(copy) / FETCH(copy).
Holds no attention arithmetic and runs nothing on the GPU.
"""
import argparse
import collections
import csv
import glob
import os
import re


def _find(d, prefix, suffix):
    hits = glob.glob(os.path.join(d, "**", prefix + suffix), recursive=True)
    if not hits:
        raise SystemExit("no %s%s under %s" % (prefix, suffix, d))
    return hits[0]


def _short(name):
    if "at::" in name:
        return "torch: " + name.split("<")[0][:60]
    return name[:96]


def kernel_stats(d, prefix):
    out = ["kernel-trace stats (Name, Calls, TotalDurationNs, AverageNs, Percentage, MinNs, MaxNs)"]
    for r in csv.DictReader(open(_find(d, prefix, "_kernel_stats.csv"))):
        out.append("%-96s calls=%4s total_ms=%9.3f avg_us=%10.1f pct=%6s min_us=%9.1f max_us=%9.1f" % (
            _short(r["Name"]), r["Calls"], float(r["TotalDurationNs"]) / 1e6, float(r["AverageNs"]) / 1e3,
            r["Percentage"], float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3))
    return out


def counters(d, prefix):
    """{kernel: {counter: [values per dispatch]}} without torch's kernels."""
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(_find(d, prefix, "_counter_collection.csv"))):
        if "at::" in r["Kernel_Name"]:
            continue
        agg[_short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return agg


def counter_table(tag, agg):
    out = ["", "pmc pass '%s': per kernel, counter: launches, mean, min, max" % tag]
    for k, v in agg.items():
        for c, vals in sorted(v.items()):
            out.append("%-96s %-26s n=%3d mean=%.6g min=%.6g max=%.6g" % (k, c, len(vals), sum(vals) / len(vals),
                                                                      min(vals), max(vals)))
    return out


# triangular-step instantiations: fwd / dq <RAGGED=false, FULL=false, ...>, dkdv <TRI=true, RAGGED=false, ...>
_TRI = {"fwd_mfma_kernel": "<false, false", "bwd_dq_mfma_kernel": "<false, false", "bwd_dkdv_mfma_kernel": "<true, false"}


def traffic_lines(fetch, write):
    mean = lambda agg, k, c: sum(agg[k][c]) / len(agg[k][c])
    copy = [k for k in fetch if "permute_kernel" in k and k in write]
    if not copy:
        return ["", "(no permute_kernel launches in the counter runs: FETCH_SIZE cannot be calibrated)"]
    f_copy, w_copy = mean(fetch, copy[0], "FETCH_SIZE"), mean(write, copy[0], "WRITE_SIZE")
    factor = w_copy / f_copy
    out = ["", "HBM bytes per launch (KiB counters; FETCH_SIZE x %.3f, the factor that makes the copy kernel's "
               "reads equal its %.4g KiB of writes)" % (factor, w_copy)]
    for kern, inst in _TRI.items():
        for k in fetch:
            if re.search(r"\b%s%s" % (kern, re.escape(inst)), k) and k in write:
                rd = mean(fetch, k, "FETCH_SIZE") * factor * 1024 / 1e9
                wr = mean(write, k, "WRITE_SIZE") * 1024 / 1e9
                out.append("TRAFFIC %s read_GB=%.3f written_GB=%.3f" % (kern, rd, wr))
                break
    return out


def main():
    ap = argparse.ArgumentParser()
    for a in ("kt", "fetch", "write", "sq"):
        ap.add_argument("--" + a)
    ap.add_argument("--prefix", default="p")
    args = ap.parse_args()
    out = []
    if args.kt:
        out += kernel_stats(args.kt, args.prefix)
    f = counters(args.fetch, args.prefix) if args.fetch else None
    w = counters(args.write, args.prefix) if args.write else None
    if f is not None:
        out += counter_table("fetch", f)
    if w is not None:
        out += counter_table("write", w)
    if f is not None and w is not None:
        out += traffic_lines(f, w)
    if args.sq:
        out += counter_table("sq", counters(args.sq, args.prefix))
    print("\n".join(out))


if __name__ == "__main__":
    main()
