"""Summarise rocprofv3 CSV output of a bench.py run into the text kept under profiles/.

    python -m paper_2311_09431_amd.profsum [--kt DIR] [--fetch DIR] [--write DIR] [--sq DIR] [--sq2 DIR] [--prefix P]

Each DIR is the `-d` folder of one rocprofv3 run of `python bench.py ...` made with
`--output-format csv -o P`:
  --kt     `--kernel-trace --stats`              (P_kernel_stats.csv)
  --fetch  `--pmc FETCH_SIZE`                     (P_counter_collection.csv)
  --write  `--pmc WRITE_SIZE`
  --sq     `--pmc SQ_... GRBM_GUI_ACTIVE`         (any counters; listed per kernel)
  --sq2    a second counter pass of the same kind (one run holds at most 8 SQ counters)
With --kt and --sq it also prints one DERIVED line per matrix-core kernel: clock, matrix-core
busy share, instructions per MFMA and (with --sq2) the wait shares of a wavefront's cycles.
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


# MI355X: 8 XCDs (GRBM_GUI_ACTIVE is summed over them), 256 CUs x 4 SIMDs; one
# v_mfma_f32_32x32x16_bf16 is 2 x 32 x 32 x 16 flop
_XCDS, _SIMDS, _MFMA_FLOP = 8, 1024, 32768


def derived_lines(kt_dir, prefix, sq, sq2):
    avg_ns = {_short(r["Name"]): float(r["AverageNs"]) for r in
              csv.DictReader(open(_find(kt_dir, prefix, "_kernel_stats.csv")))}
    mean = lambda v, c: sum(v[c]) / len(v[c]) if c in v else None
    out = ["", "derived per matrix-core kernel (kernel-trace average duration; clock = GRBM_GUI_ACTIVE / %d XCDs / "
               "duration; busy = SQ_VALU_MFMA_BUSY_CYCLES / (%d SIMDs x GRBM_GUI_ACTIVE / %d); executed = "
               "SQ_INSTS_MFMA x %d flop / duration; waits = share of SQ_WAVE_CYCLES)" % (_XCDS, _SIMDS, _XCDS, _MFMA_FLOP)]
    for k, v in sq.items():
        n_mfma, grbm = mean(v, "SQ_INSTS_MFMA"), mean(v, "GRBM_GUI_ACTIVE")
        if not n_mfma or not grbm or k not in avg_ns:
            continue
        ns = avg_ns[k]
        line = "DERIVED %-66s avg_ms=%7.3f executed_TFLOPs=%6.0f clock_GHz=%.2f" % (
            (re.search(r"\w+<[^>]*>", k) or re.search(r".*", k)).group(0)[:66], ns / 1e6, n_mfma * _MFMA_FLOP / ns / 1e3, grbm / _XCDS / ns)
        busy, coex = mean(v, "SQ_VALU_MFMA_BUSY_CYCLES"), mean(v, "SQ_VALU_MFMA_COEXEC_CYCLES")
        if busy:
            line += " mfma_busy=%.0f%%" % (100 * busy / (_SIMDS * grbm / _XCDS))
            if coex:
                line += " valu_coexec=%.0f%%" % (100 * coex / busy)
        valu, trans, lds = mean(v, "SQ_INSTS_VALU"), mean(v, "SQ_INSTS_VALU_TRANS_F32"), mean(v, "SQ_INSTS_LDS")
        if valu and trans is not None and lds:
            line += " per_mfma: valu=%.2f exp=%.2f lds=%.2f" % ((valu - n_mfma - trans) / n_mfma, trans / n_mfma,
                                                              lds / n_mfma)
        w = sq2.get(k) if sq2 else None
        if w and mean(w, "SQ_WAVE_CYCLES"):
            wc = mean(w, "SQ_WAVE_CYCLES")
            for tag, c in (("s_waitcnt", "SQ_WAIT_ANY"), ("issue_wait", "SQ_WAIT_INST_ANY"),
                           ("lds_issue_wait", "SQ_WAIT_INST_LDS")):
                if mean(w, c) is not None:
                    line += " %s=%.0f%%" % (tag, 100 * mean(w, c) / wc)
        out.append(line)
    return out


def main():
    ap = argparse.ArgumentParser()
    for a in ("kt", "fetch", "write", "sq", "sq2"):
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
    sq = counters(args.sq, args.prefix) if args.sq else None
    sq2 = counters(args.sq2, args.prefix) if args.sq2 else None
    if sq is not None:
        out += counter_table("sq", sq)
    if sq2 is not None:
        out += counter_table("sq2", sq2)
    if args.kt and sq is not None:
        out += derived_lines(args.kt, args.prefix, sq, sq2)
    print("\n".join(out))


if __name__ == "__main__":
    main()
