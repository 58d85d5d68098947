#!/usr/bin/env python3
"""Benchmark of the Striped Attention ring step on one MI355X.

One bench "step" is one pass of the whole hot path for one device's share of the
ring under the STRIPED layout: stripe-permute Q/K/V, initialise (O, LSE), play
the device's N ring steps (forward; and backward when --bwd is on), and round
the result to bf16.  `value` is the useful causal TFLOP/s of that pass (only
unmasked query/key pairs count: 4*d flops each forward, 10*d backward) with
inputs resident in HBM.  The contiguous (Ring Attention) layout is timed beside
it for the worst-device step latencies the paper's argument is about (Sec. 1:
a round lasts as long as its slowest device).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3|cfg1|cfg2|cfg4|cfg5|3b|d64|d256|tiny]
                    [--bwd 0|1] [--cold] [--graph] [--skip-granularity BQxBK] [--kv-heads H_KV]

Prints one JSON line.
"""
import argparse
import json
import os
import statistics
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2311_09431_amd import binding as sa   # noqa: E402
from paper_2311_09431_amd import inputs           # noqa: E402

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
# kernels of each family, as rocprofv3 names them
FAMILIES = {
    "fwd": ("fwd ring step (fwd_mfma_kernel)", ("fwd_mfma_kernel",)),
    "bwd": ("bwd ring step (bwd_dq_mfma_kernel + bwd_dkdv_mfma_kernel)",
            ("bwd_dq_mfma_kernel", "bwd_dkdv_mfma_kernel")),
}


def measured_traffic(workload):
    """HBM bytes per launch of a triangular step, read from the committed rocprofv3 summary of
    this workload (profiles/ring_step_kernels_<workload>.txt): lines of the form
        TRAFFIC <kernel> read_GB=<x> written_GB=<y>
    written there from the FETCH_SIZE / WRITE_SIZE counter runs.  Returns {kernel: (read, written)};
    empty when there is no summary for the workload, so a stale figure is never reported."""
    path = os.path.join(ROOT, "profiles", "ring_step_kernels_%s.txt" % workload)
    out = {}
    try:
        with open(path) as f:
            for line in f:
                t = line.split()
                if len(t) == 4 and t[0] == "TRAFFIC" and t[2].startswith("read_GB=") and t[3].startswith("written_GB="):
                    out[t[1]] = (float(t[2].split("=")[1]), float(t[3].split("=")[1]))
    except (OSError, ValueError):
        return {}
    return out


# one device's share: the worst-loaded query device of both layouts is N-1
WORKLOADS = {
    "cfg3": dict(B=1, H=32, d=128, S=262144, N=8, q_dev=7,
                 desc="one device's share at 256k: B1 H32 d128 S262144 N8 (32768-token shards), "
                      "bf16, all 8 steps of q_dev 7"),
    "cfg2": dict(B=1, H=16, d=128, S=32768, N=8, q_dev=-1,
                 desc="forward ring sim: B1 H16 d128 S32768 N8 (4096-token shards), bf16, all 64 steps"),
    "cfg4": dict(B=1, H=16, d=128, S=131072, N=8, q_dev=7,
                 desc="B1 H16 d128 S131072 N8 (16384-token shards), bf16, q_dev 7"),
    "cfg5": dict(B=1, H=8, d=128, S=786432, N=16, q_dev=15,
                 desc="one device's share at 786k: B1 H8 d128 S786432 N16 (49152-token shards), bf16, "
                      "q_dev 15"),
    "3b": dict(B=1, H=32, d=100, S=262144, N=8, q_dev=7,
               desc="cfg3 with the head dimension of Table 1's 3B model: B1 H32 d100 S262144 N8, bf16, "
                    "q_dev 7 (matrix-core kernels, 128 columns computed)"),
    "d64": dict(B=1, H=32, d=64, S=262144, N=8, q_dev=7,
                desc="cfg3 with head dimension 64: B1 H32 d64 S262144 N8, bf16, q_dev 7 (matrix-core kernels, "
                     "64 columns computed)"),
    "d256": dict(B=1, H=16, d=256, S=262144, N=8, q_dev=7,
                 desc="cfg3's model width with head dimension 256: B1 H16 d256 S262144 N8, bf16, q_dev 7 "
                      "(matrix-core kernels, two 128-column halves)"),
    "cfg1": dict(B=1, H=1, d=64, S=256, N=4, q_dev=-1, dtype="f32",
                 desc="Tiny: B1 H1 d64 S256 N4 (64-token shards), fp32, all 16 steps (generic fp32 kernels; "
                      "launch-bound)"),
    "tiny": dict(B=1, H=2, d=128, S=4096, N=4, q_dev=-1, desc="B1 H2 d128 S4096 N4, bf16 (quick check)"),
}


def step_pairs(w, layout, j, k):
    return sa.sa_step_pairs(j, k, w["N"], layout, w["S"] // w["N"])


def played_steps(w):
    N = w["N"]
    devs = range(N) if w["q_dev"] < 0 else [w["q_dev"]]
    return [(i, j, (j - i) % N) for i in range(N) for j in devs]


def useful_flops(w, layout, per_pair):
    return sum(step_pairs(w, layout, j, k) for _, j, k in played_steps(w)) * w["B"] * w["H"] * per_pair * w["d"]


class Runner:
    def __init__(self, w, seed, bwd, skip=(0, 0)):
        self.w, self.bwd, self.skip = w, bwd, skip
        B, H, S, d, N = w["B"], w["H"], w["S"], w["d"], w["N"]
        dev = "cuda"
        n_in = 4 if bwd else 3
        hkv = w.get("H_kv", H)           # K and V (inputs 1 and 2) may have fewer heads
        self.dtype = torch.float32 if w.get("dtype") == "f32" else torch.bfloat16
        self.orig = [inputs.gaussian((B, hkv if i in (1, 2) else H, S, d), seed * 16 + i, self.dtype,
                                     device=dev) for i in range(n_in)]
        self.perm = [torch.empty_like(x) for x in self.orig]
        self.O = torch.empty(B, H, S, d, dtype=torch.float32, device=dev)
        self.LSE = torch.empty(B, H, S, dtype=torch.float32, device=dev)
        self.out = torch.empty(B, H, S, d, dtype=self.dtype, device=dev)
        self.c = S // N
        self.shape = sa.shard_shape(self.orig[0], self.c, self.LSE, kv=self.orig[1] if hkv != H else None)
        if bwd:
            self.delta = torch.empty_like(self.LSE)
            self.dQ = torch.empty_like(self.O)
            self.dK, self.dV = (torch.empty(B, hkv, S, d, dtype=torch.float32, device=dev) for _ in range(2))

    def one_pass(self, layout, timed):
        """The hot path for the played device(s).  Returns per-step ms tables or None."""
        w, c = self.w, self.c
        if layout == sa.STRIPED:
            for x, y in zip(self.orig, self.perm):
                sa.sa_stripe_permute(x, y, w["N"])
            ins = self.perm
        else:
            ins = self.orig
        bq, bk = self.skip      # (0, 0): the kernels' own skipping granularity
        t_f = sa.sa_ring_fwd_tiled(ins[0], ins[1], ins[2], self.O, self.LSE, w["N"], layout, self.shape,
                                   bq, bk, w["q_dev"], timed)
        devs = range(w["N"]) if w["q_dev"] < 0 else [w["q_dev"]]
        for j in devs:
            sa.sa_finalize(self.O[:, :, j * c:], self.out[:, :, j * c:], self.shape)
        t_b = None
        if self.bwd:
            t_b = sa.sa_ring_bwd_tiled(ins[0], ins[1], ins[2], ins[3], self.O, self.LSE, self.delta,
                                       self.dQ, self.dK, self.dV, w["N"], layout, self.shape, bq, bk,
                                       w["q_dev"], timed)
        return t_f, t_b


def cold_forward(run, layout, reps=2):
    """Forward ring with L2 and the memory-side cache flushed before every step (a 1 GiB
    read-modify-write), timed step by step from the host side of the C ABI: in a real ring a
    visiting K/V shard arrives from the neighbour, not from this device's caches.  Returns the
    [N][N] table of step durations (ms), averaged over reps."""
    w, c, N = run.w, run.c, run.w["N"]
    ins = run.perm if layout == sa.STRIPED else run.orig
    flush = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda")
    devs = range(N) if w["q_dev"] < 0 else [w["q_dev"]]
    table = [[0.0] * N for _ in range(N)]
    rows = lambda t, dev: t[:, :, dev * c:]
    for _ in range(reps):
        for j in devs:
            sa.sa_state_init(rows(run.O, j), rows(run.LSE, j), run.shape)
        for i in range(N):
            for j in devs:
                k = (j - i) % N
                flush.add_(1)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                sa.sa_attn_step_fwd(rows(ins[0], j), rows(ins[1], k), rows(ins[2], k), rows(run.O, j),
                                    rows(run.LSE, j), j, k, N, layout, run.shape)
                e1.record()
                e1.synchronize()
                table[i][j] += e0.elapsed_time(e1) / reps
    return table


def hbm_bound_kernels(run, reps=5):
    """The HBM-bound kernels of the pass, each timed alone (HIP events on the launch stream):
    GB/s of algorithmic bytes (tensor read + tensor written) and the fraction of the 8 TB/s peak."""
    w, c = run.w, run.c
    B, H, S, d, N = w["B"], w["H"], w["S"], w["d"], w["N"]
    j = max(w["q_dev"], 0)
    rows = lambda t: t[:, :, j * c:]
    cases = {
        "stripe_permute (one [B,H,S,d] bf16 tensor)":
            (lambda: sa.sa_stripe_permute(run.orig[0], run.perm[0], N), 2 * B * H * S * d * 2),
        "state_init (one shard)":
            (lambda: sa.sa_state_init(rows(run.O), rows(run.LSE), run.shape), B * H * c * (d * 4 + 4)),
        "finalize (one shard)":
            (lambda: sa.sa_finalize(rows(run.O), rows(run.out), run.shape), B * H * c * d * (4 + 2)),
    }
    if run.bwd:
        cases["bwd_preprocess (one shard)"] = (
            lambda: sa.sa_bwd_preprocess(rows(run.O), rows(run.perm[3]), rows(run.delta), run.shape),
            B * H * c * (d * (4 + 2) + 4))
    out = {}
    for name, (fn, nbytes) in cases.items():
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        e1.synchronize()
        ms = e0.elapsed_time(e1) / reps
        gbs = nbytes / ms / 1e6
        out[name] = {"ms": round(ms, 4), "bytes": nbytes, "GB/s": round(gbs, 1),
                     "frac_of_hbm_peak": round(gbs / PEAK_HBM_GBS, 3)}
    return out


def summarize_steps(w, layout, table, per_pair, table_min=None, table_med=None):
    """Per-step latency (mean over the timed passes; the fastest pass and the median if given)
    / TFLOP/s rows and the worst-device latency of every round."""
    N = w["N"]
    rows, worst = [], []
    for i in range(N):
        ms_round = 0.0
        for _, j, k in [s for s in played_steps(w) if s[0] == i]:
            ms = table[i][j]
            pairs = step_pairs(w, layout, j, k)
            fl = pairs * w["B"] * w["H"] * per_pair * w["d"]
            rows.append(dict(round=i, q_dev=j, kv_dev=k, ms=round(ms, 4),
                             tflops=round(fl / (ms * 1e9), 3) if ms > 0 else 0.0))
            if table_min is not None:
                rows[-1]["ms_min"] = round(table_min[i][j], 4)
            if table_med is not None:
                rows[-1]["ms_median"] = round(table_med[i][j], 4)
            ms_round = max(ms_round, ms)
        worst.append(round(ms_round, 4))
    return rows, worst


def cpu_baseline():
    """The fp64 oracle, as it stands, on a bounded sample of the same workload shape: one head of
    d = 128, the forward at a sequence length it finishes in ~10 s and the gradient (row by row,
    much slower per pair) at one it finishes in ~20 s.  `value` is the useful causal rate of
    forward + backward together, as the GPU figure is."""
    import numpy as np
    from oracle import striped_attention as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    d, S_f, S_b = 128, 32768, 8192
    scale = 1.0 / np.sqrt(d)
    q, k, v, g = (inputs.to_f64(x)[0, 0] for x in inputs.qkv(1, 1, S_f, d, 99, torch.bfloat16, with_dout=True))
    t0 = time.perf_counter()
    orc.causal_attention(q, k, v, scale)
    t_f = time.perf_counter() - t0
    t0 = time.perf_counter()
    orc.causal_attention_grad(q[:S_b], k[:S_b], v[:S_b], g[:S_b], scale)
    t_b = time.perf_counter() - t0
    fl_f = S_f * (S_f + 1) // 2 * 4 * d
    fl_b = S_b * (S_b + 1) // 2 * 10 * d
    return dict(value=(fl_f + fl_b) / (t_f + t_b) / 1e12, unit="TFLOP/s (useful causal, fp64)", cores=cores,
                kind="oracle", seconds=round(t_f + t_b, 2),
                forward=dict(tflops=fl_f / t_f / 1e12, seconds=round(t_f, 2), n_seq=S_f),
                backward=dict(tflops=fl_b / t_b / 1e12, seconds=round(t_b, 2), n_seq=S_b),
                sample="1 head, d=128: oracle.causal_attention at S=%d (%.1f GFLOP useful) and "
                       "oracle.causal_attention_grad at S=%d (%.1f GFLOP useful)" %
                       (S_f, fl_f / 1e9, S_b, fl_b / 1e9))


def device_info():
    """Compute units and clock as the runtime reports them, and the bf16 MFMA peak they imply
    (4096 flop per clock and compute unit); the roofline keeps the published 2.5 PFLOP/s."""
    cus, khz, mem = sa.sa_device_props()
    info = {"name": torch.cuda.get_device_name(0), "compute_units": cus, "max_clock_mhz": round(khz / 1e3, 1),
            "hbm_GB": round(mem / 1e9, 1),
            "bf16_peak_from_cus_and_clock_tflops": round(cus * khz * 1e3 * 4096 / 1e12, 1)}
    return info


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed passes (default 10; 50 for the workloads whose steps last under 1 ms)")
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg3", choices=sorted(WORKLOADS))
    ap.add_argument("--bwd", type=int, default=1, help="0: forward ring only (default: forward + backward)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--seed", type=int, default=3)
    ap.add_argument("--cold", action="store_true",
                    help="also time the forward steps with the caches flushed before each one")
    ap.add_argument("--skip-granularity", default="", metavar="BQxBK",
                    help="emulate tile skipping per BQ x BK tile (Sec. 3.1 of the paper), e.g. 2048x4096; "
                         "default: the kernels' own 32 x 32")
    ap.add_argument("--kv-heads", type=int, default=0, metavar="H_KV",
                    help="K and V with H_KV heads shared by groups of query heads (an extension; "
                         "default: as many as query heads, the paper's models)")
    ap.add_argument("--graph", action="store_true",
                    help="also record one pass into a HIP graph and time its replays (no per-step events)")
    args = ap.parse_args()
    skip = tuple(int(x) for x in args.skip_granularity.lower().split("x")) if args.skip_granularity else (0, 0)
    if len(skip) != 2:
        ap.error("--skip-granularity takes BQxBK")
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (the ring's N devices are played in sequence on "
              "it); --gpus N > 1 is not supported", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    sa.lib()
    w = dict(WORKLOADS[args.workload])
    if args.steps is None:
        args.steps = 50 if args.workload in ("cfg1", "cfg2", "tiny") else 10
    if args.kv_heads:
        if args.kv_heads < 1 or w["H"] % args.kv_heads:
            ap.error("--kv-heads must divide the workload's %d heads" % w["H"])
        w["H_kv"] = args.kv_heads
        w["desc"] += ", %d key/value heads" % args.kv_heads
    run = Runner(w, args.seed, bool(args.bwd), skip)
    torch.cuda.synchronize()

    for _ in range(args.warmup):
        run.one_pass(sa.STRIPED, False)
    torch.cuda.synchronize()
    # timed region: K passes of the striped hot path, per-step HIP events inside
    tables_f, tables_b = [], []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        tf, tb = run.one_pass(sa.STRIPED, True)
        tables_f.append(tf)
        tables_b.append(tb)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    N = w["N"]
    avg = lambda tabs: [[sum(t[i][j] for t in tabs) / len(tabs) for j in range(N)] for i in range(N)]
    low = lambda tabs: [[min(t[i][j] for t in tabs) for j in range(N)] for i in range(N)]
    med = lambda tabs: [[statistics.median(t[i][j] for t in tabs) for j in range(N)] for i in range(N)]
    per_pair_total = 4 + (10 if args.bwd else 0)
    flops = useful_flops(w, sa.STRIPED, per_pair_total)
    value = flops / (ms_per_step * 1e9)
    striped_rows, striped_worst = summarize_steps(w, sa.STRIPED, avg(tables_f), 4, low(tables_f), med(tables_f))

    # the comparison layout, same shapes (not part of `value`)
    run.one_pass(sa.CONTIGUOUS, False)
    torch.cuda.synchronize()
    ctab_f, ctab_b = [], []
    for _ in range(max(1, args.steps)):
        tf, tb = run.one_pass(sa.CONTIGUOUS, True)
        ctab_f.append(tf)
        ctab_b.append(tb)
    contig_rows, contig_worst = summarize_steps(w, sa.CONTIGUOUS, avg(ctab_f), 4, low(ctab_f), med(ctab_f))

    # roofline per kernel family: algorithmic flops of one launch / its average HIP-event
    # duration (events recorded by the ring driver on the launch stream); the dominant one
    # (largest share of the pass) is reported as "roofline"
    plain = not args.kv_heads and skip == (0, 0)
    traffic = measured_traffic(args.workload) if plain else {}
    c_rows = w["S"] // N

    f32 = w.get("dtype") == "f32"      # the generic kernels: fp32 FMA arithmetic, vector ALU peak
    peak, bound = (157.3, "alu") if f32 else (PEAK_BF16_TFLOPS, "mfma")

    def roof(rows, family, alg_bytes):
        name, kernels = FAMILIES[family]
        if f32:
            name = name.replace("_mfma_kernel", "_generic_kernel").replace("bwd_dkdv", "bwd_dkv")
        live = [r for r in rows if r["ms"] > 0]
        tot_ms = sum(r["ms"] for r in live)
        ach = sum(r["tflops"] * r["ms"] for r in live) / max(1e-9, tot_ms)
        out = dict(bound=bound, kernel=name, achieved=round(ach, 3), peak=peak,
                   unit="TFLOP/s", frac=round(ach / peak, 4), traffic=None,
                   avg_launch_ms=round(tot_ms / max(1, len(live)), 4), total_ms=round(tot_ms, 3))
        if all(k in traffic for k in kernels):      # bytes per launch (read + written) from the profile
            rd, wr = (sum(traffic[k][i] for k in kernels) for i in (0, 1))
            out["traffic"] = int(round((rd + wr) * 1e9))
            out["traffic_detail"] = {"read_GB": round(rd, 2), "written_GB": round(wr, 2),
                                     "algorithmic_GB": round(alg_bytes / 1e9, 2),
                                     "source": "profiles/ring_step_kernels_%s.txt" % args.workload}
        return out
    # algorithmic bytes of one step: Q, K, V once, O and LSE read and written (forward);
    # Q, K, V, dO once per kernel, LSE and delta, dQ / dK / dV read and written (backward)
    bh = w["B"] * w["H"]
    alg_f = bh * c_rows * (3 * w["d"] * 2 + 2 * w["d"] * 4 + 2 * 4)
    alg_b = bh * c_rows * (2 * 4 * w["d"] * 2 + 2 * 2 * 4 + 3 * 2 * w["d"] * 4)
    roofs = {"fwd": roof(striped_rows, "fwd", alg_f)}
    if args.bwd:
        rows_b, _ = summarize_steps(w, sa.STRIPED, avg(tables_b), 10)
        roofs["bwd"] = roof(rows_b, "bwd", alg_b)
    roofline = max(roofs.values(), key=lambda r: r["total_ms"])

    result = {
        "metric": "useful causal TFLOP/s per ring step (striped layout, worst-loaded device's share)",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.get("dtype", "bf16"), "data": "synthetic",
        "config": {"workload": args.workload + ": " + w["desc"], "B": w["B"], "H": w["H"],
                   "H_kv": w.get("H_kv", w["H"]), "d": w["d"],
                   "n_seq": w["S"], "N": N, "c": w["S"] // N, "q_dev": w["q_dev"],
                   "pass": "stripe_permute + ring fwd" + (" + ring bwd" if args.bwd else "") + " + finalize"},
        "frac_of_bf16_peak": round(value / PEAK_BF16_TFLOPS, 4),
        "device": device_info(),
        "roofline": roofline,
        "roofline_by_kernel": roofs,
        "striped": {"worst_device_ms_per_round": striped_worst, "ring_sum_ms": round(sum(striped_worst), 4),
                    "steps": striped_rows},
        "contiguous": {"worst_device_ms_per_round": contig_worst, "ring_sum_ms": round(sum(contig_worst), 4),
                       "steps": contig_rows},
        "worst_device_latency_ratio_contiguous_over_striped":
            round(sum(contig_worst) / max(1e-9, sum(striped_worst)), 3),
        "paper_context": "end-to-end training speedups 1.45x (256k, 8xA100) and 1.65x (786k, 16 TPUv4); "
                         "not step latencies",
    }
    if args.bwd:
        rb, wb = summarize_steps(w, sa.STRIPED, avg(tables_b), 10, low(tables_b), med(tables_b))
        result["striped"]["bwd_steps"], result["striped"]["bwd_worst_device_ms_per_round"] = rb, wb
        rb, wb = summarize_steps(w, sa.CONTIGUOUS, avg(ctab_b), 10, low(ctab_b), med(ctab_b))
        result["contiguous"]["bwd_steps"], result["contiguous"]["bwd_worst_device_ms_per_round"] = rb, wb
    if skip != (0, 0):
        from paper_2311_09431_amd import tms
        c = w["S"] // N
        if args.bwd:
            tot = lambda r: sum(a + b for a, b in zip(r["worst_device_ms_per_round"],
                                                      r["bwd_worst_device_ms_per_round"]))
        else:
            tot = lambda r: sum(r["worst_device_ms_per_round"])
        result["skip_granularity"] = {
            "tile_q": skip[0], "tile_k": skip[1],
            "note": "useful TFLOP/s still count unmasked pairs only; masked parts of computed tiles are waste",
            "worst_device_ratio_measured": round(tot(result["contiguous"]) / max(1e-9, tot(result["striped"])), 3),
            "worst_device_ratio_computed_tiles": round(
                tms.tiled_attention_limit(N, c, *skip, devices=None if w["q_dev"] < 0 else [w["q_dev"]]), 3),
            "worst_device_ratio_element_granularity": round(tms.attention_only_limit(N, c), 3),
        }
    if args.cold:
        cold = {}
        for name, layout in (("striped", sa.STRIPED), ("contiguous", sa.CONTIGUOUS)):
            if layout == sa.STRIPED:
                run.one_pass(sa.STRIPED, False)          # leaves the permuted inputs in place
            rows_c, worst_c = summarize_steps(w, layout, cold_forward(run, layout), 4)
            live = [r for r in rows_c if r["ms"] > 0]
            cold[name] = {"worst_device_ms_per_round": worst_c, "ring_sum_ms": round(sum(worst_c), 4),
                          "mean_step_ms": round(sum(r["ms"] for r in live) / max(1, len(live)), 4)}
        cold["worst_device_latency_ratio_contiguous_over_striped"] = round(
            cold["contiguous"]["ring_sum_ms"] / max(1e-9, cold["striped"]["ring_sum_ms"]), 3)
        cold["note"] = "forward steps, L2 and memory-side cache flushed before each step"
        result["cold_cache"] = cold
    if args.graph:
        # the same pass without per-step events, recorded once and replayed: what is left when
        # the host side (launches, event records) is taken out
        graph = torch.cuda.CUDAGraph()
        run.one_pass(sa.STRIPED, False)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            run.one_pass(sa.STRIPED, False)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        result["graph_replay"] = {"ms_per_step": round(g_ms, 4), "value": round(flops / (g_ms * 1e9), 2),
                                  "unit": "TFLOP/s"}
    result["hbm_bound_kernels"] = hbm_bound_kernels(run)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
