"""One transformer layer of ONE sequence-parallel device at the paper's model shapes (Table 1),
forward + backward, Striped vs Ring Attention layout, on one GPU.

    python -m paper_2311_09431_amd.layer_bench --model 7B --seq 262144 --N 8 [--reps 3]

What a device does per layer (Sec. 2.2 / 2.3, Algorithm 1): project its c = n_seq / N tokens
to Q, K, V, rotate Q and K by their position ids (which travelled with the tokens through the
stripe permutation), play its N ring steps against the visiting K/V shards, project the
output, run the MLP; backward in reverse.  Here the worst-loaded device (the last one, under
both layouts) is played: the attention part runs on this library's ring drivers
(`q_dev_only`), the projections and the two-matrix MLP are plain torch matmuls (they are the
same under both layouts and are not part of the hot path); the other devices' K/V shards are
synthetic.  Nothing is sharded or communicated: a round of the real ring lasts as long as its
slowest device (Sec. 1), which is what is timed.

Printed beside the measurement: the Theoretical Maximum Speedup of Sec. 4 for the same model,
sequence length and N, with the logits term left out (one layer, no vocabulary projection) and
attention priced like every other FLOP (bf16 matrix cores for both).  The paper's end-to-end
figures (1.45x on 8 A100, 1.65x on 16 TPUv4) include effects this single-GPU run does not have
(communication, the embedding and logits layers, a second mesh axis) and are context only.
"""
import argparse
import json
import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

from paper_2311_09431_amd import binding as sa   # noqa: E402
from paper_2311_09431_amd import inputs           # noqa: E402
from paper_2311_09431_amd import tms               # noqa: E402


def layer_tms(model, n_seq, N):
    """Sec. 4's model for one layer: no logits term, attention FLOPs at the price of the others."""
    m = dict(tms.MODELS[model] if isinstance(model, str) else model)
    m["n_vocab"] = 0
    return tms.tms(m, n_seq, N, 1.0)


class DeviceLayer:
    """Weights, activations and buffers of the played device; every tensor lives on the GPU."""

    def __init__(self, model, n_seq, N, layout, seed=7):
        m = tms.MODELS[model] if isinstance(model, str) else model
        self.m, self.N, self.layout = m, N, layout
        self.S, self.c, self.dev = n_seq, n_seq // N, N - 1
        self.H, self.dm, self.dff = m["n_head"], m["d_model"], m["d_ff"]
        self.d = self.dm // self.H
        g = lambda shape, k, std=1.0: inputs.gaussian(shape, seed * 64 + k, torch.bfloat16, std, device="cuda")
        dm, dff, H, d, c, S = self.dm, self.dff, self.H, self.d, self.c, self.S
        self.x = g((c, dm), 0)
        self.Wqkv, self.Wo = g((dm, 3 * dm), 1, dm ** -0.5), g((dm, dm), 2, dm ** -0.5)
        self.W1, self.W2 = g((dm, dff), 3, dm ** -0.5), g((dff, dm), 4, dff ** -0.5)
        self.dy = g((c, dm), 5)
        # K and V of the whole sequence in device order, stored [B, rows, H, d] as a projection
        # writes them; the played device's shard is overwritten with its own projection
        self.K, self.V = g((1, S, H, d), 6), g((1, S, H, d), 7)
        self.Q = torch.empty(1, S, H, d, dtype=torch.bfloat16, device="cuda")
        self.dO = torch.empty_like(self.Q)
        bhsd = lambda t: t.permute(0, 2, 1, 3)
        self.Qv, self.Kv, self.Vv, self.dOv = bhsd(self.Q), bhsd(self.K), bhsd(self.V), bhsd(self.dO)
        f32 = lambda: torch.empty(1, S, H, d, dtype=torch.float32, device="cuda")
        self.O, self.dQ, self.dK, self.dV = (bhsd(f32()) for _ in range(4))
        self.LSE = torch.empty(1, H, S, dtype=torch.float32, device="cuda")
        self.delta = torch.empty_like(self.LSE)
        self.out = bhsd(torch.empty(1, S, H, d, dtype=torch.bfloat16, device="cuda"))
        self.shape = sa.shard_shape(self.Qv, c, self.LSE)
        # position ids of the played device's rows: they travel with the tokens (Sec. 2.3)
        ids = torch.arange(S, dtype=torch.int32, device="cuda")
        if layout == sa.STRIPED:
            p = torch.empty_like(ids)
            sa.sa_stripe_permute(ids, p, N, seq_axis=0)
            ids = p
        self.pos = ids[self.dev * c:(self.dev + 1) * c].contiguous()

    def rows(self, t):
        return t[:, :, self.dev * self.c:(self.dev + 1) * self.c]

    # ---- the parts that do not depend on the layout: torch matmuls
    def project_in(self):
        qkv = (self.x @ self.Wqkv).view(self.c, 3, self.H, self.d)
        for i, t in enumerate((self.Q, self.K, self.V)):
            t[0, self.dev * self.c:(self.dev + 1) * self.c].copy_(qkv[:, i])

    def project_out_and_mlp(self):
        a = self.rows(self.out).permute(0, 2, 1, 3).reshape(self.c, self.dm)
        self.a = a
        self.h0 = a @ self.Wo
        self.h1 = torch.relu(self.h0 @ self.W1)
        return self.h1 @ self.W2

    def backward_dense_tail(self):
        # MLP and output projection: weight and input gradients
        dW2 = self.h1.t() @ self.dy
        dh1 = (self.dy @ self.W2.t()) * (self.h1 > 0)
        dW1 = self.h0.t() @ dh1
        dh0 = dh1 @ self.W1.t()
        dWo = self.a.t() @ dh0
        da = dh0 @ self.Wo.t()
        self.dO[0, self.dev * self.c:(self.dev + 1) * self.c].copy_(da.view(self.c, self.H, self.d))
        return dW2, dW1, dWo

    def backward_dense_head(self):
        c, dev = self.c, self.dev
        sl = slice(dev * c, (dev + 1) * c)
        dqkv = torch.stack([self.dQ.permute(0, 2, 1, 3)[0, sl], self.dK.permute(0, 2, 1, 3)[0, sl],
                            self.dV.permute(0, 2, 1, 3)[0, sl]], dim=1).to(torch.bfloat16).view(c, 3 * self.dm)
        return self.x.t() @ dqkv, dqkv @ self.Wqkv.t()

    # ---- the attention part: this library
    def attention_forward(self):
        sa.sa_rope(self.rows(self.Qv), self.rows(self.Qv), self.pos, self.shape)
        sa.sa_rope(self.rows(self.Kv), self.rows(self.Kv), self.pos, self.shape)
        sa.sa_ring_fwd(self.Qv, self.Kv, self.Vv, self.O, self.LSE, self.N, self.layout, self.shape, self.dev)
        sa.sa_finalize(self.rows(self.O), self.rows(self.out), self.shape)

    def attention_backward(self):
        sa.sa_ring_bwd(self.Qv, self.Kv, self.Vv, self.dOv, self.O, self.LSE, self.delta, self.dQ, self.dK,
                       self.dV, self.N, self.layout, self.shape, self.dev)
        # gradients w.r.t. the unrotated q and k of the played device's own shard
        sa.sa_rope(self.rows(self.dQ), self.rows(self.dQ), self.pos, self.f32_shape(), inverse=True)
        sa.sa_rope(self.rows(self.dK), self.rows(self.dK), self.pos, self.f32_shape(), inverse=True)

    def f32_shape(self):
        return sa.shard_shape(self.dQ, self.c, self.LSE)

    def step(self, ev):
        """One forward + backward of the layer; ev(name) records an event on the stream."""
        ev("start")
        self.project_in()
        ev("in")
        self.attention_forward()
        ev("attn_f")
        y = self.project_out_and_mlp()
        tail = self.backward_dense_tail()
        ev("dense")
        self.attention_backward()
        ev("attn_b")
        head = self.backward_dense_head()
        ev("end")
        return y, tail, head


def time_layer(model, n_seq, N, layout, reps):
    layer = DeviceLayer(model, n_seq, N, layout)
    names = ["start", "in", "attn_f", "dense", "attn_b", "end"]
    totals = {k: 0.0 for k in ("dense_ms", "attention_fwd_ms", "attention_bwd_ms")}
    for rep in range(reps + 1):
        evs = {}

        def ev(name):
            e = torch.cuda.Event(enable_timing=True)
            e.record()
            evs[name] = e
        layer.step(ev)
        torch.cuda.synchronize()
        if rep == 0:
            continue                         # warm-up
        t = [evs[a].elapsed_time(evs[b]) for a, b in zip(names, names[1:])]
        totals["dense_ms"] += (t[0] + t[2] + t[4]) / reps
        totals["attention_fwd_ms"] += t[1] / reps
        totals["attention_bwd_ms"] += t[3] / reps
    totals["layer_ms"] = sum(totals.values())
    return {k: round(v, 3) for k, v in totals.items()}


def run(model, n_seq, N, reps=3):
    striped = time_layer(model, n_seq, N, sa.STRIPED, reps)
    ring = time_layer(model, n_seq, N, sa.CONTIGUOUS, reps)
    m = tms.MODELS[model] if isinstance(model, str) else model
    c = n_seq // N
    tok_s = lambda r: round(c / (r["layer_ms"] * 1e-3), 1)
    attn = lambda r: r["attention_fwd_ms"] + r["attention_bwd_ms"]
    return {
        "what": "one layer (forward + backward) of the worst-loaded sequence-parallel device, one MI355X",
        "model": model if isinstance(model, str) else "custom", "d_model": m["d_model"], "n_head": m["n_head"],
        "d_head": m["d_model"] // m["n_head"], "d_ff": m["d_ff"], "n_seq": n_seq, "N": N, "c": c,
        "dtype": "bf16", "data": "synthetic", "striped": striped, "ring": ring,
        "tokens_per_s_per_layer": {"striped": tok_s(striped), "ring": tok_s(ring)},
        "layer_speedup_striped_over_ring": round(ring["layer_ms"] / striped["layer_ms"], 3),
        "attention_speedup_striped_over_ring": round(attn(ring) / attn(striped), 3),
        "tms_one_layer_model": round(layer_tms(model, n_seq, N), 3),
        "attention_only_limit": round(tms.attention_only_limit(N, c), 3),
        "paper_context": "end-to-end training speedups 1.45x (3B, 256k, 8 A100) and 1.65x (3B, 786k, 16 TPUv4)",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--model", default="7B", choices=sorted(tms.MODELS))
    ap.add_argument("--seq", type=int, default=262144)
    ap.add_argument("--N", type=int, default=8)
    ap.add_argument("--reps", type=int, default=3)
    args = ap.parse_args()
    if args.seq % args.N:
        ap.error("--seq must be a multiple of --N")
    if not torch.cuda.is_available():
        print("layer_bench: no GPU visible", file=sys.stderr)
        sys.exit(1)
    print(json.dumps(run(args.model, args.seq, args.N, args.reps)))


if __name__ == "__main__":
    main()
