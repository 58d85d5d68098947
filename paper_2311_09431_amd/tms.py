"""Theoretical Maximum Speedup (TMS) of Striped over Ring Attention (Sec. 4 of the paper).

A closed-form model, host-only, not part of the GPU path: communication fully
overlapped, non-matmul FLOPs free, attention FLOPs costing `attn_cost` times the
other FLOPs (2 on A100, where attention ran in TF32; 1 on TPU).  Per token and
layer:
    other     = 2 (4 d^2 + 2 d d_ff) + 2 n_vocab d / n_layer      (projections, MLP, logits)
    attention = 4 n_seq d * attn_cost                             (QK^T and PV over the full row)
Ring Attention's slowest device does c(c+1)/2 + (N-1) c^2 of the N c^2 interactions a
device-row holds, i.e. the fraction (N - 1/2)/N for large c; Striped Attention does 1/2.
    TMS = (other + attention (N - 1/2)/N) / (other + attention / 2)
This reading of Sec. 4 reproduces the TMS columns the paper prints to two decimals
(tests/golden/tms_values.txt).
"""

MODELS = {  # Table 1: n_vocab, d_model, d_ff, n_layer, n_head
    "1B": dict(n_vocab=32000, d_model=2048, d_ff=5504, n_layer=22, n_head=16),
    "3B": dict(n_vocab=32000, d_model=3200, d_ff=8640, n_layer=26, n_head=32),
    "7B": dict(n_vocab=32000, d_model=4096, d_ff=11008, n_layer=32, n_head=32),
}


def tms(model, n_seq, N, attn_cost):
    """TMS for `model` ("1B" / "3B" / "7B" or a dict like MODELS' values), total sequence
    length n_seq, N sequence-parallel devices, attention FLOP cost factor attn_cost."""
    m = MODELS[model] if isinstance(model, str) else model
    d = m["d_model"]
    other = 2 * (4 * d * d + 2 * d * m["d_ff"]) + 2 * m["n_vocab"] * d / m["n_layer"]
    attn = 4 * n_seq * d * attn_cost
    return (other + attn * (N - 0.5) / N) / (other + attn * 0.5)


def attention_only_limit(N, c=None):
    """Ratio of the per-round worst-device work summed over the ring, contiguous over
    striped: (c(c+1)/2 + (N-1) c^2) / (N c(c+1)/2); (2N-1)/N as c grows (Sec. 2.3)."""
    if c is None:
        return (2 * N - 1) / N
    return (c * (c + 1) / 2 + (N - 1) * c * c) / (N * c * (c + 1) / 2)


def computed_tiles(q_dev, kv_dev, c, striped, tile_q, tile_k):
    """Tiles of the step's c x c block that hold at least one allowed pair, i.e. are computed
    when work is skipped per tile_q x tile_k tile (Sec. 2.2.1, 3.1).  Allowed pairs in local
    indices: key b <= query a - off (Sec. 2.2, 2.3)."""
    nq, nk = c // tile_q, c // tile_k
    if striped:
        off = 1 if kv_dev > q_dev else 0
    elif q_dev < kv_dev:
        return 0
    elif q_dev > kv_dev:
        return nq * nk
    else:
        off = 0
    n = 0
    for r in range(nq):
        last_key = (r + 1) * tile_q - 1 - off
        if last_key >= 0:
            n += min(nk, last_key // tile_k + 1)
    return n


def tiled_attention_limit(N, c, tile_q, tile_k, devices=None):
    """attention_only_limit when work is skipped per tile_q x tile_k tile: per-round worst-device
    number of computed tiles summed over the ring, contiguous over striped.  1.0 means striping
    gains nothing at that granularity (Sec. 3.2: c = 4096 with 2048 x 4096 tiles).  `devices`
    restricts the maximum to those query devices (default: all N)."""
    devs = range(N) if devices is None else devices

    def ring_sum(striped):
        return sum(max(computed_tiles(j, (j - i) % N, c, striped, tile_q, tile_k) for j in devs)
                   for i in range(N))
    return ring_sum(False) / ring_sum(True)
