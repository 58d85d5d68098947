"""Plain fp64 CPU oracle for causal attention, its gradient, the stripe
permutation, the per-step masks and the ring schedule of Striped Attention
(arxiv 2311.09431).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's
CPU-baseline leg.  It shares no code with the HIP library and never imports it.

The method is exact (Sec. 1: the permutation does not change the output), so the
forward oracle is the definition of causal attention in Sec. 2.1 written out
one query row at a time, and the backward oracle is the analytic gradient of
that definition (the paper does not describe a backward pass; it only states,
Fig. 1 caption, that the layout persists through it).  The ring functions follow
Algorithm 1 with the mask of a step decided from the tokens' positions in the
original sequence (Sec. 2.3, "causal with respect to the order in which tokens
appear in the original input sequence"), never from a local-index shortcut.

All arithmetic is float64.  Matrices of one head are [n_seq, d_head]; the
*_bh wrappers map over leading [B, H] axes.  Notation follows the paper:
N devices, block size c = n_seq / N, query device j, key/value device k.

Pinned by tests/test_oracle_*.py against: brute-force S x S softmax with the
mask matrix C, closed forms (Q = 0, V = 1, first row), a library causal SDPA
and library autograd in fp64, central finite differences (the matrix-form gradient over a row set also against
the row-by-row one), the paper's printed
stripe example, its Work(i, j) formula and its tiling examples; the grouped-head
functions (fewer key/value heads, an extension) against the library's grouped
attention and autograd, repeated heads and finite differences.
"""
import numpy as np

CONTIGUOUS = 0   # Ring Attention layout (Sec. 2.2)
STRIPED = 1      # Striped Attention layout (Sec. 2.3)


# --------------------------------------------------------------------------
# Sec. 2.1: causal self-attention, one query row at a time
# --------------------------------------------------------------------------
def causal_mask(n_seq):
    """C[i, j] = -inf if i < j else 0 (Sec. 2.1)."""
    i = np.arange(n_seq)[:, None]
    j = np.arange(n_seq)[None, :]
    return np.where(i < j, -np.inf, 0.0)


def causal_attention_rows(Q, K, V, scale, rows):
    """Rows `rows` of Softmax(scale * Q K^T + C) V and their log-sum-exp.

    Row i sees keys 0..i (C[i, j] = 0 iff i >= j).  LSE_i is the natural log of
    the softmax denominator, scale included.
    """
    Q = np.asarray(Q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    rows = np.asarray(rows, np.int64)
    O = np.zeros((len(rows), V.shape[1]))
    LSE = np.zeros(len(rows))
    for n, i in enumerate(rows):
        s = scale * (K[: i + 1] @ Q[i])
        m = s.max()
        p = np.exp(s - m)
        l = p.sum()
        O[n] = (p @ V[: i + 1]) / l
        LSE[n] = m + np.log(l)
    return O, LSE


def causal_attention(Q, K, V, scale):
    """CausalAttn(Q, K, V) of Sec. 2.1 for one head; returns (O, LSE)."""
    return causal_attention_rows(Q, K, V, scale, np.arange(Q.shape[0]))


def causal_attention_grad(Q, K, V, dO, scale, rows=None):
    """Gradient of sum(O * dO) w.r.t. Q, K, V for O = CausalAttn(Q, K, V).

    With P = Softmax(scale Q K^T + C): dV = P^T dO; dP = dO V^T;
    dS_ij = P_ij (dP_ij - sum_t dO_it O_it); dQ = scale dS K; dK = scale dS^T Q.
    If `rows` is given, dO is treated as zero outside those query rows.
    """
    Q = np.asarray(Q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    dO = np.asarray(dO, np.float64)
    n_seq = Q.shape[0]
    rows = np.arange(n_seq) if rows is None else np.asarray(rows, np.int64)
    dQ = np.zeros_like(Q)
    dK = np.zeros_like(K)
    dV = np.zeros_like(V)
    for i in rows:
        s = scale * (K[: i + 1] @ Q[i])
        p = np.exp(s - s.max())
        p /= p.sum()
        o = p @ V[: i + 1]
        dV[: i + 1] += np.outer(p, dO[i])
        dp = V[: i + 1] @ dO[i]
        ds = p * (dp - dO[i] @ o)
        dQ[i] = scale * (ds @ K[: i + 1])
        dK[: i + 1] += scale * np.outer(ds, Q[i])
    return dQ, dK, dV


def causal_attention_grad_matrix(Q, K, V, dO, scale, rows):
    """The same gradient for a set of query rows, in the matrix form of Sec. 2.1.

    With R = `rows` (dO is treated as zero outside R): S = scale Q_R K^T + C_R is formed whole
    (|R| rows; the columns after the last row of R, which C masks for all of R, are left
    out), P = Softmax(S) row-wise, O_R = P V, dV = P^T dO_R, dP = dO_R V^T,
    dS = P * (dP - rowsum(dO_R * O_R)), dQ_R = scale dS K, dK = scale dS^T Q_R.
    Nothing is blocked: memory is a few |R| x n_seq float64 matrices, so callers keep |R|
    moderate (the gradient is additive over disjoint row sets).  Also returns O_R and LSE_R.
    Since dQ_i depends on row i of dO only, dQ[R] is also the dense-dO answer for those rows.
    """
    Q = np.asarray(Q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    dO = np.asarray(dO, np.float64)
    rows = np.asarray(rows, np.int64)
    n = int(rows.max()) + 1      # keys at later positions are masked for every row of R: left out
    K, V = K[:n], V[:n]
    S = scale * (Q[rows] @ K.T)
    S[np.arange(n)[None, :] > rows[:, None]] = -np.inf      # C[i, j] = -inf iff i < j
    m = S.max(axis=1, keepdims=True)
    P = np.exp(S - m)
    l = P.sum(axis=1, keepdims=True)
    P /= l
    O = P @ V
    g = dO[rows]
    dV = P.T @ g
    dS = P * (g @ V.T - (g * O).sum(axis=1, keepdims=True))
    dQ = np.zeros_like(Q)
    dQ[rows] = scale * (dS @ K)
    dK = np.zeros_like(Q)
    dK[:n] = scale * (dS.T @ Q[rows])
    dVf = np.zeros((Q.shape[0], V.shape[1]))
    dVf[:n] = dV
    return dQ, dK, dVf, O, (m + np.log(l))[:, 0]


def _map_bh(fn, n_out, *arrays):
    B, H = arrays[0].shape[:2]
    outs = [[[None] * H for _ in range(B)] for _ in range(n_out)]
    for b in range(B):
        for h in range(H):
            res = fn(*[a[b, h] for a in arrays])
            for n in range(n_out):
                outs[n][b][h] = res[n]
    return tuple(np.array(o) for o in outs)


def causal_attention_bh(Q, K, V, scale):
    """causal_attention over leading [B, H] axes."""
    return _map_bh(lambda q, k, v: causal_attention(q, k, v, scale), 2, Q, K, V)


def causal_attention_grad_bh(Q, K, V, dO, scale, rows=None):
    """causal_attention_grad over leading [B, H] axes."""
    return _map_bh(lambda q, k, v, g: causal_attention_grad(q, k, v, g, scale, rows),
                   3, Q, K, V, dO)


# --------------------------------------------------------------------------
# Fewer key/value heads than query heads (grouped-query / multi-query attention).
# Not part of the paper: each query head is the attention of Sec. 2.1 against the
# key/value head its group shares, so the oracle is that definition per query
# head, and a shared head's gradient is the sum over the query heads that read it.
# --------------------------------------------------------------------------
def kv_head_of(h, H, H_kv):
    """Key/value head read by query head h: consecutive groups of H / H_kv query heads."""
    assert H % H_kv == 0
    return h // (H // H_kv)


def causal_attention_gqa(Q, K, V, scale):
    """Q [B, H, S, d], K and V [B, H_kv, S, d] -> (O [B, H, S, d], LSE [B, H, S])."""
    B, H = Q.shape[:2]
    H_kv = K.shape[1]
    O = np.zeros(Q.shape)
    LSE = np.zeros(Q.shape[:3])
    for b in range(B):
        for h in range(H):
            hk = kv_head_of(h, H, H_kv)
            O[b, h], LSE[b, h] = causal_attention(Q[b, h], K[b, hk], V[b, hk], scale)
    return O, LSE


def causal_attention_gqa_grad(Q, K, V, dO, scale):
    """Gradient of sum(O * dO) for causal_attention_gqa: dQ like Q, dK and dV like K, V."""
    B, H = Q.shape[:2]
    H_kv = K.shape[1]
    dQ = np.zeros(Q.shape)
    dK = np.zeros(K.shape)
    dV = np.zeros(V.shape)
    for b in range(B):
        for h in range(H):
            hk = kv_head_of(h, H, H_kv)
            q, k, v = causal_attention_grad(Q[b, h], K[b, hk], V[b, hk], dO[b, h], scale)
            dQ[b, h] = q
            dK[b, hk] += k
            dV[b, hk] += v
    return dQ, dK, dV


# --------------------------------------------------------------------------
# Sec. 2.2 / 2.3: which device owns which token
# --------------------------------------------------------------------------
def global_position(dev, a, N, c, layout):
    """Position in the original sequence of local row `a` of device `dev`.

    Contiguous (Sec. 2.2): device j owns rows j*c .. j*c+c-1.
    Striped (Sec. 2.3): device j owns the tokens congruent to j modulo N.
    """
    if layout == CONTIGUOUS:
        return dev * c + a
    if layout == STRIPED:
        return a * N + dev
    raise ValueError("unknown layout")


def stripe_source_index(n_seq, N):
    """src[p] = original position of the token at permuted position p, where the
    permuted sequence, split contiguously, gives device j the tokens j, j+N, ...
    (Sec. 2.3: permute, then partition as in Ring Attention)."""
    if n_seq % N:
        raise ValueError("n_seq must be a multiple of N")
    c = n_seq // N
    src = np.empty(n_seq, np.int64)
    for dev in range(N):
        for a in range(c):
            src[dev * c + a] = global_position(dev, a, N, c, STRIPED)
    return src


def stripe_permute(x, N, axis):
    """Apply the stripe permutation along `axis` (bit-exact copy of rows)."""
    x = np.asarray(x)
    return np.take(x, stripe_source_index(x.shape[axis], N), axis=axis)


def unstripe_permute(x, N, axis):
    """Inverse of stripe_permute along `axis`."""
    x = np.asarray(x)
    src = stripe_source_index(x.shape[axis], N)
    inv = np.empty_like(src)
    inv[src] = np.arange(len(src))
    return np.take(x, inv, axis=axis)


def rope(x, pos, base=10000.0, inverse=False):
    """Rotary position embedding of the rows of x[..., rows, d] at positions pos[rows] (or
    pos[..., rows] broadcastable to x's leading axes): pairs (x_i, x_{i+d/2}) are rotated by
    the angle pos * base**(-2i/d), i < d/2.  Sec. 2.3 only requires that each token keeps the
    position id of its ORIGINAL place when the sequence is permuted; the rotation itself is
    the usual one (rotate-half form).  inverse=True rotates by the negative angle (the
    transpose, which maps gradients back)."""
    x = np.asarray(x, np.float64)
    d = x.shape[-1]
    if d % 2:
        raise ValueError("head dimension must be even")
    half = d // 2
    inv_freq = np.asarray(base, np.float64) ** (-2.0 * np.arange(half) / d)
    ang = np.asarray(pos, np.float64)[..., None] * inv_freq          # [..., rows, half]
    if inverse:
        ang = -ang
    cs, sn = np.cos(ang), np.sin(ang)
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * cs - hi * sn, hi * cs + lo * sn], axis=-1)


# --------------------------------------------------------------------------
# GetMask(j, k): the c x c tile of the causal mask seen by a ring step
# --------------------------------------------------------------------------
def get_mask(j, k, N, c, layout):
    """allowed[a, b] = True iff query row a of device j may attend to key row b
    of device k, decided in the original token order: key position <= query
    position (Sec. 2.1 for the rule, Sec. 2.3 for applying it to original
    positions)."""
    a = np.arange(c)[:, None]
    b = np.arange(c)[None, :]
    return global_position(k, b, N, c, layout) <= global_position(j, a, N, c, layout)


def work(j, k, N, c, layout):
    """Number of unmasked query/key interactions of step (j, k) (Sec. 2.3, Work)."""
    return int(get_mask(j, k, N, c, layout).sum())


def classify_tiles(allowed, tile_q, tile_k):
    """Split a block's mask into tile_q x tile_k tiles (Sec. 2.2.1) and count
    (fully unmasked, partially masked, fully masked).  A tile is computed iff it
    has at least one unmasked element (Sec. 3.1), i.e. the first two classes."""
    cq, ck = allowed.shape
    if cq % tile_q or ck % tile_k:
        raise ValueError("tile must divide the block")
    full = part = empty = 0
    for r in range(0, cq, tile_q):
        for s in range(0, ck, tile_k):
            t = allowed[r:r + tile_q, s:s + tile_k]
            if t.all():
                full += 1
            elif t.any():
                part += 1
            else:
                empty += 1
    return full, part, empty


# --------------------------------------------------------------------------
# Algorithm 1: one step (AccumulateAttentionFragment) and the ring
# --------------------------------------------------------------------------
def attention_fragment(Qj, Kk, Vk, allowed, scale):
    """Softmax attention of the rows of Qj over the allowed keys of (Kk, Vk):
    returns the normalised partial output and its log-sum-exp.  A row with no
    allowed key gets output 0 and LSE = -inf."""
    Qj = np.asarray(Qj, np.float64)
    Kk = np.asarray(Kk, np.float64)
    Vk = np.asarray(Vk, np.float64)
    c, d = Qj.shape[0], Vk.shape[1]
    O = np.zeros((c, d))
    LSE = np.full(c, -np.inf)
    for a in range(c):
        idx = np.nonzero(allowed[a])[0]
        if len(idx) == 0:
            continue
        s = scale * (Kk[idx] @ Qj[a])
        m = s.max()
        p = np.exp(s - m)
        l = p.sum()
        O[a] = (p @ Vk[idx]) / l
        LSE[a] = m + np.log(l)
    return O, LSE


def merge(O1, LSE1, O2, LSE2):
    """Combine two normalised partial results over disjoint key sets (the lazy
    softmax accumulation of Algorithm 1's caption): the weights are the two
    softmax denominators.  (0, -inf) is the identity."""
    LSE = np.logaddexp(LSE1, LSE2)
    with np.errstate(invalid="ignore"):
        w1 = np.where(np.isneginf(LSE1), 0.0, np.exp(LSE1 - LSE))
        w2 = np.where(np.isneginf(LSE2), 0.0, np.exp(LSE2 - LSE))
    return w1[:, None] * O1 + w2[:, None] * O2, LSE


def ring_step_fwd(O, LSE, Qj, Kk, Vk, j, k, N, layout, scale):
    """Out_j <- AccumulateAttentionFragment(Out_j, Q_j, K_k, V_k, GetMask(j, k))
    with Out_j held as normalised (O, LSE)."""
    c = Qj.shape[0]
    Of, Lf = attention_fragment(Qj, Kk, Vk, get_mask(j, k, N, c, layout), scale)
    return merge(np.asarray(O, np.float64), np.asarray(LSE, np.float64), Of, Lf)


def ring_schedule(N):
    """(round i, device j, held block k) triples in Algorithm 1's order:
    k = (j - i) mod N."""
    return [(i, j, (j - i) % N) for i in range(N) for j in range(N)]


def ring_attention(Qp, Kp, Vp, N, layout, scale, order=None):
    """Algorithm 1 on one head, all N devices played in sequence.  Qp, Kp, Vp are
    in device order (already stripe-permuted for the striped layout): device j
    owns rows j*c .. (j+1)*c-1.  Returns (O, LSE) in the same order.  `order`
    optionally replaces the schedule by any list of (j, k) pairs covering each
    pair once."""
    n_seq, d = Qp.shape[0], Vp.shape[1]
    c = n_seq // N
    O = np.zeros((n_seq, d))
    LSE = np.full(n_seq, -np.inf)
    pairs = [(j, k) for _, j, k in ring_schedule(N)] if order is None else order
    for j, k in pairs:
        qs, ks = slice(j * c, (j + 1) * c), slice(k * c, (k + 1) * c)
        O[qs], LSE[qs] = ring_step_fwd(O[qs], LSE[qs], Qp[qs], Kp[ks], Vp[ks],
                                       j, k, N, layout, scale)
    return O, LSE


def ring_step_bwd(dQj, dKk, dVk, Qj, Kk, Vk, dOj, LSEj, deltaj, j, k, N, layout, scale):
    """Gradient contribution of step (j, k), added into dQ_j, dK_k, dV_k (in
    place).  LSEj is the final log-sum-exp of device j's rows, deltaj[a] =
    sum_t dO[a, t] O[a, t] with the final O.  P is recomputed as
    exp(scale q.k - LSE) on the allowed pairs of GetMask(j, k)."""
    Qj = np.asarray(Qj, np.float64)
    Kk = np.asarray(Kk, np.float64)
    Vk = np.asarray(Vk, np.float64)
    dOj = np.asarray(dOj, np.float64)
    c = Qj.shape[0]
    allowed = get_mask(j, k, N, c, layout)
    for a in range(c):
        idx = np.nonzero(allowed[a])[0]
        if len(idx) == 0:
            continue
        p = np.exp(scale * (Kk[idx] @ Qj[a]) - LSEj[a])
        dVk[idx] += np.outer(p, dOj[a])
        ds = p * (Vk[idx] @ dOj[a] - deltaj[a])
        dQj[a] += scale * (ds @ Kk[idx])
        dKk[idx] += scale * np.outer(ds, Qj[a])


def ring_attention_grad(Qp, Kp, Vp, dOp, N, layout, scale):
    """Backward of ring_attention for one head: forward ring for (O, LSE), then
    every (j, k) step's contribution.  Inputs and outputs in device order."""
    n_seq = Qp.shape[0]
    c = n_seq // N
    O, LSE = ring_attention(Qp, Kp, Vp, N, layout, scale)
    delta = (np.asarray(dOp, np.float64) * O).sum(axis=1)
    dQ = np.zeros(Qp.shape)
    dK = np.zeros(Kp.shape)
    dV = np.zeros(Vp.shape)
    for _, j, k in ring_schedule(N):
        qs, ks = slice(j * c, (j + 1) * c), slice(k * c, (k + 1) * c)
        ring_step_bwd(dQ[qs], dK[ks], dV[ks], Qp[qs], Kp[ks], Vp[ks], dOp[qs],
                      LSE[qs], delta[qs], j, k, N, layout, scale)
    return dQ, dK, dV


# --------------------------------------------------------------------------
# Work bookkeeping used for FLOP accounting and the balance claims
# --------------------------------------------------------------------------
def worst_device_work_per_round(N, c, layout):
    """For each round i of Algorithm 1, max over devices j of Work(j, (j-i) mod N)
    (Sec. 1: a round's latency is set by its slowest device)."""
    return [max(work(j, (j - i) % N, N, c, layout) for j in range(N)) for i in range(N)]
