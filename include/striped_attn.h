/*
 * striped_attn.h - C ABI of the MI355X (gfx950) ring-step library for Striped
 * Attention (arxiv 2311.09431) and the contiguous Ring Attention layout it is
 * compared with.
 *
 * Conventions common to every entry point
 *  - All tensor pointers are DEVICE pointers unless a parameter says "host".
 *    The caller owns every buffer; the library allocates no device memory.
 *  - Q/K/V/dO/O/dQ/dK/dV are indexed [batch, head, row, 0..d) with d contiguous;
 *    batch, head and row strides are given in elements and are the same for all
 *    of them (K, V, dK, dV take their own when sa_shape.H_kv is set), so both
 *    [B, H, rows, d] (stride_s = d) and [B, rows, H, d] (stride_h = d,
 *    stride_s = H d) memory orders work.  A device's shard of c
 *    rows is a row offset into such a tensor.  LSE and delta are [B, H, rows]
 *    fp32 (rows contiguous) with their own batch/head strides.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls only enqueue work; they do not synchronise, except sa_ring_fwd /
 *    sa_ring_bwd when asked for per-step timings.
 *  - Return value: SA_OK (0) or a negative sa_status.  Arguments are validated
 *    before anything is enqueued: on every error except SA_ERR_HIP nothing has
 *    been launched.  SA_ERR_HIP from a single-kernel entry point means its launch
 *    failed; from the ring drivers (and from a backward step, which is several
 *    launches) it can come after earlier kernels were enqueued, and the read-
 *    modify-write outputs (O, LSE, dQ, dK, dV) are then undefined.  No entry
 *    point throws.
 *  - Pointers must be aligned to 16 bytes (permutes: to min(16, inner_bytes
 *    rounded down to a power of two)).
 *  - Notation follows the paper: N devices, block size c = n_seq / N, query
 *    device j = q_dev, key/value device k = kv_dev.
 */
#ifndef STRIPED_ATTN_H
#define STRIPED_ATTN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SA_OK = 0,
    SA_ERR_NULL = -1,    /* a required pointer is NULL */
    SA_ERR_SHAPE = -2,   /* non-positive size, n_seq % N != 0, unsupported d, bad stride */
    SA_ERR_DEV = -3,     /* q_dev or kv_dev outside [0, N) or N < 1 */
    SA_ERR_DTYPE = -4,   /* dtype not SA_F32 / SA_BF16 */
    SA_ERR_LAYOUT = -5,  /* layout not SA_CONTIGUOUS / SA_STRIPED, or src == dst in a permute */
    SA_ERR_ALIGN = -6,   /* pointer or stride not aligned as required */
    SA_ERR_HIP = -7      /* a HIP call failed (the HIP error is left pending) */
} sa_status;

typedef enum { SA_CONTIGUOUS = 0, SA_STRIPED = 1 } sa_layout;
typedef enum { SA_F32 = 0, SA_BF16 = 1 } sa_dtype;

/* Shape of one device's shard as seen by a ring step. */
typedef struct {
    int32_t B, H;          /* batch, heads */
    int32_t c;             /* rows per device (block size) */
    int32_t d;             /* head dimension: any multiple of 4 up to 256 (Table 1's
                              models have 128 and 100);
                              bf16 with c >= 128 (and d a multiple of 8 when d > 128) takes
                              the MFMA kernels, which compute 64 columns for d <= 64, 112 for
                              d <= 112, 128 for d <= 128 and 256 above; the
                              columns beyond d are zeros on both sides of every product:
                              nothing that follows a row's d elements in memory is read
                              into a result, and nothing beyond them is written) */
    int64_t stride_b;      /* elements between batches in Q/K/V/dO/O/dQ/dK/dV */
    int64_t stride_h;      /* elements between heads in the same tensors */
    int64_t stride_s;      /* elements between consecutive rows; 0 selects d.  A multiple of 4,
                              >= d.  Either stride_h >= c * stride_s (heads apart) or
                              stride_s >= H * stride_h (heads interleaved within a row step) */
    int64_t stat_stride_b; /* elements between batches in LSE / delta */
    int64_t stat_stride_h; /* elements between heads in LSE / delta */
    int32_t dtype;         /* sa_dtype of Q/K/V/dO (O, LSE, delta, dQ, dK, dV are fp32) */
    float softmax_scale;   /* multiplies q.k inside the softmax; <= 0 selects 1/sqrt(d) */
    /* Fewer key/value heads than query heads (grouped-query and multi-query attention; an
       extension, the paper's models have H_kv = H).  H_kv = 0 means H, and then K, V, dK, dV
       have the strides above and the three fields below are not looked at.  H_kv > 0 must
       divide H; query head h reads key/value head h / (H / H_kv), and K, V, dK, dV are
       [B, H_kv, c, d]-shaped with the strides below, under the same rules as stride_b,
       stride_h, stride_s (with H_kv for H).  Q, dO, O, dQ, LSE and delta keep H heads and the
       strides above.  Only the step and ring entry points look at these fields. */
    int32_t H_kv;
    int64_t kv_stride_b;
    int64_t kv_stride_h;
    int64_t kv_stride_s;   /* 0 selects d */
} sa_shape;

/*
 * Stripe permutation (Sec. 2.3: token t goes to device t mod N; realised as a
 * permutation followed by a contiguous split).  src and dst are [outer, n_seq,
 * inner_bytes] byte arrays; dst[o, (t mod N) * c + t div N, :] = src[o, t, :]
 * with c = n_seq / N.  Serves Q/K/V rows as well as token ids, position ids and
 * targets.  Bit-exact byte movement.  src and dst must not overlap.  outer == 0
 * or n_seq == 0 is a successful no-op (pointers are then not looked at).
 * Errors: NULL, n_seq % N != 0 or sizes <= 0 (SHAPE), N < 1 (DEV), src == dst
 * (LAYOUT), misalignment (ALIGN).
 */
int sa_stripe_permute(const void* src, void* dst, int64_t outer, int64_t n_seq,
                      int64_t inner_bytes, int32_t N, void* stream);

/* Inverse of sa_stripe_permute: dst[o, t, :] = src[o, (t mod N) * c + t div N, :]. */
int sa_unstripe_permute(const void* src, void* dst, int64_t outer, int64_t n_seq,
                        int64_t inner_bytes, int32_t N, void* stream);

/*
 * Rotary position embedding with explicit position ids.  Sec. 2.3: when the tokens are
 * stripe-permuted the position ids are permuted with them (the same sa_stripe_permute call on
 * the id array), so that row a of device dev keeps the id a * N + dev of its original place.
 * y[b, h, r, :] = x[b, h, r, :] with every pair (x_i, x_{i + d/2}), i < d/2, rotated by the
 * angle pos[b, r] * base^(-2 i / d) (by the negative angle if inverse != 0: the transpose,
 * which takes gradients back).  x and y have `shape`'s dtype and strides, shape->c rows; y
 * may be x.  pos: device int32 [B, c], batches pos_stride_b elements apart (0: one id row
 * shared by all batches).  Angles are formed in double precision.
 * Errors: NULL, SHAPE (as sa_shape, or base <= 1, or 0 < pos_stride_b < c), ALIGN.
 */
int sa_rope(const void* x, void* y, const int32_t* pos, int64_t pos_stride_b, const sa_shape* shape,
            float base, int32_t inverse, void* stream);

/*
 * Initialise a device's output accumulator (Algorithm 1, first line): O = 0,
 * LSE = -inf.  o is fp32 [B, H, c, d], lse fp32 [B, H, c], strides from `shape`.
 */
int sa_state_init(float* o, float* lse, const sa_shape* shape, void* stream);

/*
 * One ring step, forward (Algorithm 1, AccumulateAttentionFragment): the c query
 * rows of device q_dev attend to the c key/value rows of device kv_dev under
 * GetMask(q_dev, kv_dev) and the result is folded into the running (o, lse):
 *   lse' = log(exp(lse) + sum_allowed exp(scale q.k)),
 *   o'   = (exp(lse - lse') o + sum_allowed exp(scale q.k - lse') v).
 * The mask is causal in the ORIGINAL token order (Sec. 2.1, 2.3).  With local
 * rows a (query) and b (key): contiguous layout (Sec. 2.2): q_dev < kv_dev
 * nothing allowed (no launch), q_dev == kv_dev allowed iff b <= a, q_dev >
 * kv_dev everything allowed; striped layout (Sec. 2.3): kv_dev <= q_dev allowed
 * iff b <= a, kv_dev > q_dev allowed iff b < a.  Tiles without an allowed pair
 * are skipped (Sec. 2.2.1).
 * q, k, v: shard pointers of dtype shape->dtype; o, lse: fp32, read and written.
 * Rows that see no key keep their state (o = 0, lse = -inf if never touched).
 */
int sa_attn_step_fwd(const void* q, const void* k, const void* v, float* o, float* lse,
                     int32_t q_dev, int32_t kv_dev, int32_t N, int32_t layout,
                     const sa_shape* shape, void* stream);

/*
 * sa_attn_step_fwd with the rotary embedding of the QUERY rows fused into their load (Sec. 2.3:
 * every token keeps the position id of its original place, so device q_dev's row a carries
 * id a * N + q_dev under the striped layout; the ids come from running sa_stripe_permute on
 * 0..n_seq-1).  q holds UNROTATED rows; they are rotated as sa_rope would (same pairing, angle
 * q_pos[b, a] * rope_base^(-2 i / d), reduced in double precision, result rounded once to
 * bf16) on their way into the matrix-core operands and nothing is written back.  k must hold
 * rows already rotated by sa_rope: a key shard is read by every query tile, so rotating it once
 * per shard is the cheaper place.  q_pos: device int32 [B, c], pos_stride_b elements between
 * batches (0: one id row shared by all batches).  Forward only: the backward kernels stream Q
 * through LDS in both products and take rotated tensors from sa_rope.
 * Shapes: bf16, d = 64 or 128, c a multiple of 128 (the matrix-core forward kernel); anything
 * else returns SA_ERR_SHAPE.  Other arguments and errors as sa_attn_step_fwd and sa_rope.
 */
int sa_attn_step_fwd_rope(const void* q, const void* k, const void* v, float* o, float* lse,
                          const int32_t* q_pos, int64_t pos_stride_b, float rope_base, int32_t q_dev,
                          int32_t kv_dev, int32_t N, int32_t layout, const sa_shape* shape, void* stream);

/*
 * End of the ring (Algorithm 1, "normalize"): the running o is kept normalised,
 * so this only rounds fp32 o to `shape->dtype` into `out` (same strides).
 */
int sa_finalize(const float* o, void* out, const sa_shape* shape, void* stream);

/*
 * Backward preprocessing: delta[b, h, a] = sum_t dout[b, h, a, t] * o[b, h, a, t]
 * with the FINAL fp32 o of the forward ring.  (The paper gives no backward
 * pass; this and sa_attn_step_bwd are the analytic gradient of Sec. 2.1.)
 */
int sa_bwd_preprocess(const float* o, const void* dout, float* delta, const sa_shape* shape,
                      void* stream);

/*
 * One ring step, backward.  With P = exp(scale q.k - lse) on the allowed pairs of
 * GetMask(q_dev, kv_dev) (same rule as the forward step; lse and delta are the
 * FINAL values for device q_dev's rows):
 *   dv += P^T dout,  dS = P * (dout v^T - delta),  dq += scale dS k,  dk += scale dS^T q.
 * dq (rows of q_dev), dk, dv (rows of kv_dev) are fp32 accumulators, read and
 * written; the caller zeroes them before the first step.
 */
int sa_attn_step_bwd(const void* q, const void* k, const void* v, const void* dout,
                     const float* lse, const float* delta, float* dq, float* dk, float* dv,
                     int32_t q_dev, int32_t kv_dev, int32_t N, int32_t layout,
                     const sa_shape* shape, void* stream);

/*
 * Ring driver, forward (Algorithm 1 played on one GPU): for round i = 0..N-1 and
 * device j = 0..N-1, k = (j - i) mod N, run sa_attn_step_fwd on shard j of Q/O/LSE
 * and shard k of K/V.  Q, K, V, O are full [B, H, N*c, d] tensors in device order
 * (stripe-permuted for SA_STRIPED), LSE is [B, H, N*c]; `shape` describes one
 * shard (c rows) and the strides of the full tensors.  O and LSE are initialised
 * here.  q_dev_only >= 0 plays only that device's N steps (one device's share).
 * step_ms: NULL, or a HOST array of N*N floats receiving the duration of step
 * (round i, device j) at [i*N + j] in milliseconds (steps not played: 0); when
 * non-NULL the call synchronises the stream before returning.
 */
int sa_ring_fwd(const void* Q, const void* K, const void* V, float* O, float* LSE, int32_t N,
                int32_t layout, const sa_shape* shape, int32_t q_dev_only, float* step_ms,
                void* stream);

/*
 * Ring driver, backward: delta = rowsum(dO * O) for the played devices, then the
 * same schedule calling sa_attn_step_bwd.  dQ, dK, dV are full fp32 tensors,
 * zeroed here.  With q_dev_only >= 0 only that device's steps are played (dQ is
 * then complete for that device; dK/dV hold only its contributions).
 */
int sa_ring_bwd(const void* Q, const void* K, const void* V, const void* dO, const float* O,
                const float* LSE, float* delta, float* dQ, float* dK, float* dV, int32_t N,
                int32_t layout, const sa_shape* shape, int32_t q_dev_only, float* step_ms,
                void* stream);

/*
 * Emulated tile-skipping granularity (Sec. 3.1, 3.2: the paper's implementation skips work
 * per 2048 x 4096 or 2048 x 2048 tile of a block).  The *_tiled variants compute the SAME
 * result as sa_attn_step_fwd / sa_attn_step_bwd / sa_ring_fwd / sa_ring_bwd, bit for bit,
 * but do the work of a skip_bq (queries) x skip_bk (keys) tile in full as soon as the tile
 * holds one allowed pair (masked elements inside contribute exact zeros), and skip it only
 * if it holds none.  They exist to measure what striping gains at a given granularity, to
 * set beside the paper's tables; skip_bq = skip_bk = 0 selects the kernels' own granularity
 * (32 x 32) and is what the plain entry points do.  Otherwise both must be multiples of 128
 * that divide c, and the shape must be one the MFMA kernels take (bf16, see sa_shape.d,
 * c % 128 == 0); anything else returns SA_ERR_SHAPE.  All other arguments as in the plain
 * entry points.
 */
int sa_attn_step_fwd_tiled(const void* q, const void* k, const void* v, float* o, float* lse,
                           int32_t q_dev, int32_t kv_dev, int32_t N, int32_t layout,
                           const sa_shape* shape, int32_t skip_bq, int32_t skip_bk, void* stream);
int sa_attn_step_bwd_tiled(const void* q, const void* k, const void* v, const void* dout,
                           const float* lse, const float* delta, float* dq, float* dk, float* dv,
                           int32_t q_dev, int32_t kv_dev, int32_t N, int32_t layout,
                           const sa_shape* shape, int32_t skip_bq, int32_t skip_bk, void* stream);
int sa_ring_fwd_tiled(const void* Q, const void* K, const void* V, float* O, float* LSE, int32_t N,
                      int32_t layout, const sa_shape* shape, int32_t skip_bq, int32_t skip_bk,
                      int32_t q_dev_only, float* step_ms, void* stream);
int sa_ring_bwd_tiled(const void* Q, const void* K, const void* V, const void* dO, const float* O,
                      const float* LSE, float* delta, float* dQ, float* dK, float* dV, int32_t N,
                      int32_t layout, const sa_shape* shape, int32_t skip_bq, int32_t skip_bk,
                      int32_t q_dev_only, float* step_ms, void* stream);

/*
 * Host-only helpers (no GPU work).
 * sa_step_mask: the step's mask, GetMask(q_dev, kv_dev) of Sec. 2.2 / 2.3 in local
 * indices.  Writes both outputs: *kind = 0 empty (nothing allowed) / 1 triangular (key b
 * allowed for query a iff b <= a - *off) / 2 full (everything allowed), and *off = 0 or 1
 * (0 unless the block is triangular).  Errors: NULL, DEV, LAYOUT.
 * sa_step_pairs: number of allowed (query, key) pairs of the step, i.e. Work(j, k)
 * of Sec. 2.3 for the striped layout and c^2 / c(c+1)/2 / 0 for the contiguous one.
 */
int sa_step_mask(int32_t q_dev, int32_t kv_dev, int32_t N, int32_t layout, int32_t* kind,
                 int32_t* off);
int64_t sa_step_pairs(int32_t q_dev, int32_t kv_dev, int32_t N, int32_t layout, int64_t c);
/*
 * sa_step_tiles: the step's c x c block cut into skip_bq x skip_bk tiles (Sec. 2.2.1): *total =
 * number of tiles, *computed = those with at least one allowed pair (the rest are skipped,
 * Sec. 3.1).  Any positive sizes dividing c.  Errors: NULL, DEV, LAYOUT, SHAPE.
 */
int sa_step_tiles(int32_t q_dev, int32_t kv_dev, int32_t N, int32_t layout, int64_t c,
                  int64_t skip_bq, int64_t skip_bk, int64_t* computed, int64_t* total);

/*
 * Host-only: compute units, peak engine clock (kHz) and device memory (bytes) of the current
 * HIP device, as hipGetDeviceProperties reports them; the benchmark prints them beside the
 * peak it prices against.  Errors: NULL, HIP.
 */
int sa_device_props(int32_t* compute_units, int32_t* clock_khz, int64_t* memory_bytes);

/* Human-readable name of a status code; never NULL. */
const char* sa_status_str(int status);

#ifdef __cplusplus
}
#endif
#endif /* STRIPED_ATTN_H */
