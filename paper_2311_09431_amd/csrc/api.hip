// C ABI of libstriped_attn: argument validation, mask classification, dispatch to
// the kernels, and the single-GPU ring drivers (Algorithm 1 played in sequence).
#include <math.h>

#include <vector>

#include "sa_internal.h"

namespace {

using sa::StepArgs;

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int64_t row_stride(const sa_shape* s) { return s->stride_s > 0 ? s->stride_s : s->d; }

// strides of one [B, heads, rows, d]-like tensor family
struct Geom { int heads; int64_t sb, sh, ss; };
inline Geom q_geom(const sa_shape* s) { return {s->H, s->stride_b, s->stride_h, row_stride(s)}; }
inline bool grouped(const sa_shape* s) { return s->H_kv > 0; }
inline Geom kv_geom(const sa_shape* s) {
    if (!grouped(s)) return q_geom(s);
    return {s->H_kv, s->kv_stride_b, s->kv_stride_h, s->kv_stride_s > 0 ? s->kv_stride_s : s->d};
}

// rows rows per (batch, head) must not overlap each other
int check_geom(const Geom& g, int B, int64_t rows, int d) {
    const int dmul = 4;      // rows are read four elements at a time (16 or 8 bytes)
    if (g.ss < d) return SA_ERR_SHAPE;
    // heads apart ([B, H, rows, d]-like) or interleaved within a row step ([B, rows, H, d]-like)
    const bool heads_apart = g.sh >= rows * g.ss;
    const bool heads_inside = g.sh >= d && g.ss >= (int64_t)g.heads * g.sh;
    if (!heads_apart && !heads_inside) return SA_ERR_SHAPE;
    if (B > 1 && g.sb < (heads_apart ? g.sh : rows * g.ss)) return SA_ERR_SHAPE;
    if (g.sb % dmul || g.sh % dmul || g.ss % dmul) return SA_ERR_ALIGN;
    return SA_OK;
}

int check_shape(const sa_shape* s) {
    if (!s) return SA_ERR_NULL;
    if (s->dtype != SA_F32 && s->dtype != SA_BF16) return SA_ERR_DTYPE;
    if (s->B < 1 || s->H < 1 || s->c < 1 || s->d < 1 || s->d > 256) return SA_ERR_SHAPE;
    if ((int64_t)s->B * s->H > 65535) return SA_ERR_SHAPE;
    if (s->d % 4) return SA_ERR_SHAPE;
    if (s->H_kv < 0 || (grouped(s) && s->H % s->H_kv)) return SA_ERR_SHAPE;
    if (s->stat_stride_h < s->c || (s->B > 1 && s->stat_stride_b < s->stat_stride_h)) return SA_ERR_SHAPE;
    if (int e = check_geom(q_geom(s), s->B, s->c, s->d)) return e;
    if (grouped(s))
        if (int e = check_geom(kv_geom(s), s->B, s->c, s->d)) return e;
    return SA_OK;
}

// the ring drivers address N shards of c rows inside the same tensors
int check_ring_extent(const sa_shape* s, int N) {
    const int64_t rows = (int64_t)N * s->c;
    if (s->stat_stride_h < rows) return SA_ERR_SHAPE;
    if (check_geom(q_geom(s), s->B, rows, s->d) || check_geom(kv_geom(s), s->B, rows, s->d))
        return SA_ERR_SHAPE;
    return SA_OK;
}

int check_step(int q_dev, int kv_dev, int N, int layout) {
    if (N < 1 || q_dev < 0 || q_dev >= N || kv_dev < 0 || kv_dev >= N) return SA_ERR_DEV;
    if (layout != SA_CONTIGUOUS && layout != SA_STRIPED) return SA_ERR_LAYOUT;
    return SA_OK;
}

// GetMask(j, k) in local indices (Sec. 2.2, 2.3): query a = original position
// j*c + a (contiguous) or a*N + j (striped); key b likewise with k.  Allowed iff
// key position <= query position, which reduces to b <= a - off.
void classify(int q_dev, int kv_dev, int layout, int* kind, int* off) {
    *off = 0;
    if (layout == SA_CONTIGUOUS) {
        *kind = q_dev < kv_dev ? sa::MASK_EMPTY : (q_dev == kv_dev ? sa::MASK_TRI : sa::MASK_FULL);
    } else {
        *kind = sa::MASK_TRI;
        *off = kv_dev > q_dev ? 1 : 0;
    }
}

StepArgs make_args(const sa_shape* s) {
    StepArgs a{};
    a.B = s->B; a.H = s->H; a.c = s->c; a.d = s->d;
    a.stride_b = s->stride_b; a.stride_h = s->stride_h;
    a.stat_stride_b = s->stat_stride_b; a.stat_stride_h = s->stat_stride_h;
    a.stride_s = row_stride(s);
    const Geom kv = kv_geom(s);
    a.H_kv = kv.heads; a.kv_stride_b = kv.sb; a.kv_stride_h = kv.sh; a.kv_stride_s = kv.ss;
    a.scale = s->softmax_scale > 0.f ? s->softmax_scale : 1.0f / sqrtf((float)s->d);
    return a;
}

int permute_common(const void* src, void* dst, int64_t outer, int64_t n_seq, int64_t inner_bytes,
                   int N, bool inverse, void* stream) {
    if (N < 1) return SA_ERR_DEV;
    if (outer < 0 || n_seq < 0 || inner_bytes < 1 || n_seq % N) return SA_ERR_SHAPE;
    if (outer == 0 || n_seq == 0) return SA_OK;   // empty: nothing to move, pointers may be NULL
    if (!src || !dst) return SA_ERR_NULL;
    if (src == dst) return SA_ERR_LAYOUT;
    int64_t al = 16;
    while (inner_bytes % al) al >>= 1;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & (uintptr_t)(al - 1))
        return SA_ERR_ALIGN;
    return sa::launch_permute(src, dst, outer, n_seq, inner_bytes, N, inverse, (hipStream_t)stream) ==
                   hipSuccess ? SA_OK : SA_ERR_HIP;
}

// Emulated tile-skipping granularity (Sec. 3.1): both 0 (the kernels' own), or multiples of
// 128 dividing c on a shape the MFMA kernels take.
int check_skip(const sa_shape* s, int bq, int bk) {
    if (bq == 0 && bk == 0) return SA_OK;
    if (bq < 128 || bk < 128 || bq % 128 || bk % 128 || s->c % bq || s->c % bk) return SA_ERR_SHAPE;
    StepArgs a = make_args(s);
    return sa::fwd_mfma_supported(a, s->dtype) && sa::bwd_mfma_supported(a, s->dtype) ? SA_OK
                                                                                      : SA_ERR_SHAPE;
}

int step_fwd(const void* q, const void* k, const void* v, float* o, float* lse, int q_dev, int kv_dev,
             int layout, const sa_shape* s, int bq, int bk, hipStream_t st, const int32_t* q_pos = nullptr,
             int64_t pos_stride_b = 0, float rope_base = 0.f) {
    StepArgs a = make_args(s);
    classify(q_dev, kv_dev, layout, &a.kind, &a.off);
    a.q = q; a.k = k; a.v = v; a.o = o; a.lse = lse;
    a.skip_bq = bq; a.skip_bk = bk;
    if (q_pos) {
        if (!sa::fwd_mfma_rope_supported(a, s->dtype)) return SA_ERR_SHAPE;
        a.q_pos = q_pos; a.pos_stride_b = pos_stride_b; a.rope_log2_base = log2((double)rope_base);
    }
    if (a.kind == sa::MASK_EMPTY) return SA_OK;   // entirely masked block: nothing to launch
    hipError_t e = sa::fwd_mfma_supported(a, s->dtype) ? sa::launch_fwd_mfma(a, st)
                                                       : sa::launch_fwd_generic(a, s->dtype, st);
    return e == hipSuccess ? SA_OK : SA_ERR_HIP;
}

int step_bwd(const void* q, const void* k, const void* v, const void* dout, const float* lse,
             const float* delta, float* dq, float* dk, float* dv, int q_dev, int kv_dev, int layout,
             const sa_shape* s, int bq, int bk, hipStream_t st) {
    StepArgs a = make_args(s);
    classify(q_dev, kv_dev, layout, &a.kind, &a.off);
    if (a.kind == sa::MASK_EMPTY) return SA_OK;
    a.skip_bq = bq; a.skip_bk = bk;
    a.q = q; a.k = k; a.v = v; a.dout = dout; a.lse = const_cast<float*>(lse); a.delta = delta;
    a.dq = dq; a.dk = dk; a.dv = dv;
    hipError_t e = sa::bwd_mfma_supported(a, s->dtype) ? sa::launch_bwd_mfma(a, st)
                                                       : sa::launch_bwd_generic(a, s->dtype, st);
    return e == hipSuccess ? SA_OK : SA_ERR_HIP;
}

size_t elt_size(int dtype) { return dtype == SA_F32 ? 4 : 2; }

// Event bookkeeping for the drivers' optional per-step timings.
struct StepTimer {
    std::vector<hipEvent_t> ev;
    std::vector<int> slot;
    bool on;
    explicit StepTimer(bool enabled) : on(enabled) {}
    bool begin(hipStream_t st, int s) {
        if (!on) return true;
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess) return false;
        if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return false; }
        ev.push_back(a); ev.push_back(b); slot.push_back(s);
        return hipEventRecord(a, st) == hipSuccess;
    }
    bool end(hipStream_t st) { return !on || hipEventRecord(ev.back(), st) == hipSuccess; }
    bool collect(hipStream_t st, float* out) {
        if (!on) return true;
        bool ok = hipStreamSynchronize(st) == hipSuccess;
        for (size_t i = 0; i < slot.size(); ++i) {
            float ms = 0.f;
            if (ok && hipEventElapsedTime(&ms, ev[2 * i], ev[2 * i + 1]) == hipSuccess) out[slot[i]] = ms;
            else ok = false;
        }
        return ok;
    }
    ~StepTimer() { for (hipEvent_t e : ev) (void)hipEventDestroy(e); }
};

}  // namespace

extern "C" {

int sa_stripe_permute(const void* src, void* dst, int64_t outer, int64_t n_seq, int64_t inner_bytes,
                      int32_t N, void* stream) {
    return permute_common(src, dst, outer, n_seq, inner_bytes, N, false, stream);
}

int sa_unstripe_permute(const void* src, void* dst, int64_t outer, int64_t n_seq, int64_t inner_bytes,
                        int32_t N, void* stream) {
    return permute_common(src, dst, outer, n_seq, inner_bytes, N, true, stream);
}

int sa_state_init(float* o, float* lse, const sa_shape* shape, void* stream) {
    if (!o || !lse) return SA_ERR_NULL;
    if (int e = check_shape(shape)) return e;
    if (!aligned16(o)) return SA_ERR_ALIGN;
    return sa::launch_state_init(o, lse, *shape, (hipStream_t)stream) == hipSuccess ? SA_OK : SA_ERR_HIP;
}

int sa_rope(const void* x, void* y, const int32_t* pos, int64_t pos_stride_b, const sa_shape* shape,
            float base, int32_t inverse, void* stream) {
    if (!x || !y || !pos) return SA_ERR_NULL;
    if (int e = check_shape(shape)) return e;
    if (pos_stride_b < 0 || (pos_stride_b > 0 && pos_stride_b < shape->c) || !(base > 1.f)) return SA_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(y) || (reinterpret_cast<uintptr_t>(pos) & 3u)) return SA_ERR_ALIGN;
    return sa::launch_rope(x, y, pos, pos_stride_b, *shape, base, inverse != 0, (hipStream_t)stream) ==
                   hipSuccess ? SA_OK : SA_ERR_HIP;
}

int sa_attn_step_fwd_tiled(const void* q, const void* k, const void* v, float* o, float* lse,
                           int32_t q_dev, int32_t kv_dev, int32_t N, int32_t layout, const sa_shape* shape,
                           int32_t skip_bq, int32_t skip_bk, void* stream) {
    if (!q || !k || !v || !o || !lse) return SA_ERR_NULL;
    if (int e = check_shape(shape)) return e;
    if (int e = check_step(q_dev, kv_dev, N, layout)) return e;
    if (int e = check_skip(shape, skip_bq, skip_bk)) return e;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return SA_ERR_ALIGN;
    return step_fwd(q, k, v, o, lse, q_dev, kv_dev, layout, shape, skip_bq, skip_bk, (hipStream_t)stream);
}

int sa_attn_step_fwd_rope(const void* q, const void* k, const void* v, float* o, float* lse,
                          const int32_t* q_pos, int64_t pos_stride_b, float rope_base, int32_t q_dev,
                          int32_t kv_dev, int32_t N, int32_t layout, const sa_shape* shape, void* stream) {
    if (!q || !k || !v || !o || !lse || !q_pos) return SA_ERR_NULL;
    if (int e = check_shape(shape)) return e;
    if (int e = check_step(q_dev, kv_dev, N, layout)) return e;
    if (pos_stride_b < 0 || (pos_stride_b > 0 && pos_stride_b < shape->c) || !(rope_base > 1.f)) return SA_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) ||
        (reinterpret_cast<uintptr_t>(q_pos) & 3u))
        return SA_ERR_ALIGN;
    return step_fwd(q, k, v, o, lse, q_dev, kv_dev, layout, shape, 0, 0, (hipStream_t)stream, q_pos,
                    pos_stride_b, rope_base);
}

int sa_attn_step_fwd(const void* q, const void* k, const void* v, float* o, float* lse, int32_t q_dev,
                     int32_t kv_dev, int32_t N, int32_t layout, const sa_shape* shape, void* stream) {
    return sa_attn_step_fwd_tiled(q, k, v, o, lse, q_dev, kv_dev, N, layout, shape, 0, 0, stream);
}

int sa_finalize(const float* o, void* out, const sa_shape* shape, void* stream) {
    if (!o || !out) return SA_ERR_NULL;
    if (int e = check_shape(shape)) return e;
    if (!aligned16(o) || !aligned16(out)) return SA_ERR_ALIGN;
    return sa::launch_finalize(o, out, *shape, (hipStream_t)stream) == hipSuccess ? SA_OK : SA_ERR_HIP;
}

int sa_bwd_preprocess(const float* o, const void* dout, float* delta, const sa_shape* shape,
                      void* stream) {
    if (!o || !dout || !delta) return SA_ERR_NULL;
    if (int e = check_shape(shape)) return e;
    if (!aligned16(o) || !aligned16(dout)) return SA_ERR_ALIGN;
    return sa::launch_bwd_preprocess(o, dout, delta, *shape, (hipStream_t)stream) == hipSuccess
               ? SA_OK : SA_ERR_HIP;
}

int sa_attn_step_bwd_tiled(const void* q, const void* k, const void* v, const void* dout,
                           const float* lse, const float* delta, float* dq, float* dk, float* dv,
                           int32_t q_dev, int32_t kv_dev, int32_t N, int32_t layout, const sa_shape* shape,
                           int32_t skip_bq, int32_t skip_bk, void* stream) {
    if (!q || !k || !v || !dout || !lse || !delta || !dq || !dk || !dv) return SA_ERR_NULL;
    if (int e = check_shape(shape)) return e;
    if (int e = check_step(q_dev, kv_dev, N, layout)) return e;
    if (int e = check_skip(shape, skip_bq, skip_bk)) return e;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(dout) || !aligned16(dq) ||
        !aligned16(dk) || !aligned16(dv))
        return SA_ERR_ALIGN;
    return step_bwd(q, k, v, dout, lse, delta, dq, dk, dv, q_dev, kv_dev, layout, shape, skip_bq, skip_bk,
                    (hipStream_t)stream);
}

int sa_attn_step_bwd(const void* q, const void* k, const void* v, const void* dout, const float* lse,
                     const float* delta, float* dq, float* dk, float* dv, int32_t q_dev, int32_t kv_dev,
                     int32_t N, int32_t layout, const sa_shape* shape, void* stream) {
    return sa_attn_step_bwd_tiled(q, k, v, dout, lse, delta, dq, dk, dv, q_dev, kv_dev, N, layout, shape,
                                  0, 0, stream);
}

int sa_ring_fwd_tiled(const void* Q, const void* K, const void* V, float* O, float* LSE, int32_t N,
                      int32_t layout, const sa_shape* shape, int32_t skip_bq, int32_t skip_bk,
                      int32_t q_dev_only, float* step_ms, void* stream) {
    if (!Q || !K || !V || !O || !LSE) return SA_ERR_NULL;
    if (int e = check_shape(shape)) return e;
    if (int e = check_skip(shape, skip_bq, skip_bk)) return e;
    if (N < 1 || q_dev_only >= N) return SA_ERR_DEV;
    if (layout != SA_CONTIGUOUS && layout != SA_STRIPED) return SA_ERR_LAYOUT;
    if (int e = check_ring_extent(shape, N)) return e;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O)) return SA_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const size_t es = elt_size(shape->dtype);
    const int64_t shard = (int64_t)shape->c * row_stride(shape);     // elements between shards
    const int64_t kv_shard = (int64_t)shape->c * kv_geom(shape).ss;  // ... of K and V
    auto in_at = [&](const void* p, int dev) { return (const char*)p + (size_t)dev * shard * es; };
    auto kv_at = [&](const void* p, int dev) { return (const char*)p + (size_t)dev * kv_shard * es; };
    if (step_ms) for (int i = 0; i < N * N; ++i) step_ms[i] = 0.f;
    const int j0 = q_dev_only >= 0 ? q_dev_only : 0, j1 = q_dev_only >= 0 ? q_dev_only + 1 : N;
    for (int j = j0; j < j1; ++j)
        if (sa::launch_state_init(O + j * shard, LSE + (int64_t)j * shape->c, *shape, st) != hipSuccess)
            return SA_ERR_HIP;
    StepTimer timer(step_ms != nullptr);
    for (int i = 0; i < N; ++i) {
        for (int j = j0; j < j1; ++j) {
            const int k = ((j - i) % N + N) % N;            // Algorithm 1: block held in round i
            if (!timer.begin(st, i * N + j)) return SA_ERR_HIP;
            int e = step_fwd(in_at(Q, j), kv_at(K, k), kv_at(V, k), O + j * shard,
                             LSE + (int64_t)j * shape->c, j, k, layout, shape, skip_bq, skip_bk, st);
            if (e) return e;
            if (!timer.end(st)) return SA_ERR_HIP;
        }
    }
    return timer.collect(st, step_ms) ? SA_OK : SA_ERR_HIP;
}

int sa_ring_fwd(const void* Q, const void* K, const void* V, float* O, float* LSE, int32_t N,
                int32_t layout, const sa_shape* shape, int32_t q_dev_only, float* step_ms, void* stream) {
    return sa_ring_fwd_tiled(Q, K, V, O, LSE, N, layout, shape, 0, 0, q_dev_only, step_ms, stream);
}

int sa_ring_bwd_tiled(const void* Q, const void* K, const void* V, const void* dO, const float* O,
                      const float* LSE, float* delta, float* dQ, float* dK, float* dV, int32_t N,
                      int32_t layout, const sa_shape* shape, int32_t skip_bq, int32_t skip_bk,
                      int32_t q_dev_only, float* step_ms, void* stream) {
    if (!Q || !K || !V || !dO || !O || !LSE || !delta || !dQ || !dK || !dV) return SA_ERR_NULL;
    if (int e = check_shape(shape)) return e;
    if (int e = check_skip(shape, skip_bq, skip_bk)) return e;
    if (N < 1 || q_dev_only >= N) return SA_ERR_DEV;
    if (layout != SA_CONTIGUOUS && layout != SA_STRIPED) return SA_ERR_LAYOUT;
    if (int e = check_ring_extent(shape, N)) return e;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(dO) || !aligned16(O) ||
        !aligned16(dQ) || !aligned16(dK) || !aligned16(dV))
        return SA_ERR_ALIGN;
    hipStream_t st = (hipStream_t)stream;
    const size_t es = elt_size(shape->dtype);
    const int64_t shard = (int64_t)shape->c * row_stride(shape);     // elements between shards
    const Geom kvg = kv_geom(shape);
    const int64_t kv_shard = (int64_t)shape->c * kvg.ss;             // ... of K, V, dK, dV
    auto in_at = [&](const void* p, int dev) { return (const char*)p + (size_t)dev * shard * es; };
    auto kv_at = [&](const void* p, int dev) { return (const char*)p + (size_t)dev * kv_shard * es; };
    if (step_ms) for (int i = 0; i < N * N; ++i) step_ms[i] = 0.f;
    const int j0 = q_dev_only >= 0 ? q_dev_only : 0, j1 = q_dev_only >= 0 ? q_dev_only + 1 : N;
    sa_shape kv_shape = *shape;          // dK and dV as a tensor family of their own
    kv_shape.H = kvg.heads; kv_shape.stride_b = kvg.sb; kv_shape.stride_h = kvg.sh; kv_shape.stride_s = kvg.ss;
    for (int dev = 0; dev < N; ++dev) {
        if (sa::launch_zero_f32(dQ + dev * shard, *shape, st) != hipSuccess ||
            sa::launch_zero_f32(dK + dev * kv_shard, kv_shape, st) != hipSuccess ||
            sa::launch_zero_f32(dV + dev * kv_shard, kv_shape, st) != hipSuccess)
            return SA_ERR_HIP;
    }
    for (int j = j0; j < j1; ++j)
        if (sa::launch_bwd_preprocess(O + j * shard, in_at(dO, j), delta + (int64_t)j * shape->c, *shape,
                                      st) != hipSuccess)
            return SA_ERR_HIP;
    StepTimer timer(step_ms != nullptr);
    for (int i = 0; i < N; ++i) {
        for (int j = j0; j < j1; ++j) {
            const int k = ((j - i) % N + N) % N;
            if (!timer.begin(st, i * N + j)) return SA_ERR_HIP;
            int e = step_bwd(in_at(Q, j), kv_at(K, k), kv_at(V, k), in_at(dO, j),
                             LSE + (int64_t)j * shape->c, delta + (int64_t)j * shape->c, dQ + j * shard,
                             dK + k * kv_shard, dV + k * kv_shard, j, k, layout, shape, skip_bq, skip_bk,
                             st);
            if (e) return e;
            if (!timer.end(st)) return SA_ERR_HIP;
        }
    }
    return timer.collect(st, step_ms) ? SA_OK : SA_ERR_HIP;
}

int sa_ring_bwd(const void* Q, const void* K, const void* V, const void* dO, const float* O,
                const float* LSE, float* delta, float* dQ, float* dK, float* dV, int32_t N, int32_t layout,
                const sa_shape* shape, int32_t q_dev_only, float* step_ms, void* stream) {
    return sa_ring_bwd_tiled(Q, K, V, dO, O, LSE, delta, dQ, dK, dV, N, layout, shape, 0, 0, q_dev_only,
                             step_ms, stream);
}

int sa_step_mask(int32_t q_dev, int32_t kv_dev, int32_t N, int32_t layout, int32_t* kind, int32_t* off) {
    if (!kind || !off) return SA_ERR_NULL;
    if (int e = check_step(q_dev, kv_dev, N, layout)) return e;
    int kd, of;
    classify(q_dev, kv_dev, layout, &kd, &of);
    *kind = kd;
    *off = of;
    return SA_OK;
}

int64_t sa_step_pairs(int32_t q_dev, int32_t kv_dev, int32_t N, int32_t layout, int64_t c) {
    if (check_step(q_dev, kv_dev, N, layout) || c < 0) return -1;
    int kind, off;
    classify(q_dev, kv_dev, layout, &kind, &off);
    if (kind == sa::MASK_EMPTY) return 0;
    if (kind == sa::MASK_FULL) return c * c;
    return off ? c * (c - 1) / 2 : c * (c + 1) / 2;
}

int sa_step_tiles(int32_t q_dev, int32_t kv_dev, int32_t N, int32_t layout, int64_t c, int64_t skip_bq,
                  int64_t skip_bk, int64_t* computed, int64_t* total) {
    if (!computed || !total) return SA_ERR_NULL;
    if (int e = check_step(q_dev, kv_dev, N, layout)) return e;
    if (c < 1 || skip_bq < 1 || skip_bk < 1 || c % skip_bq || c % skip_bk) return SA_ERR_SHAPE;
    int kind, off;
    classify(q_dev, kv_dev, layout, &kind, &off);
    const int64_t nq = c / skip_bq, nk = c / skip_bk;
    *total = nq * nk;
    if (kind == sa::MASK_EMPTY) { *computed = 0; return SA_OK; }
    if (kind == sa::MASK_FULL) { *computed = nq * nk; return SA_OK; }
    // tile (r, s) holds an allowed pair iff its first key s*bk <= its last query (r+1)*bq - 1 - off
    int64_t n = 0;
    for (int64_t r = 0; r < nq; ++r) {
        const int64_t last = (r + 1) * skip_bq - 1 - off;       // last key any query of the tile sees
        if (last >= 0) n += (last / skip_bk + 1 < nk) ? last / skip_bk + 1 : nk;
    }
    *computed = n;
    return SA_OK;
}

int sa_device_props(int32_t* compute_units, int32_t* clock_khz, int64_t* memory_bytes) {
    if (!compute_units || !clock_khz || !memory_bytes) return SA_ERR_NULL;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return SA_ERR_HIP;
    *compute_units = prop.multiProcessorCount;
    *clock_khz = prop.clockRate;
    *memory_bytes = (int64_t)prop.totalGlobalMem;
    return SA_OK;
}

const char* sa_status_str(int status) {
    switch (status) {
        case SA_OK: return "ok";
        case SA_ERR_NULL: return "null pointer";
        case SA_ERR_SHAPE: return "bad shape";
        case SA_ERR_DEV: return "device index out of range";
        case SA_ERR_DTYPE: return "unsupported dtype";
        case SA_ERR_LAYOUT: return "bad layout";
        case SA_ERR_ALIGN: return "misaligned pointer or stride";
        case SA_ERR_HIP: return "HIP call failed";
        default: return "unknown status";
    }
}

}  // extern "C"
