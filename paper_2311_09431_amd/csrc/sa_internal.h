// Internal declarations shared by the HIP translation units of libstriped_attn.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "striped_attn.h"

namespace sa {

// Mask of one ring step in local indices: key b is allowed for query a iff
// b <= a - off (kind == TRI) or always (kind == FULL).  Derived from the
// original token positions: striped a*N + dev, contiguous dev*c + a.
enum MaskKind : int { MASK_EMPTY = 0, MASK_TRI = 1, MASK_FULL = 2 };

struct StepArgs {
    const void* q;
    const void* k;
    const void* v;
    const void* dout;     // backward only
    float* o;             // forward: running output
    float* lse;           // forward: running log-sum-exp; backward: final (read-only)
    const float* delta;   // backward only
    float* dq;
    float* dk;
    float* dv;
    int B, H, c, d;
    int64_t stride_b, stride_h, stat_stride_b, stat_stride_h;
    int64_t stride_s;     // elements between consecutive rows (>= d)
    // K, V, dK, dV: H_kv heads (H_kv divides H; query head h reads head h / (H / H_kv)) with
    // strides of their own; equal to H and the strides above for plain multi-head attention
    int H_kv;
    int64_t kv_stride_b, kv_stride_h, kv_stride_s;
    // dK/dV kernels run once per member of a group of H / H_kv query heads: this launch takes
    // query head kv_head * (H / H_kv) + member
    int member;
    float scale;
    int kind;             // MaskKind (never MASK_EMPTY at launch)
    int off;              // 0 or 1 when kind == MASK_TRI
    // Emulated tile-skipping granularity (Sec. 3.1), MFMA kernels only: 0 = the kernel's own
    // (32 x 32); otherwise every sub-tile of a skip_bq x skip_bk tile of the block that holds
    // at least one allowed pair is computed (masked elements contribute exact zeros).
    // Both are multiples of 128 that divide c.
    int skip_bq, skip_bk;
    // Forward only, MFMA kernels only: rotary embedding of the QUERY rows applied while they
    // are loaded (q holds unrotated rows; k is expected rotated already).  q_pos: position ids
    // of the c query rows per batch (int32, pos_stride_b elements between batches, 0 = shared),
    // NULL = no rotation.  rope_log2_base = log2 of the frequency base.
    const int32_t* q_pos;
    int64_t pos_stride_b;
    double rope_log2_base;
};

// launchers: return hipSuccess or the launch error
hipError_t launch_permute(const void* src, void* dst, int64_t outer, int64_t n_seq,
                          int64_t inner_bytes, int N, bool inverse, hipStream_t st);
hipError_t launch_state_init(float* o, float* lse, const sa_shape& s, hipStream_t st);
hipError_t launch_finalize(const float* o, void* out, const sa_shape& s, hipStream_t st);
hipError_t launch_bwd_preprocess(const float* o, const void* dout, float* delta,
                                 const sa_shape& s, hipStream_t st);
hipError_t launch_zero_f32(float* p, const sa_shape& s, hipStream_t st);
hipError_t launch_rope(const void* x, void* y, const int32_t* pos, int64_t pos_stride_b, const sa_shape& s,
                       float base, bool inverse, hipStream_t st);

hipError_t launch_fwd_generic(const StepArgs& a, int dtype, hipStream_t st);
hipError_t launch_bwd_generic(const StepArgs& a, int dtype, hipStream_t st);
bool fwd_mfma_supported(const StepArgs& a, int dtype);
bool fwd_mfma_rope_supported(const StepArgs& a, int dtype);
hipError_t launch_fwd_mfma(const StepArgs& a, hipStream_t st);
bool bwd_mfma_supported(const StepArgs& a, int dtype);
hipError_t launch_bwd_mfma(const StepArgs& a, hipStream_t st);

}  // namespace sa
