// Bandwidth-bound helpers around the ring step: accumulator initialisation
// (Algorithm 1, first line), the final cast (Algorithm 1, "normalize": the running
// output is kept normalised, so only a rounding is left) and the backward
// preprocessing delta = rowsum(dO * O).
#include <hip/hip_bf16.h>

#include "sa_internal.h"

namespace sa {

// grid: (row blocks, B*H); each thread handles 4 floats of a row; rows are ss elements apart.
__global__ void __launch_bounds__(256)
state_init_kernel(float* __restrict__ o, float* __restrict__ lse, int H, int c, int d,
                  int64_t sb, int64_t sh, int64_t ss, int64_t ssb, int64_t ssh, float lse_value,
                  bool touch_lse) {
    const int bh = blockIdx.y, b = bh / H, h = bh - b * H;
    float* ob = o + b * sb + h * sh;
    const int d4 = d / 4;
    const int64_t n4 = (int64_t)c * d4;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) {
        const int64_t row = i / d4;
        *reinterpret_cast<float4*>(ob + row * ss + (i - row * d4) * 4) = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if (touch_lse) {
        float* lb = lse + b * ssb + h * ssh;
        for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < c; i += (int64_t)gridDim.x * 256)
            lb[i] = lse_value;
    }
}

static unsigned row_blocks(int64_t work_items) {
    int64_t g = (work_items + 255) / 256;
    if (g > 4096) g = 4096;
    if (g < 1) g = 1;
    return (unsigned)g;
}

static int64_t row_stride(const sa_shape& s) { return s.stride_s > 0 ? s.stride_s : s.d; }

hipError_t launch_state_init(float* o, float* lse, const sa_shape& s, hipStream_t st) {
    dim3 grid(row_blocks((int64_t)s.c * s.d / 4), s.B * s.H);
    hipLaunchKernelGGL(state_init_kernel, grid, dim3(256), 0, st, o, lse, s.H, s.c, s.d, s.stride_b,
                       s.stride_h, row_stride(s), s.stat_stride_b, s.stat_stride_h, -INFINITY, true);
    return hipGetLastError();
}

hipError_t launch_zero_f32(float* p, const sa_shape& s, hipStream_t st) {
    dim3 grid(row_blocks((int64_t)s.c * s.d / 4), s.B * s.H);
    hipLaunchKernelGGL(state_init_kernel, grid, dim3(256), 0, st, p, (float*)nullptr, s.H, s.c, s.d,
                       s.stride_b, s.stride_h, row_stride(s), (int64_t)0, (int64_t)0, 0.f, false);
    return hipGetLastError();
}

template <typename OutT>
__device__ inline void store4(OutT* p, float4 v);
template <>
__device__ inline void store4<float>(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
template <>
__device__ inline void store4<__hip_bfloat16>(__hip_bfloat16* p, float4 v) {
    __hip_bfloat16 t[4] = {__float2bfloat16(v.x), __float2bfloat16(v.y), __float2bfloat16(v.z),
                           __float2bfloat16(v.w)};
    *reinterpret_cast<uint2*>(p) = *reinterpret_cast<uint2*>(t);
}

template <typename OutT>
__global__ void __launch_bounds__(256)
finalize_kernel(const float* __restrict__ o, OutT* __restrict__ out, int H, int c, int d, int64_t sb,
                int64_t sh, int64_t ss) {
    const int bh = blockIdx.y, b = bh / H, h = bh - b * H;
    const float* ob = o + b * sb + h * sh;
    OutT* yb = out + b * sb + h * sh;
    const int d4 = d / 4;
    const int64_t n4 = (int64_t)c * d4;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) {
        const int64_t row = i / d4, at = row * ss + (i - row * d4) * 4;
        store4<OutT>(yb + at, *reinterpret_cast<const float4*>(ob + at));
    }
}

hipError_t launch_finalize(const float* o, void* out, const sa_shape& s, hipStream_t st) {
    dim3 grid(row_blocks((int64_t)s.c * s.d / 4), s.B * s.H);
    if (s.dtype == SA_F32)
        hipLaunchKernelGGL(finalize_kernel<float>, grid, dim3(256), 0, st, o, (float*)out, s.H, s.c,
                           s.d, s.stride_b, s.stride_h, row_stride(s));
    else
        hipLaunchKernelGGL(finalize_kernel<__hip_bfloat16>, grid, dim3(256), 0, st, o,
                           (__hip_bfloat16*)out, s.H, s.c, s.d, s.stride_b, s.stride_h, row_stride(s));
    return hipGetLastError();
}

template <typename T>
__device__ inline float4 load4(const T* p);
template <>
__device__ inline float4 load4<float>(const float* p) { return *reinterpret_cast<const float4*>(p); }
template <>
__device__ inline float4 load4<__hip_bfloat16>(const __hip_bfloat16* p) {
    uint2 raw = *reinterpret_cast<const uint2*>(p);
    float4 r;
    r.x = __uint_as_float(raw.x << 16);
    r.y = __uint_as_float(raw.x & 0xffff0000u);
    r.z = __uint_as_float(raw.y << 16);
    r.w = __uint_as_float(raw.y & 0xffff0000u);
    return r;
}

// One 16-lane group per row (d/4 <= 64 float4 per row, strided over the group);
// a 256-thread block covers 16 rows.
template <typename T>
__global__ void __launch_bounds__(256)
bwd_preprocess_kernel(const float* __restrict__ o, const T* __restrict__ dout, float* __restrict__ delta,
                      int H, int c, int d, int64_t sb, int64_t sh, int64_t ss, int64_t ssb, int64_t ssh) {
    const int bh = blockIdx.y, b = bh / H, h = bh - b * H;
    const int g = threadIdx.x >> 4, l = threadIdx.x & 15;
    for (int64_t row = (int64_t)blockIdx.x * 16 + g; row < c; row += (int64_t)gridDim.x * 16) {
        const float* orow = o + b * sb + h * sh + row * ss;
        const T* grow = dout + b * sb + h * sh + row * ss;
        float acc = 0.f;
        for (int t = l * 4; t < d; t += 64) {
            float4 x = *reinterpret_cast<const float4*>(orow + t);
            float4 y = load4<T>(grow + t);
            acc += x.x * y.x + x.y * y.y + x.z * y.z + x.w * y.w;
        }
        acc += __shfl_xor(acc, 8, 16);
        acc += __shfl_xor(acc, 4, 16);
        acc += __shfl_xor(acc, 2, 16);
        acc += __shfl_xor(acc, 1, 16);
        if (l == 0) delta[b * ssb + h * ssh + row] = acc;
    }
}

hipError_t launch_bwd_preprocess(const float* o, const void* dout, float* delta, const sa_shape& s,
                                 hipStream_t st) {
    int64_t g = ((int64_t)s.c + 15) / 16;
    if (g > 8192) g = 8192;
    dim3 grid((unsigned)g, s.B * s.H);
    if (s.dtype == SA_F32)
        hipLaunchKernelGGL(bwd_preprocess_kernel<float>, grid, dim3(256), 0, st, o, (const float*)dout,
                           delta, s.H, s.c, s.d, s.stride_b, s.stride_h, row_stride(s), s.stat_stride_b,
                           s.stat_stride_h);
    else
        hipLaunchKernelGGL(bwd_preprocess_kernel<__hip_bfloat16>, grid, dim3(256), 0, st, o,
                           (const __hip_bfloat16*)dout, delta, s.H, s.c, s.d, s.stride_b, s.stride_h,
                           row_stride(s), s.stat_stride_b, s.stat_stride_h);
    return hipGetLastError();
}

// Rotary position embedding with explicit position ids (Sec. 2.3: with the striped layout the
// ids are permuted together with the tokens, so row a of device dev carries id a N + dev).
// A thread owns two neighbouring pairs (x_i, x_{i+d/2}) of one row and keeps their sines and
// cosines, computed in double precision (ids reach 10^6, where an fp32 angle is off by 0.05
// rad), across all heads (and batches, when they share the ids).
template <typename T>
__device__ inline float2 ld2(const T* p);
template <>
__device__ inline float2 ld2<float>(const float* p) { return *reinterpret_cast<const float2*>(p); }
template <>
__device__ inline float2 ld2<__hip_bfloat16>(const __hip_bfloat16* p) {
    const uint32_t raw = *reinterpret_cast<const uint32_t*>(p);
    return make_float2(__uint_as_float(raw << 16), __uint_as_float(raw & 0xffff0000u));
}
template <typename T>
__device__ inline void st2(T* p, float2 v);
template <>
__device__ inline void st2<float>(float* p, float2 v) { *reinterpret_cast<float2*>(p) = v; }
template <>
__device__ inline void st2<__hip_bfloat16>(__hip_bfloat16* p, float2 v) {
    __hip_bfloat16 t[2] = {__float2bfloat16(v.x), __float2bfloat16(v.y)};
    *reinterpret_cast<uint32_t*>(p) = *reinterpret_cast<uint32_t*>(t);
}

template <typename T>
__global__ void __launch_bounds__(256)
rope_kernel(const T* __restrict__ x, T* __restrict__ y, const int32_t* __restrict__ pos, int64_t pos_sb,
            int B, int H, int c, int d, int64_t sb, int64_t sh, int64_t ss, double log2_base, bool inverse) {
    const int half = d / 2, per_row = half / 2;          // two pairs per thread
    const int64_t total = (int64_t)c * per_row;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        const int64_t row = idx / per_row;
        const int i = 2 * (int)(idx - row * per_row);
        const double f0 = exp2(-2.0 * i / d * log2_base), f1 = exp2(-2.0 * (i + 1) / d * log2_base);
        double s0 = 0., c0 = 1., s1 = 0., c1 = 1.;
        for (int b = 0; b < B; ++b) {
            if (b == 0 || pos_sb != 0) {
                const double p = (double)pos[b * pos_sb + row];
                sincos(p * f0, &s0, &c0);
                sincos(p * f1, &s1, &c1);
                if (inverse) { s0 = -s0; s1 = -s1; }
            }
            const float cf0 = (float)c0, sf0 = (float)s0, cf1 = (float)c1, sf1 = (float)s1;
            for (int h = 0; h < H; ++h) {
                const int64_t at = b * sb + h * sh + row * ss + i;
                const float2 lo = ld2<T>(x + at), hi = ld2<T>(x + at + half);
                st2<T>(y + at, make_float2(lo.x * cf0 - hi.x * sf0, lo.y * cf1 - hi.y * sf1));
                st2<T>(y + at + half, make_float2(hi.x * cf0 + lo.x * sf0, hi.y * cf1 + lo.y * sf1));
            }
        }
    }
}

hipError_t launch_rope(const void* x, void* y, const int32_t* pos, int64_t pos_stride_b, const sa_shape& s,
                       float base, bool inverse, hipStream_t st) {
    const int64_t total = (int64_t)s.c * (s.d / 4);
    dim3 grid(row_blocks(total));
    const double l2b = log2((double)base);
    if (s.dtype == SA_F32)
        hipLaunchKernelGGL(rope_kernel<float>, grid, dim3(256), 0, st, (const float*)x, (float*)y, pos,
                           pos_stride_b, s.B, s.H, s.c, s.d, s.stride_b, s.stride_h, row_stride(s), l2b, inverse);
    else
        hipLaunchKernelGGL(rope_kernel<__hip_bfloat16>, grid, dim3(256), 0, st, (const __hip_bfloat16*)x,
                           (__hip_bfloat16*)y, pos, pos_stride_b, s.B, s.H, s.c, s.d, s.stride_b, s.stride_h,
                           row_stride(s), l2b, inverse);
    return hipGetLastError();
}

}  // namespace sa
