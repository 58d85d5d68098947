// Generic ring-step kernels in plain fp32 arithmetic (no matrix cores): any head
// dimension up to 256, any block size, fp32 or bf16 inputs.  They serve the fp32
// configuration (error budget 1e-5, so no reduced-precision products and the
// accurate expf/logf) and every shape the MFMA kernels do not take.
//
// One wavefront owns one query row (forward, dQ) or one key row (dK/dV) at a
// time; the 64 lanes span 64 rows of the other operand.  Accumulation over the
// ring is deterministic: each output row is read-modify-written by one wave.
#include <hip/hip_bf16.h>

#include "sa_internal.h"

namespace sa {

namespace {

constexpr int kWaves = 4;          // waves per block
constexpr int kRowsPerWave = 4;    // rows handled one after another by a wave
constexpr int kMaxD = 256;

template <typename T>
__device__ inline float ld(const T* p);
template <>
__device__ inline float ld<float>(const float* p) { return *p; }
template <>
__device__ inline float ld<__hip_bfloat16>(const __hip_bfloat16* p) {
    return __uint_as_float((uint32_t)(*reinterpret_cast<const uint16_t*>(p)) << 16);
}

__device__ inline float wave_max(float x) {
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}
__device__ inline float wave_sum(float x) {
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// dot product of an fp32 row held in LDS with a row in global memory
template <typename T>
__device__ inline float dot_row(const float* __restrict__ a_lds, const T* __restrict__ g, int d) {
    float s = 0.f;
    for (int t = 0; t < d; t += 4) {
        s = fmaf(a_lds[t + 0], ld<T>(g + t + 0), s);
        s = fmaf(a_lds[t + 1], ld<T>(g + t + 1), s);
        s = fmaf(a_lds[t + 2], ld<T>(g + t + 2), s);
        s = fmaf(a_lds[t + 3], ld<T>(g + t + 3), s);
    }
    return s;
}

// number of keys query row a may see: keys 0 .. n-1
__device__ inline int keys_for_query(int a, int c, int kind, int off) {
    if (kind == MASK_FULL) return c;
    int n = a - off + 1;
    return n < 0 ? 0 : (n > c ? c : n);
}

template <typename T>
__global__ void __launch_bounds__(kWaves * 64)
fwd_generic_kernel(StepArgs p) {
    __shared__ float q_lds[kWaves][kMaxD];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int bh = blockIdx.y, b = bh / p.H, h = bh - b * p.H;
    const int64_t base = b * p.stride_b + h * p.stride_h;
    // key/value head of this query head's group (the same head when H_kv == H)
    const int64_t kv_base = b * p.kv_stride_b + (h / (p.H / p.H_kv)) * p.kv_stride_h;
    const T* Q = (const T*)p.q + base;
    const T* K = (const T*)p.k + kv_base;
    const T* V = (const T*)p.v + kv_base;
    float* O = p.o + base;
    float* L = p.lse + b * p.stat_stride_b + h * p.stat_stride_h;
    const int d = p.d;
    const int64_t ss = p.stride_s;        // elements between consecutive rows of Q and O
    const int64_t ks = p.kv_stride_s;     // ... of K and V

    for (int r = 0; r < kRowsPerWave; ++r) {
        const int a = (blockIdx.x * kWaves + wave) * kRowsPerWave + r;
        if (a >= p.c) break;                                  // wave-uniform
        const int nkeys = keys_for_query(a, p.c, p.kind, p.off);
        if (nkeys == 0) continue;                             // row sees nothing: state unchanged
        for (int t = lane; t < d; t += 64) q_lds[wave][t] = ld<T>(Q + (int64_t)a * ss + t);
        // running state: weight exp(lse) with l = 1 (or nothing yet)
        float m = L[a];
        float l = (m == -INFINITY) ? 0.f : 1.f;
        float acc[kMaxD / 64];
#pragma unroll
        for (int i = 0; i < kMaxD / 64; ++i) {
            const int t = lane + 64 * i;
            acc[i] = (t < d) ? O[(int64_t)a * ss + t] : 0.f;
        }
        __builtin_amdgcn_wave_barrier();
        for (int b0 = 0; b0 < nkeys; b0 += 64) {
            const int key = b0 + lane;
            const bool valid = key < nkeys;
            float s = valid ? p.scale * dot_row<T>(q_lds[wave], K + (int64_t)key * ks, d) : -INFINITY;
            const float m_new = fmaxf(m, wave_max(s));        // finite: lane 0 is always valid
            const float alpha = (m == -INFINITY) ? 0.f : expf(m - m_new);
            const float pr = valid ? expf(s - m_new) : 0.f;
            l = l * alpha + wave_sum(pr);
#pragma unroll
            for (int i = 0; i < kMaxD / 64; ++i) acc[i] *= alpha;
            const int nk = min(64, nkeys - b0);
            for (int kk = 0; kk < nk; ++kk) {
                const float pk = __shfl(pr, kk);
                const T* vrow = V + (int64_t)(b0 + kk) * ks;
#pragma unroll
                for (int i = 0; i < kMaxD / 64; ++i) {
                    const int t = lane + 64 * i;
                    if (t < d) acc[i] = fmaf(pk, ld<T>(vrow + t), acc[i]);
                }
            }
            m = m_new;
        }
        const float inv = 1.f / l;
#pragma unroll
        for (int i = 0; i < kMaxD / 64; ++i) {
            const int t = lane + 64 * i;
            if (t < d) O[(int64_t)a * ss + t] = acc[i] * inv;
        }
        if (lane == 0) L[a] = m + logf(l);
        __builtin_amdgcn_wave_barrier();
    }
}

// dQ: one wave per query row, lanes over keys.
template <typename T>
__global__ void __launch_bounds__(kWaves * 64)
bwd_dq_generic_kernel(StepArgs p) {
    __shared__ float q_lds[kWaves][kMaxD];
    __shared__ float g_lds[kWaves][kMaxD];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int bh = blockIdx.y, b = bh / p.H, h = bh - b * p.H;
    const int64_t base = b * p.stride_b + h * p.stride_h;
    const int64_t kv_base = b * p.kv_stride_b + (h / (p.H / p.H_kv)) * p.kv_stride_h;
    const T* Q = (const T*)p.q + base;
    const T* K = (const T*)p.k + kv_base;
    const T* V = (const T*)p.v + kv_base;
    const T* G = (const T*)p.dout + base;
    float* DQ = p.dq + base;
    const float* L = p.lse + b * p.stat_stride_b + h * p.stat_stride_h;
    const float* D = p.delta + b * p.stat_stride_b + h * p.stat_stride_h;
    const int d = p.d;
    const int64_t ss = p.stride_s;        // elements between consecutive rows of Q, dO, dQ
    const int64_t ks = p.kv_stride_s;     // ... of K and V

    for (int r = 0; r < kRowsPerWave; ++r) {
        const int a = (blockIdx.x * kWaves + wave) * kRowsPerWave + r;
        if (a >= p.c) break;
        const int nkeys = keys_for_query(a, p.c, p.kind, p.off);
        if (nkeys == 0) continue;
        for (int t = lane; t < d; t += 64) {
            q_lds[wave][t] = ld<T>(Q + (int64_t)a * ss + t);
            g_lds[wave][t] = ld<T>(G + (int64_t)a * ss + t);
        }
        const float lse = L[a], delta = D[a];
        float acc[kMaxD / 64];
#pragma unroll
        for (int i = 0; i < kMaxD / 64; ++i) acc[i] = 0.f;
        __builtin_amdgcn_wave_barrier();
        for (int b0 = 0; b0 < nkeys; b0 += 64) {
            const int key = b0 + lane;
            float ds = 0.f;
            if (key < nkeys) {
                const float s = p.scale * dot_row<T>(q_lds[wave], K + (int64_t)key * ks, d);
                const float pr = expf(s - lse);
                const float dp = dot_row<T>(g_lds[wave], V + (int64_t)key * ks, d);
                ds = pr * (dp - delta);
            }
            const int nk = min(64, nkeys - b0);
            for (int kk = 0; kk < nk; ++kk) {
                const float x = __shfl(ds, kk);
                const T* krow = K + (int64_t)(b0 + kk) * ks;
#pragma unroll
                for (int i = 0; i < kMaxD / 64; ++i) {
                    const int t = lane + 64 * i;
                    if (t < d) acc[i] = fmaf(x, ld<T>(krow + t), acc[i]);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < kMaxD / 64; ++i) {
            const int t = lane + 64 * i;
            if (t < d) DQ[(int64_t)a * ss + t] += p.scale * acc[i];
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// dK, dV: one wave per key row, lanes over the queries that may see it, the query heads of
// the group that shares the key/value head one after the other.
template <typename T>
__global__ void __launch_bounds__(kWaves * 64)
bwd_dkv_generic_kernel(StepArgs p) {
    __shared__ float k_lds[kWaves][kMaxD];
    __shared__ float v_lds[kWaves][kMaxD];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int bh = blockIdx.y, b = bh / p.H_kv, kvh = bh - b * p.H_kv;
    const int group = p.H / p.H_kv;
    const int64_t kv_base = b * p.kv_stride_b + kvh * p.kv_stride_h;
    const T* K = (const T*)p.k + kv_base;
    const T* V = (const T*)p.v + kv_base;
    float* DK = p.dk + kv_base;
    float* DV = p.dv + kv_base;
    const int d = p.d;
    const int64_t ss = p.stride_s;        // elements between consecutive rows of Q and dO
    const int64_t ks = p.kv_stride_s;     // ... of K, V, dK, dV

    for (int r = 0; r < kRowsPerWave; ++r) {
        const int key = (blockIdx.x * kWaves + wave) * kRowsPerWave + r;
        if (key >= p.c) break;
        // queries a with key <= a - off  <=>  a >= key + off
        const int a_first = (p.kind == MASK_FULL) ? 0 : key + p.off;
        if (a_first >= p.c) continue;
        for (int t = lane; t < d; t += 64) {
            k_lds[wave][t] = ld<T>(K + (int64_t)key * ks + t);
            v_lds[wave][t] = ld<T>(V + (int64_t)key * ks + t);
        }
        float acc_k[kMaxD / 64], acc_v[kMaxD / 64];
#pragma unroll
        for (int i = 0; i < kMaxD / 64; ++i) acc_k[i] = acc_v[i] = 0.f;
        __builtin_amdgcn_wave_barrier();
        for (int member = 0; member < group; ++member) {
            const int h = kvh * group + member;
            const int64_t base = b * p.stride_b + h * p.stride_h;
            const T* Q = (const T*)p.q + base;
            const T* G = (const T*)p.dout + base;
            const float* L = p.lse + b * p.stat_stride_b + h * p.stat_stride_h;
            const float* D = p.delta + b * p.stat_stride_b + h * p.stat_stride_h;
            for (int a0 = a_first; a0 < p.c; a0 += 64) {
                const int a = a0 + lane;
                float pr = 0.f, ds = 0.f;
                if (a < p.c) {
                    const float s = p.scale * dot_row<T>(k_lds[wave], Q + (int64_t)a * ss, d);
                    pr = expf(s - L[a]);
                    const float dp = dot_row<T>(v_lds[wave], G + (int64_t)a * ss, d);
                    ds = pr * (dp - D[a]);
                }
                const int na = min(64, p.c - a0);
                for (int kk = 0; kk < na; ++kk) {
                    const float x = __shfl(pr, kk), y = __shfl(ds, kk);
                    const T* grow = G + (int64_t)(a0 + kk) * ss;
                    const T* qrow = Q + (int64_t)(a0 + kk) * ss;
#pragma unroll
                    for (int i = 0; i < kMaxD / 64; ++i) {
                        const int t = lane + 64 * i;
                        if (t < d) {
                            acc_v[i] = fmaf(x, ld<T>(grow + t), acc_v[i]);
                            acc_k[i] = fmaf(y, ld<T>(qrow + t), acc_k[i]);
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int i = 0; i < kMaxD / 64; ++i) {
            const int t = lane + 64 * i;
            if (t < d) {
                DV[(int64_t)key * ks + t] += acc_v[i];
                DK[(int64_t)key * ks + t] += p.scale * acc_k[i];
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

dim3 row_grid(const StepArgs& a, int heads) {
    const int rows_per_block = kWaves * kRowsPerWave;
    return dim3((a.c + rows_per_block - 1) / rows_per_block, a.B * heads);
}

}  // namespace

hipError_t launch_fwd_generic(const StepArgs& a, int dtype, hipStream_t st) {
    if (dtype == SA_F32)
        hipLaunchKernelGGL(fwd_generic_kernel<float>, row_grid(a, a.H), dim3(kWaves * 64), 0, st, a);
    else
        hipLaunchKernelGGL(fwd_generic_kernel<__hip_bfloat16>, row_grid(a, a.H), dim3(kWaves * 64), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_bwd_generic(const StepArgs& a, int dtype, hipStream_t st) {
    const dim3 block(kWaves * 64);
    if (dtype == SA_F32) hipLaunchKernelGGL(bwd_dq_generic_kernel<float>, row_grid(a, a.H), block, 0, st, a);
    else hipLaunchKernelGGL(bwd_dq_generic_kernel<__hip_bfloat16>, row_grid(a, a.H), block, 0, st, a);
    if (hipError_t e = hipGetLastError()) return e;
    if (dtype == SA_F32) hipLaunchKernelGGL(bwd_dkv_generic_kernel<float>, row_grid(a, a.H_kv), block, 0, st, a);
    else hipLaunchKernelGGL(bwd_dkv_generic_kernel<__hip_bfloat16>, row_grid(a, a.H_kv), block, 0, st, a);
    return hipGetLastError();
}

}  // namespace sa
