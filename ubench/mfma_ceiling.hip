// Hardware ceilings for the matrix-core kernels, measured rather than assumed:
//  (1) a register-only stream of v_mfma_f32_32x32x16_bf16 on constant and on random bf16
//      operands (the chip is power-limited: the operand data changes the sustained clock);
//  (2) the same stream with the VALU, transcendental, LDS-read and global -> LDS tile-load
//      instructions of an attention inner loop riding along, on registers the MFMAs do not
//      touch: what the instruction mix allows before any dependency, barrier or memory wait.
// Build: python ubench/build.py     Run: _build/mfma_ceiling
#include <hip/hip_runtime.h>
#include <cstdio>
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ inline unsigned hash(unsigned x) { x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16; return x; }
// NV fma, NE exp per MFMA; NL2 = ds_read_b128 per TWO MFMAs; ND = 1 KiB global -> LDS loads per
// FOUR MFMAs (from an L2-resident buffer); OCC wavefronts per SIMD; CONST: constant operands
// instead of random ones
template <int NV, int NE, int NL2, int OCC, bool CONST = false, int ND = 0>
__global__ void __launch_bounds__(256, OCC) k(float* out, int iters, const char* gsrc = nullptr) {
    __shared__ __attribute__((aligned(16))) float lds[4096];
    for (int i = threadIdx.x; i < 4096; i += 256) lds[i] = 1.0f;
    __syncthreads();
    bf16x8 a, b;
    {
        u32x4 ra, rb;
        for (int e = 0; e < 4; ++e) {
            unsigned h1 = hash(threadIdx.x * 64 + e + blockIdx.x * 7919), h2 = hash(h1 + 12345);
            auto mk = [](unsigned h) { return ((h & 0x8000u) | 0x3f00u | (h & 0xffu)) & 0xffffu; };
            ra[e] = CONST ? 0x3c003c00u : (mk(h1) | (mk(h1 >> 16) << 16));
            rb[e] = CONST ? 0x3c003c00u : (mk(h2) | (mk(h2 >> 16) << 16));
        }
        a = __builtin_bit_cast(bf16x8, ra);
        b = __builtin_bit_cast(bf16x8, rb);
    }
    f32x16 c[4] = {{0}, {0}, {0}, {0}};
    float x[8], e[4];
    for (int j = 0; j < 8; ++j) x[j] = 0.001f * (threadIdx.x + j);
    for (int j = 0; j < 4; ++j) e[j] = -0.5f - 0.001f * threadIdx.x;
    const float k1 = 0.999f, k2 = 0.0001f;
    f32x4 l[4];
    const unsigned addr = (threadIdx.x & 63) * 16;
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    i32x4 rsrc; { unsigned long long a = (unsigned long long)gsrc; rsrc[0] = (int)(unsigned)a; rsrc[1] = (int)((unsigned)(a >> 32) & 0xffffu); rsrc[2] = 1 << 20; rsrc[3] = 0x00020000; }
    const unsigned wave_lds = __builtin_amdgcn_readfirstlane(8192 + (threadIdx.x >> 6) * 1024);
    const unsigned goff = (threadIdx.x & 63) * 16 + (blockIdx.x & 15) * 65536;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c[u % 4]) : "v"(a), "v"(b));
#pragma unroll
            for (int j = 0; j < NV; ++j) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[(u * NV + j) % 8]) : "v"(k1), "v"(k2));
#pragma unroll
            for (int j = 0; j < NE; ++j) asm volatile("v_exp_f32 %0, %0" : "+v"(e[(u * NE + j) % 4]));
            if (ND > 0 && (u % 4) < ND) {
                int so = (it & 15) * 4096 + (u / 4) * 1024;
                asm volatile("" : "+s"(so));
                asm volatile("s_add_u32 m0, %0, 0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" :: "s"(wave_lds), "v"(goff), "s"(rsrc), "s"(so) : "memory", "m0", "scc");
            }
            if (u == 15 && ND > 0) asm volatile("s_waitcnt vmcnt(4)");
            if (NL2 > 0) {
                const int nl = (u & 1) ? NL2 / 2 : NL2 - NL2 / 2;
#pragma unroll
                for (int j = 0; j < nl; ++j) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(l[j % 4]) : "v"(addr), "n"(1024 * (j % 4)));
                if (nl) asm volatile("s_waitcnt lgkmcnt(4)");
            }
        }
        if ((it & 63) == 63)
            for (int j = 0; j < 4; ++j) for (int r = 0; r < 16; ++r) c[j][r] *= 1e-3f;
    }
    asm volatile("s_waitcnt lgkmcnt(0)");
    float s = 0;
    for (int j = 0; j < 4; ++j) for (int r = 0; r < 16; ++r) s += c[j][r];
    for (int j = 0; j < 8; ++j) s += x[j];
    for (int j = 0; j < 4; ++j) s += e[j] + l[j][0];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}
template <typename F> float timeit(F f) {
    hipEvent_t e0, e1; (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
    f(); (void)hipDeviceSynchronize();
    (void)hipEventRecord(e0); f(); (void)hipEventRecord(e1); (void)hipEventSynchronize(e1);
    float ms; (void)hipEventElapsedTime(&ms, e0, e1); return ms;
}
template <int NV, int NE, int NL2, int OCC, bool CONST = false, int ND = 0> void run(float* out, const char* g = nullptr) {
    const int iters = 6000, blocks = 256 * OCC;
    const double fl = 16.0 * iters * 32768.0 * 4 * blocks;
    float ms = timeit([&] { hipLaunchKernelGGL((k<NV, NE, NL2, OCC, CONST, ND>), dim3(blocks), dim3(256), 0, 0, out, iters, g); });
    printf("%d waves/SIMD  %s operands  per MFMA: %d fma %d exp %.1f ds_read_b128 %d/4 tile loads : %7.2f ms %5.0f TFLOP/s\n", OCC, CONST ? "constant" : "random  ", NV, NE, NL2 / 2.0, ND, ms, fl / ms * 1e-9);
    fflush(stdout);
}
int main() {
    float* out; (void)hipMalloc(&out, 4 * 1024 * 256);
    char* g; (void)hipMalloc(&g, 2 << 20); (void)hipMemset(g, 1, 2 << 20);
    run<0, 0, 0, 2>(out);                      // warm-up, printed but not to be quoted
    run<0, 0, 0, 2, true>(out); run<0, 0, 0, 2>(out); run<0, 0, 0, 1, true>(out); run<0, 0, 0, 1>(out);
    run<2, 0, 0, 2>(out); run<4, 0, 0, 2>(out); run<6, 0, 0, 2>(out);
    run<4, 1, 0, 2>(out); run<4, 1, 2, 2>(out); run<4, 1, 3, 2>(out); run<4, 1, 4, 2>(out);
    run<4, 1, 3, 2, false, 1>(out, g); run<5, 1, 3, 2, false, 1>(out, g);      // forward-like, with its tile loads
    run<3, 1, 3, 2>(out); run<3, 1, 3, 2, false, 1>(out, g);                    // dQ-like
    run<3, 1, 0, 1>(out); run<3, 1, 3, 1>(out); run<3, 1, 4, 1>(out); run<3, 1, 4, 1, false, 1>(out, g);   // dK/dV-like
    run<4, 1, 1, 1>(out); run<4, 1, 2, 1>(out);          // 64 queries per wavefront, one wavefront per SIMD
    run<2, 1, 3, 2, false, 1>(out, g);                    // brackets the dQ kernel's count from above (2.4 + 0.67 exp)
    run<2, 1, 4, 1, false, 1>(out, g);                    // brackets the dK/dV kernel's count from above (1.45 + 0.6 exp)
    return 0;
}
