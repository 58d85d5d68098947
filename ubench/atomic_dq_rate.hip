// What would fp32 atomic accumulation of dQ cost?  A backward step that computes S and dP once
// (5 contractions instead of 7) has key-owning workgroups add their partial dQ tiles into global
// memory.  This microbenchmark issues exactly that traffic and nothing else: 256 workgroups (one
// per compute unit) of 4 wavefronts; workgroup b plays key block b / 8 of head b % 8 and walks
// 32-query sub-tiles from its diagonal on, each wavefront adding a 32-query x 32-column fp32
// tile per sub-tile (16 wave-wide global_atomic_add_f32, 2 rows x 128 bytes each), i.e. 16 KiB
// of atomic payload per workgroup and sub-tile, the figure of a 128-key workgroup.
//
//   pattern "xcd":   consecutive workgroup indices go round-robin to the 8 XCDs, so the 32
//                    workgroups of a head share one XCD's L2 (the backward kernels' grid order)
//   pattern "cross": the 256 workgroups all play one head, so every dQ row is hit from all XCDs
//   mode "atomic" / "plain" (racy load-add-store, for the rate of the same bytes without atomics)
//
// Build: python ubench/build.py     Run: _build/atomic_dq_rate
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>

#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e_)); exit(1); } } while (0)

constexpr int D = 128;

template <bool ATOMIC>
__global__ void __launch_bounds__(256) add_tiles(float* dq, int rows, int subtiles, int cross, float val) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n = lane & 31, h = lane >> 5;
    const int head = cross ? 0 : blockIdx.x % 8;
    const int kb = cross ? blockIdx.x : blockIdx.x / 8;       // key block of 128 rows
    float* base = dq + (size_t)head * rows * D;
    int q0 = kb * 128;                                        // first query sub-tile: the diagonal
    for (int u = 0; u < subtiles; ++u) {
        const int row0 = (q0 + 32 * u) % rows;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float* p = base + (size_t)(row0 + 8 * (r / 4) + 4 * h + (r % 4)) * D + 32 * wave + n;
            if (ATOMIC) unsafeAtomicAdd(p, val);
            else *p += val;
        }
    }
}

int main() {
    const int rows = 32768, heads = 8, subtiles = 512;
    float* dq;
    CHECK(hipMalloc(&dq, (size_t)heads * rows * D * 4));
    CHECK(hipMemset(dq, 0, (size_t)heads * rows * D * 4));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const double bytes = 256.0 * subtiles * 4 * 16 * 64 * 4;      // payload per launch
    for (int cross = 0; cross < 2; ++cross)
        for (int atomic = 1; atomic >= 0; --atomic) {
            float best = 1e30f;
            for (int rep = 0; rep < 4; ++rep) {
                CHECK(hipEventRecord(e0));
                if (atomic) hipLaunchKernelGGL(add_tiles<true>, dim3(256), dim3(256), 0, 0, dq, rows, subtiles, cross, 1.0f);
                else hipLaunchKernelGGL(add_tiles<false>, dim3(256), dim3(256), 0, 0, dq, rows, subtiles, cross, 1.0f);
                CHECK(hipGetLastError());
                CHECK(hipEventRecord(e1));
                CHECK(hipEventSynchronize(e1));
                float ms;
                CHECK(hipEventElapsedTime(&ms, e0, e1));
                if (rep && ms < best) best = ms;
            }
            printf("pattern %-5s mode %-6s  %.3f ms  %.2f TB/s of fp32 payload (%.1f GB per launch)\n",
                   cross ? "cross" : "xcd", atomic ? "atomic" : "plain", best, bytes / best * 1e-9, bytes * 1e-9);
        }
    // the atomic sums are exact small integers: check one element per pattern
    float hv;
    CHECK(hipMemcpy(&hv, dq, 4, hipMemcpyDeviceToHost));
    printf("dq[0] = %.1f\n", hv);
    return 0;
}
