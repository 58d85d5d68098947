// Where do the workgroups of a small grid land?  The matrix-core kernels order a grid that is
// resident all at once (at most two workgroups per CU) so that workgroups L and L + 256 carry
// about the same total work, on the assumption that those two share a CU.  This launches 512
// workgroups with the forward kernel's footprint (256 threads, 64 KiB of LDS: two per CU), has
// each report the CU it runs on (hardware id registers), and counts how many CUs hold exactly
// the pair (L, L + 256).
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <map>
#include <vector>

#define CHECK(x)                                                                 \
    do {                                                                         \
        hipError_t e_ = (x);                                                     \
        if (e_ != hipSuccess) {                                                  \
            std::printf("%s failed: %s\n", #x, hipGetErrorString(e_));           \
            return 1;                                                            \
        }                                                                        \
    } while (0)

__global__ void __launch_bounds__(256, 2) where_am_i(unsigned* out, int naps) {
    __shared__ char lds[65536];
    unsigned hw, xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    lds[threadIdx.x] = (char)hw;       // keeps the LDS allocation
    __syncthreads();
    // a bounded nap, so that every workgroup is still resident when the last one starts
    for (int i = 0; i < naps; ++i) __builtin_amdgcn_s_sleep(10);
    if (threadIdx.x == 0) {
        out[2 * blockIdx.x] = hw;
        out[2 * blockIdx.x + 1] = xcc + (lds[1] & 0);
    }
}

int main() {
    const int n = 512;
    unsigned* d = nullptr;
    CHECK(hipMalloc(&d, 8 * n));
    for (int rep = 0; rep < 2; ++rep) {      // the second launch is the one reported
        CHECK(hipMemset(d, 0, 8 * n));
        hipLaunchKernelGGL(where_am_i, dim3(n), dim3(256), 0, 0, d, 2000);
        CHECK(hipGetLastError());
        CHECK(hipDeviceSynchronize());
    }
    std::vector<unsigned> h(2 * n);
    CHECK(hipMemcpy(h.data(), d, 8 * n, hipMemcpyDeviceToHost));
    std::map<unsigned, std::vector<int>> cus;
    for (int i = 0; i < n; ++i) {
        const unsigned hw = h[2 * i], xcc = h[2 * i + 1] & 0xf;
        // HW_ID: cu_id bits 11:8, sh_id bit 12, se_id bits 15:13
        cus[(xcc << 12) | (((hw >> 13) & 7) << 8) | (((hw >> 12) & 1) << 4) | ((hw >> 8) & 0xf)].push_back(i);
    }
    int pairs = 0, partners = 0;
    for (auto& kv : cus)
        if (kv.second.size() == 2) {
            ++pairs;
            if (std::abs(kv.second[0] - kv.second[1]) == 256) ++partners;
        }
    std::printf("%d workgroups on %zu distinct CUs; CUs holding exactly two: %d, of which the pair is (L, L + 256): %d\n",
                n, cus.size(), pairs, partners);
    for (int i = 0; i < 16; ++i)
        std::printf("workgroup %2d: xcc %u  se %u  cu %2u\n", i, h[2 * i + 1] & 0xf, (h[2 * i] >> 13) & 7, (h[2 * i] >> 8) & 0xf);
    CHECK(hipFree(d));
    return 0;
}
