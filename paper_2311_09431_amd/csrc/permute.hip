// Stripe / unstripe permutation (Sec. 2.3): token t of the original sequence
// lives at row (t mod N) * c + t div N of the permuted one.  Pure byte movement,
// HBM-bandwidth bound: every row is read once and written once.
#include "sa_internal.h"

namespace sa {

// One thread moves one VEC-byte chunk.  Threads are laid out over the
// DESTINATION so stores are fully coalesced; a row of `chunks` chunks is read
// contiguously as well (256-byte rows = 16 lanes x 16 B), only the row start
// jumps.  forward: dst row p = dev*c + a takes src row a*N + dev.
// inverse: dst row t = a*N + dev takes src row dev*c + a.
template <typename VecT>
__global__ void __launch_bounds__(256)
permute_kernel(const VecT* __restrict__ src, VecT* __restrict__ dst, int64_t n_seq, int64_t chunks,
               int N, int64_t c, bool inverse, int64_t total) {
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t step = (int64_t)gridDim.x * blockDim.x;
    for (; idx < total; idx += step) {
        const int64_t x = idx % chunks;
        const int64_t row = idx / chunks;      // o * n_seq + dst row
        const int64_t o = row / n_seq;
        const int64_t r = row - o * n_seq;
        int64_t s;
        if (!inverse) {
            const int64_t dev = r / c, a = r - dev * c;
            s = a * N + dev;
        } else {
            const int64_t a = r / N, dev = r - a * N;
            s = dev * c + a;
        }
        dst[idx] = src[(o * n_seq + s) * chunks + x];
    }
}

template <typename VecT>
static hipError_t run(const void* src, void* dst, int64_t outer, int64_t n_seq, int64_t inner_bytes,
                      int N, bool inverse, hipStream_t st) {
    const int64_t chunks = inner_bytes / (int64_t)sizeof(VecT);
    const int64_t total = outer * n_seq * chunks;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;   // grid-stride beyond 64 blocks per CU
    hipLaunchKernelGGL(permute_kernel<VecT>, dim3((unsigned)blocks), dim3(256), 0, st,
                       (const VecT*)src, (VecT*)dst, n_seq, chunks, N, n_seq / N, inverse, total);
    return hipGetLastError();
}

hipError_t launch_permute(const void* src, void* dst, int64_t outer, int64_t n_seq,
                          int64_t inner_bytes, int N, bool inverse, hipStream_t st) {
    if (outer * n_seq * inner_bytes == 0) return hipSuccess;
    if (inner_bytes % 16 == 0) return run<uint4>(src, dst, outer, n_seq, inner_bytes, N, inverse, st);
    if (inner_bytes % 8 == 0) return run<uint2>(src, dst, outer, n_seq, inner_bytes, N, inverse, st);
    if (inner_bytes % 4 == 0) return run<uint32_t>(src, dst, outer, n_seq, inner_bytes, N, inverse, st);
    if (inner_bytes % 2 == 0) return run<uint16_t>(src, dst, outer, n_seq, inner_bytes, N, inverse, st);
    return run<uint8_t>(src, dst, outer, n_seq, inner_bytes, N, inverse, st);
}

}  // namespace sa
