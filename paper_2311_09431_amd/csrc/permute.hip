// Stripe / unstripe permutation (Sec. 2.3): token t of the original sequence
// lives at row (t mod N) * c + t div N of the permuted one.  Pure byte movement,
// HBM-bandwidth bound: every row is read once and written once.
#include "sa_internal.h"

namespace sa {

// One thread moves one VEC-byte chunk at a time; a row of `chunks` chunks is read and written
// contiguously (256-byte rows = 16 lanes x 16 B), only the row start jumps.  A block is laid
// out as (rows, lanes per row) with a power-of-two number of lanes per row, blockIdx.y walks the
// outer index, so the only division a thread does is one in 32 bits (n_seq < 2^31; longer
// sequences take 64-bit arithmetic).
//
// The threads walk the rows of one side front to back ("here") and jump on the other:
//   other(t) = (t mod div) * mul + t div div
//   stripe,   walking the source:       scatter dst[other(t)] = src[t],  div = N, mul = c
//   stripe,   walking the destination:  gather  dst[t] = src[other(t)],  div = c, mul = N
//   unstripe, walking the destination:  gather  dst[t] = src[other(t)],  div = N, mul = c
// Walking the side in the ORIGINAL token order means rows t and t + N are neighbours on the
// other side, so N-row groups of consecutive rows touch N runs of consecutive rows there.  For
// rows that are a whole number of 128-byte lines that is the fastest form in both directions
// (2 GiB tensors of 256-byte rows: stripe 5.05-5.2 TB/s scattering, 4.86 gathering; a plain
// device-to-device copy of the same size runs at 4.93 TB/s).  Rows that end inside a line
// (200 bytes: head dimension 100) are only written contiguously: scattered, their partial
// lines reach memory before the neighbouring row has filled them (3.05 TB/s against 4.8).
template <typename VecT, typename IdxT>
__global__ void __launch_bounds__(256)
permute_kernel(const VecT* __restrict__ src, VecT* __restrict__ dst, int64_t outer, int64_t n_seq,
               int64_t chunks, int64_t div, int64_t mul, bool gather, int lpr_log2) {
    const int lpr = 1 << lpr_log2;                       // lanes per row
    const int x0 = threadIdx.x & (lpr - 1), r = threadIdx.x >> lpr_log2;
    const int64_t rows_per_block = 256 >> lpr_log2;
    for (int64_t o = blockIdx.y; o < outer; o += gridDim.y) {
        const VecT* s = src + o * n_seq * chunks;
        VecT* d = dst + o * n_seq * chunks;
        for (int64_t t = blockIdx.x * rows_per_block + r; t < n_seq; t += gridDim.x * rows_per_block) {
            const IdxT q = (IdxT)t / (IdxT)div, rem = (IdxT)t - q * (IdxT)div;
            const int64_t here = t * chunks, other = ((int64_t)rem * mul + (int64_t)q) * chunks;
            for (int64_t x = x0; x < chunks; x += lpr) {
                if (gather) d[here + x] = s[other + x];
                else d[other + x] = s[here + x];
            }
        }
    }
}

template <typename VecT>
static hipError_t run(const void* src, void* dst, int64_t outer, int64_t n_seq, int64_t inner_bytes,
                      int N, bool inverse, hipStream_t st) {
    const int64_t chunks = inner_bytes / (int64_t)sizeof(VecT);
    int lpr_log2 = 0;
    while (lpr_log2 < 8 && (int64_t(1) << lpr_log2) < chunks) ++lpr_log2;
    const int64_t rows_per_block = 256 >> lpr_log2;
    // about 64 blocks per CU over both grid dimensions, grid-stride beyond
    const int64_t gy = outer < 65535 ? outer : 65535;
    int64_t gx = (n_seq + rows_per_block - 1) / rows_per_block;
    const int64_t cap = (256 * 64 + gy - 1) / gy;
    if (gx > cap) gx = cap;
    const dim3 grid((unsigned)gx, (unsigned)gy), block(256);
    const int64_t c = n_seq / N;
    const bool gather = inverse || inner_bytes % 128 != 0;
    const bool walk_original = inverse || !gather;      // else: stripe walking its destination
    const int64_t div = walk_original ? N : c, mul = walk_original ? c : N;
    if (n_seq < (int64_t(1) << 31))
        hipLaunchKernelGGL((permute_kernel<VecT, uint32_t>), grid, block, 0, st, (const VecT*)src, (VecT*)dst,
                           outer, n_seq, chunks, div, mul, gather, lpr_log2);
    else
        hipLaunchKernelGGL((permute_kernel<VecT, int64_t>), grid, block, 0, st, (const VecT*)src, (VecT*)dst,
                           outer, n_seq, chunks, div, mul, gather, lpr_log2);
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
