// Tile staging shared by the matrix-core kernels: 64-row x 128-column bf16 tiles
// go from global memory through registers into LDS, either row-major or
// transposed, in the layouts the v_mfma_f32_32x32x16_bf16 operands want.
//
// Register layouts of that instruction (lane = 32*h + n):
//   A operand: row n of the 32 x 16 left matrix, 8 consecutive k starting at 8h
//   B operand: column n of the 16 x 32 right matrix, the same 8 k
//   C/D:       column n, rows 8*(r/4) + 4h + r%4 for register r = 0..15
// A C/D tile whose rows are the contraction index of the next product can be
// fed to it as a B operand straight from registers: registers 8g'..8g'+7 of a
// 32-row block are rows {0..3, 8..11} + 4h of a group of 16.  The transposed LDS
// tiles therefore store every group of 16 columns in the order
// 0-3, 8-11, 4-7, 12-15, so that one 16-byte read gives a lane its 8 values.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int TD = 128;          // tile columns = head dimension
constexpr int TR = 64;           // tile rows streamed per iteration
constexpr int RS = TD + 8;       // LDS row stride of a row-major tile, elements (272 B)
constexpr int TS = TR + 8;       // LDS row stride of a transposed tile, elements (144 B)
constexpr int ROW_TILE = TR * RS;    // elements
constexpr int TRN_TILE = TD * TS;    // elements
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

// Row-major staging.  Thread t of 256 takes the 16-byte chunk t%16 of rows t/16 + 16 i.
__device__ inline void load_rows(u32x4 (&r)[4], const __bf16* __restrict__ g, int tid) {
    const __bf16* p = g + (int64_t)(tid >> 4) * TD + (tid & 15) * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = *reinterpret_cast<const u32x4*>(p + (int64_t)i * 16 * TD);
}
__device__ inline void store_rows(const u32x4 (&r)[4], __bf16* __restrict__ lds_tile, int tid) {
    __bf16* p = lds_tile + (tid >> 4) * RS + (tid & 15) * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(p + i * 16 * RS) = r[i];
}

// Transposed staging.  Thread t takes the column pair t%64 of the row quads
// (t/64) + 4 i, one 4-byte load per row, so a wavefront reads whole 256-byte
// rows; two byte-permutes per quad build the 8-byte column pieces.
__device__ inline void load_quads(uint32_t (&r)[16], const __bf16* __restrict__ g, int tid) {
    const __bf16* p = g + (int64_t)(4 * (tid >> 6)) * TD + (tid & 63) * 2;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            r[4 * i + j] = *reinterpret_cast<const uint32_t*>(p + (int64_t)(16 * i + j) * TD);
}
__device__ inline void store_transposed(const uint32_t (&r)[16], __bf16* __restrict__ lds_tile, int tid) {
    __bf16* p = lds_tile + (tid & 63) * 2 * TS;
    const int q = tid >> 6;                              // quad within its group of 16 rows
    const int pos = 4 * (((q & 1) << 1) | (q >> 1));     // quads stored in the order 0, 2, 1, 3
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        u32x2 lo, hi;
        lo.x = __builtin_amdgcn_perm(r[4 * i + 1], r[4 * i + 0], 0x05040100u);
        lo.y = __builtin_amdgcn_perm(r[4 * i + 3], r[4 * i + 2], 0x05040100u);
        hi.x = __builtin_amdgcn_perm(r[4 * i + 1], r[4 * i + 0], 0x07060302u);
        hi.y = __builtin_amdgcn_perm(r[4 * i + 3], r[4 * i + 2], 0x07060302u);
        *reinterpret_cast<u32x2*>(p + 16 * i + pos) = lo;
        *reinterpret_cast<u32x2*>(p + TS + 16 * i + pos) = hi;
    }
}

// A-operand reads.  Row-major tile: row `row`, k-step ks (16 columns), half h.
__device__ inline bf16x8 read_a_rows(const __bf16* lds_tile, int row, int ks, int h) {
    return *reinterpret_cast<const bf16x8*>(lds_tile + row * RS + 16 * ks + 8 * h);
}
// Transposed tile: row `col` (a column of the original), group g of 16 original rows.
__device__ inline bf16x8 read_a_trn(const __bf16* lds_tile, int col, int g, int h) {
    return *reinterpret_cast<const bf16x8*>(lds_tile + col * TS + 16 * g + 8 * h);
}

__device__ inline f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// 128-column row of `g` as B-operand fragments: 8 k-steps of 16
__device__ inline void load_b_frags(bf16x8 (&f)[8], const __bf16* __restrict__ row, int h) {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) f[ks] = *reinterpret_cast<const bf16x8*>(row + 16 * ks + 8 * h);
}

}  // namespace sa
