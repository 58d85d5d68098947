// Tile staging shared by the matrix-core kernels: 64-row x 128-column bf16 tiles
// go from global memory straight into swizzled LDS tiles and are read from there
// in the layouts the v_mfma_f32_32x32x16_bf16 operands want.
//
// Register layouts of that instruction (lane = 32*h + n):
//   A operand: row n of the 32 x 16 left matrix, 8 consecutive k starting at 8h
//   B operand: column n of the 16 x 32 right matrix, the same 8 k
//   C/D:       column n, rows 8*(r/4) + 4h + r%4 for register r = 0..15
// A C/D tile whose rows are the contraction index of the next product can be
// fed to it as a B operand straight from registers: registers 8g'..8g'+7 of a
// 32-row block are rows {0..3, 8..11} + 4h of a group of 16; the transposing LDS
// reads below deliver the other operand in the same order.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int TD = 128;          // tile columns: head dimensions up to 128 are zero-padded to it;
                                 // larger ones (up to 256) are held as two such tiles, columns
                                 // 0..127 and 128..255 of the same rows ("halves")
constexpr int TR = 64;           // tile rows streamed per iteration

// DP, the number of columns a kernel instantiation computes: 64, 112, 128 or 256.  Tiles are
// always 128 columns wide (two of them, "halves", for 256); a smaller DP only leaves out work:
// a contraction over the head dimension takes ksteps_of(DP) steps of 16 columns per half, a
// product whose output has head-dimension columns blocks_of(DP) blocks of 32 per half.
// 112 (head dimensions 65..112, e.g. the 100 of the paper's 3B model, Table 1) drops the last
// k-step and keeps all four output blocks.
constexpr int halves_of(int DP) { return DP > 128 ? 2 : 1; }
constexpr int ksteps_of(int DP) { return (DP / halves_of(DP) + 15) / 16; }
constexpr int blocks_of(int DP) { return (DP / halves_of(DP) + 31) / 32; }
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

// ---------------------------------------------------------------------------
// Swizzled tiles filled by direct global -> LDS loads.
//
// A tile is 64 rows x 256 bytes (128 bf16) with NO padding: a direct load
// writes the 64 lanes' 16-byte pieces contiguously (1 KiB per wavefront
// instruction, 4 rows), so a 16 KiB tile takes 16 instructions, 4 per
// wavefront.  Bank conflicts are avoided by storing the 16-byte chunk c of row
// r at chunk position c ^ f(r), f(r) = ((r & 3) << 2) | ((r >> 2) & 3):
//  * 16-byte A-operand row reads (16 consecutive rows, same logical chunk) hit
//    16 different chunks, because f is a bijection of r & 15;
//  * the transposing 8-byte reads (ds_read_b64_tr_b16: 4 consecutive rows x two
//    neighbouring 32-byte chunk pairs per half-wave) hit 8 different pairs.
// The swizzle is applied on the global side: the lane that fills chunk position
// pc of row r fetches logical chunk pc ^ f(r).
//
// Transposing read.  Within each block of 16 lanes the instruction hands lane i
// the i-th 16-bit element of what lanes 4e + i/4 (e = 0..3) point at, so lane j
// of a block points at row j/4, columns 4 (j%4) .. +3 of a 4 x 16 patch and every
// lane receives 4 consecutive rows of one column.  Two reads (rows +0 and +8)
// give the 8 contraction values {0..3, 8..11} + 4h of a group of 16 rows that
// match a C/D tile used as B operand.
constexpr int DT_ROWS = 64;
constexpr int DT_BYTES = DT_ROWS * 256;          // 16 KiB
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) char lds_char_t;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4_t;

__device__ inline int dt_swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

// Head dimensions below 128.  A lane fetches the 16-byte chunk at logical position
// pc ^ f(r) of its row.  A chunk that starts at or beyond column d is not fetched at all:
// the lane's offset is set beyond the descriptor's range, for which the load is defined to
// deliver zeros, so those LDS columns hold zeros whatever follows the row in memory.  When d
// is not a multiple of 8 the last chunk of a row holds 4 valid columns and 4 columns of
// whatever follows the row (the next row, a gap of the caller's layout); the kernels'
// PART instantiations clear those four after reading the chunk from LDS (zero_beyond_d).
constexpr uint32_t DT_OUT_OF_RANGE = 0x80000000u;     // >= any descriptor range (all are < 2^31)

// byte offsets (within a tile, global side) of the 4 pieces this lane fetches
// (pitch = bytes between rows in global memory, >= 2 d)
// (half: which 128-column half of the rows this tile holds, 0 unless d > 128)
__device__ inline void dt_load_offsets(uint32_t (&g)[4], int lane, int wave, int pitch, int d, int half = 0) {
    const int lr = lane >> 4, pc = lane & 15;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = 16 * wave + 4 * j + lr;
        const int chunk = pc ^ dt_swz(r);
        g[j] = 128 * half + 8 * chunk < d ? r * pitch + 256 * half + (chunk << 4) : DT_OUT_OF_RANGE;
    }
}
// PART (d % 8 == 4): fragment of k-step ks read by half h is the chunk 2 ks + h; in the chunk
// that holds column d the elements 4..7 are beyond the row
__device__ inline bf16x8 zero_beyond_d(bf16x8 x, bool is_last_chunk) {
    typedef int i32x4 __attribute__((ext_vector_type(4)));
    i32x4 v = __builtin_bit_cast(i32x4, x);
    v[2] = is_last_chunk ? 0 : v[2];
    v[3] = is_last_chunk ? 0 : v[3];
    return __builtin_bit_cast(bf16x8, v);
}
// The loads go through a buffer descriptor held in scalar registers: the tile's byte
// offset within the (batch, head) matrix is a scalar operand and the lane offset a 32-bit
// vector operand, so a load costs no address arithmetic at all.  The descriptor's range is
// the c rows of the matrix (stride 0, raw 32-bit data format).
//
// The instruction is issued from inline assembly on purpose.  The compiler orders LDS reads
// after a direct load it knows about with a conservative model of what the load writes, and
// puts a wait for ALL loads in flight in front of reads of a different buffer, i.e. right
// after the loads were issued.  Issued this way the loads are invisible to that model; the
// kernels order them by hand: s_waitcnt vmcnt(0) followed by a workgroup barrier before a
// buffer is read, a barrier after its last read before it is requested again.  The
// "memory" clobber keeps the compiler from moving LDS accesses across the request.
typedef int dt_rsrc __attribute__((ext_vector_type(4)));
__device__ inline dt_rsrc dt_make_rsrc(const void* matrix, int rows, int pitch, int d) {
    const uint64_t a = reinterpret_cast<uint64_t>(matrix);
    dt_rsrc r;
    r[0] = (int)(uint32_t)a;
    r[1] = (int)((uint32_t)(a >> 32) & 0xffffu);
    r[2] = (rows - 1) * pitch + 2 * d;     // ends with the last row; the range check is per dword
                                           // and reads past the end return 0
    r[3] = 0x00020000;
    return r;
}
// one 1 KiB piece: 64 lanes x 16 bytes from matrix + tile_byte_offset + lane_offset to
// lds_dst + 16 * lane (lds_dst wave-uniform)
// (m0 is named as clobbered although the compiler calls it reserved: nothing else in these
// kernels uses it, and the note it prints about that is switched off for this function)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ inline void dt_load_piece(dt_rsrc matrix, int tile_byte_offset, uint32_t lane_offset, const char* lds_dst) {
    const uint32_t dst = (uint32_t)reinterpret_cast<uintptr_t>((const lds_char_t*)lds_dst);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(dst), "v"(lane_offset), "s"(matrix), "s"(tile_byte_offset)
                 : "memory", "m0");
}
#pragma clang diagnostic pop
// wave must be wave-uniform (scalar): it selects the LDS destination of each load
__device__ inline void dt_load(dt_rsrc matrix, int tile_byte_offset, char* lds_tile, const uint32_t (&g)[4], int wave) {
#pragma unroll
    for (int j = 0; j < 4; ++j) dt_load_piece(matrix, tile_byte_offset, g[j], lds_tile + (4 * wave + j) * 1024);
}
// A-operand row reads: address of row n (within a 32-row half tile), k-step ks, half h
__device__ inline void dt_row_addrs(uint32_t (&a)[8], int n, int h) {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) a[ks] = n * 256 + (((2 * ks + h) ^ dt_swz(n)) << 4);
}
__device__ inline bf16x8 dt_read_row(const char* lds_half, uint32_t addr) {
    return *reinterpret_cast<const bf16x8*>(lds_half + addr);
}
// Transposing reads: addresses (within a group of 16 rows) for 32-column block mb,
// first read (rows +0) and second read (rows +8)
__device__ inline void dt_tr_addrs(uint32_t (&t0)[4], uint32_t (&t1)[4], int lane) {
    const int i = lane & 15, h = lane >> 5, nh = (lane >> 4) & 1, j4 = i >> 2;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) {
        const int c = 4 * mb + 2 * nh + ((i & 3) >> 1);      // logical 16-byte chunk
        const int r0 = 4 * h + j4, r1 = r0 + 8;
        t0[mb] = r0 * 256 + ((c ^ dt_swz(r0)) << 4) + (i & 1) * 8;
        t1[mb] = r1 * 256 + ((c ^ dt_swz(r1)) << 4) + (i & 1) * 8;
    }
}
__device__ inline bf16x8 dt_read_tr(const char* lds_group, uint32_t a0, uint32_t a1) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(lds_group + a0));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(lds_group + a1));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}
// max / sum over the two half-waves (lanes n and n + 32)
__device__ inline float half_wave_max(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float half_wave_sum(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ inline f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Workgroup order of a 1-D grid over (tile rank, batch*head), rank 0 = heaviest tile.
// Large grids: heads are taken in groups of 8; inside a group the index runs over
// heads fastest and tile ranks slowest, so (i) every group runs heaviest-first and
// the last workgroups to start are the lightest, and (ii) as consecutive workgroups
// go round-robin to the 8 XCDs, all tiles of one head land on one XCD and share its
// L2 while they stream the same K/V (or Q/dO) rows.
// Small grids (every workgroup resident at once, at most 2 per CU): plain
// heaviest-first over all heads; with SNAKE the second 256 workgroups run
// lightest-first, so that the two workgroups sharing a CU (indices L and L + 256)
// carry about the same total work.
constexpr int HEAD_GROUP = 8;
constexpr int N_CU = 256;
template <bool SNAKE>
__device__ inline void decode_block(int linear, int n_tiles, int n_bh, int& rank, int& bh) {
    const int total = n_tiles * n_bh;
    if (total <= 2 * N_CU) {
        int s = linear;
        if (SNAKE && linear >= N_CU) s = total - 1 - (linear - N_CU);
        rank = s / n_bh;
        bh = s - rank * n_bh;
        return;
    }
    const int per_group = HEAD_GROUP * n_tiles;
    const int grp = linear / per_group;
    const int within = linear - grp * per_group;
    const int heads = min(HEAD_GROUP, n_bh - grp * HEAD_GROUP);
    rank = within / heads;
    bh = grp * HEAD_GROUP + (within - rank * heads);
}

// Row of d <= 16 NF elements (d a multiple of 4) as B-operand fragments, NF k-steps of 16,
// zero-padded to 16 NF columns.  Nothing beyond the row is read.
template <int NF>
__device__ inline void load_b_frags(bf16x8 (&f)[NF], const __bf16* __restrict__ row, int h, int d) {
    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int ks = 0; ks < NF; ++ks) {
        const int col = 16 * ks + 8 * h;
        if (col + 8 <= d) {
            f[ks] = *reinterpret_cast<const bf16x8*>(row + col);
        } else {
            bf16x4 lo = {0, 0, 0, 0};
            if (col + 4 <= d) lo = *reinterpret_cast<const bf16x4*>(row + col);
            const bf16x4 z = {0, 0, 0, 0};
            f[ks] = __builtin_shufflevector(lo, z, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    }
}

}  // namespace sa
