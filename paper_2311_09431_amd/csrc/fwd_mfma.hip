// Forward ring step on the CDNA4 matrix cores (bf16 operands, fp32 accumulate),
// head dimension up to 256 (64, 112, 128 or 256 columns computed): AccumulateAttentionFragment
// of Algorithm 1 with the fused log-sum-exp merge, skipping every 32-key sub-tile
// that GetMask(j, k) masks entirely for a 32-query wavefront (Sec. 2.2.1); a coarser
// skipping granularity (Sec. 3.1) can be emulated on request.
//
// Work decomposition.  A workgroup of 4 wavefronts owns 128 query rows; each
// wavefront owns 32 of them for the whole kernel.  Key/value tiles of 64 rows
// stream from global memory straight into LDS (buffer_load ... lds, no register
// staging), two buffers each for K and V, one barrier per tile.
//
// The scores are computed TRANSPOSED, S^T = K Q^T (A = key rows from LDS, B = the
// query rows, resident in registers), so that a lane holds 16 keys of ONE query
// per 32-key sub-tile: row max / row sum of the online softmax are in-lane
// reductions plus one exchange between the two half-waves, and the
// probabilities already sit in the B-operand layout of the second product
// O^T += V^T P^T, whose A operand is read from the row-major V tile with the
// transposing LDS read.
//
// Software pipeline.  MFMA and VALU instructions only overlap when they are
// interleaved in one wavefront's instruction stream, so the loop runs over
// 32-key sub-tiles u with three stages in flight:
//     S(u+1) = K(u+1) Q^T   (8 MFMA)   |
//     P(u)   = softmax part of S(u)    |  issued interleaved, slice by slice
//     O^T   += V(u-1)^T P(u-1) (8 MFMA)|
// i.e. one exp2 and about three other VALU instructions per MFMA.
//
// Online softmax in base 2 with a lazily updated reference m: kappa = scale *
// log2(e) is folded into the exponent, p = exp2(s * kappa - m).  The common path
// never looks for a row maximum: sums of floating-point numbers do not care about
// a common factor, so m only has to move when a row's partial sum of probabilities
// exceeds RESCALE_SUM (or the row has no reference yet); then the sub-tile is redone
// against its row maximum and l and the 64 accumulator registers are rescaled,
// which almost never runs.  A step accumulates its own partial result from an
// empty state (the first sub-tile sets the reference) and folds it into the
// running (O, LSE) in its epilogue by log-sum-exp, which is where the running state
// is read: read in the prologue it would stand in front of every workgroup's first
// tile, and holding it there cost the kernel 30 spilled registers.  Row sums are
// taken over the fp32 probabilities before they are rounded to bf16 (summing the
// rounded values costs 1e-3 of LSE accuracy on rows with few keys).
//
// LDS layout.  Both tiles are 64 rows x 256 bytes without padding (the direct
// loads write 1 KiB per wavefront contiguously); bank conflicts are avoided by
// XOR-swizzling the 16-byte chunk index with the row: K chunk c of row r sits at
// chunk c ^ (r & 15) (16-byte A-operand reads of 16 consecutive rows hit 16
// different chunks), V chunk c of row r at c ^ ((r & 3) << 2) (the 4-row x 32-byte
// patches of the transposing read hit different 32-byte bank groups).  The
// swizzle is applied by choosing which global chunk each lane loads.
#include <hip/hip_bf16.h>

#include <type_traits>

#include "mfma_tiles.h"
#include "sa_internal.h"

namespace sa {

namespace {

constexpr int NW = 4;                   // wavefronts per workgroup (8 measured the same at 32768-token shards)
constexpr int BM = 32 * NW;             // query rows per workgroup
constexpr int D = TD;                   // columns of a tile: head dimensions below it are zero-padded
constexpr int TILE_ROWS = 64;           // key rows per LDS tile
constexpr int TILE_BYTES = TILE_ROWS * D * 2;   // 16 KiB
constexpr float RESCALE_SUM = 16777216.f;      // 2^24: a row's partial sum of probabilities beyond which its
                                                // reference is moved up to the row maximum

typedef __attribute__((address_space(3))) char lds_char;
typedef lds_s16x4_t lds_s16x4;

// One tile (64 rows) of K or V: 16 KiB = 16 wavefront loads of 1 KiB (4 rows), 4 per wavefront.
constexpr int LPW = 16 / NW;             // direct loads per wavefront and tile
// K: piece j of wavefront w covers tile rows 16 j + 4 w .. + 3.  K's swizzle depends on the
// row modulo 16, which is then the same for a lane's four pieces: one lane offset g0, the
// rest (16 j rows) goes into the scalar offset.
__device__ inline void load_tile_direct(dt_rsrc matrix, int tile_byte_offset, char* lds_tile, uint32_t g0, int wave,
                                        int pitch) {
#pragma unroll
    for (int j = 0; j < LPW; ++j)
        dt_load_piece(matrix, tile_byte_offset + j * 16 * pitch, g0, lds_tile + (4 * j + wave) * 1024);
}

__device__ inline void load_v_tile_direct(dt_rsrc matrix, int tile_byte_offset, char* lds_tile, uint32_t g0, int wave,
                                          int pitch) {
#pragma unroll
    for (int j = 0; j < LPW; ++j)     // piece j: four rows further down
        dt_load_piece(matrix, tile_byte_offset + j * 4 * pitch, g0, lds_tile + (LPW * wave + j) * 1024);
}

// LDS address of this lane's K operand for k-step ks: chunk (2 ks + h) ^ (n & 15) of row n.
__device__ inline uint32_t k_step_addr(const uint32_t (&kaddr)[8], int ks) { return kaddr[ks]; }
__device__ inline bf16x8 lds_read_b128(const char* lds, uint32_t addr) {
    return *reinterpret_cast<const bf16x8*>(lds + addr);
}
__device__ inline bf16x8 lds_read_tr(const char* lds, uint32_t addr) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(lds + addr));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(lds + addr + 8 * 256));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// One pipeline step on sub-tile u (32 keys):
//   QK: s_next = K(u+1) Q^T            k_next = LDS address of the 32 K rows of sub-tile u+1
//   SM: p_cur = exp2(s_cur * kappa - m), with the lazy reference update
//   PV: oacc += V(u-1)^T p_prev        v_prev = LDS address of the 32 V rows of sub-tile u-1
// MASK applies the element mask to s_cur: register r (key 8 (r/4) + 4h + r%4 of the
// sub-tile) is allowed iff 8 (r/4) + r%4 <= mask_lim (mask_lim already holds -4h).
// DP: columns computed.  64 for head dimensions up to 64 (k-steps 4..7 of the first product
// and column blocks 2, 3 of the second do not exist then), 112 for those up to 112 (no k-step
// 7), 128, or 256 for head dimensions above 128: the K and V tiles then come as two 128-column
// halves, TILE_BYTES apart in LDS, and every slice holds one MFMA of each product per half.  PART: d % 8 == 4, the K fragment that holds
// column d is cleared beyond it (part_ks = its k-step, or -1 for the lanes of the other
// half-wave).
template <bool QK, bool SM, bool PV, bool MASK, int DP, bool PART>
__device__ inline void step(f32x16& s_cur, f32x16& s_next, bf16x8 (&p_cur)[2], bf16x8 (&p_prev)[2],
                            f32x16 (&oacc)[4 * halves_of(DP)], const bf16x8 (&qf)[8 * halves_of(DP)], float& m,
                            float& l, float kappa, const uint32_t (&kaddr)[8], const uint32_t (&vaddr)[4],
                            const char* k_next, const char* v_prev, int mask_lim, int part_ks) {
    constexpr int NH = halves_of(DP), KS = ksteps_of(DP), MB = blocks_of(DP);      // per half
    // Operands of slice i are requested from LDS two slices ahead, so only a few of
    // them are live at a time; slice i holds, per half, QK MFMA i (k-step i) and PV MFMA i
    // (16-key group i / 4, 32-column block i % 4).
    bf16x8 ka[NH][8], va[NH][8];
    auto fetch = [&](int i) {
#pragma unroll
        for (int hh = 0; hh < NH; ++hh) {
            if (QK && i < KS) ka[hh][i] = lds_read_b128(k_next + hh * TILE_BYTES, k_step_addr(kaddr, i));
            if (PV && i % 4 < MB)
                va[hh][i] = lds_read_tr(v_prev + hh * TILE_BYTES + (i / 4) * 16 * 256, vaddr[i % 4]);
        }
    };
    // operands are requested this many slices ahead of their use (3 and 4 measured the same or
    // slightly worse: LDS latency is covered)
    constexpr int AHEAD = 2;
#pragma unroll
    for (int i = 0; i < AHEAD; ++i) fetch(i);
    if (SM && MASK) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (8 * (r / 4) + (r % 4) > mask_lim) s_cur[r] = -INFINITY;
    }
    if (QK) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s_next[r] = 0.f;
    }
    float rs0 = 0.f, rs1 = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_barrier(0);         // slices stay in program order
        if (i + AHEAD < 8) fetch(i + AHEAD);
        // MFMA, one score, MFMA, the other score: a wavefront that issues its MFMAs back to back
        // waits for the matrix pipeline with its VALU work still ahead of it (+2 % against
        // both MFMAs first; both exponentials before the second MFMA, or the operand requests
        // between the two, measured slightly worse)
#pragma unroll
        for (int hh = 0; hh < NH; ++hh)
            if (QK && i < KS)
                s_next = mfma(PART ? zero_beyond_d(ka[hh][i], 8 * hh + i == part_ks) : ka[hh][i], qf[8 * hh + i],
                              s_next);
        __builtin_amdgcn_sched_barrier(0);
        float p0 = 0.f;
        if (SM) {
            p0 = __builtin_amdgcn_exp2f(fmaf(s_cur[2 * i], kappa, -m));
            rs0 += p0;
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int hh = 0; hh < NH; ++hh)
            if (PV && i % 4 < MB) oacc[4 * hh + i % 4] = mfma(va[hh][i], p_prev[i / 4], oacc[4 * hh + i % 4]);
        __builtin_amdgcn_sched_barrier(0);
        if (SM) {
            const float p1 = __builtin_amdgcn_exp2f(fmaf(s_cur[2 * i + 1], kappa, -m));
            rs1 += p1;
            p_cur[i / 4][(2 * i) % 8] = (__bf16)p0;
            p_cur[i / 4][(2 * i) % 8 + 1] = (__bf16)p1;
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    if (SM) {
        float rs = rs0 + rs1;
        // The probabilities above were taken against the reference as it stood, without looking
        // at the scores first.  That is exact as long as nothing overflows (a floating-point
        // sum does not care about a common factor), so the reference only has to move when a
        // row's partial sum grows out of hand, or when the row has no reference yet (m = -inf
        // makes every term above +inf or NaN, so the same test catches it); then the sub-tile
        // is redone against the row maximum.  Wave-uniform and rare.
        if (__builtin_amdgcn_ballot_w64(!(rs < RESCALE_SUM)) != 0) {
            float mx = fmaxf(s_cur[0], s_cur[1]);
#pragma unroll
            for (int r = 2; r < 16; ++r) mx = fmaxf(mx, s_cur[r]);
            mx = half_wave_max(mx);
            const float m_new = fmaxf(m, mx * kappa);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;     // row with no key so far
            const float alpha = __builtin_amdgcn_exp2f(m - m_use);
            m = m_new;
            l *= alpha;
#pragma unroll
            for (int mb = 0; mb < halves_of(DP) * blocks_of(DP); ++mb)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[mb][r] *= alpha;
            rs = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float pr = __builtin_amdgcn_exp2f(fmaf(s_cur[r], kappa, -m_use));
                rs += pr;
                p_cur[r / 8][r % 8] = (__bf16)pr;
            }
        }
        l += rs;
    }
}

// Rotary embedding of a query row held as B-operand fragments (Sec. 2.3: a token keeps the
// position id of its original place, whatever device it sits on).  Rotate-half pairing: column
// i < d/2 with column i + d/2; with d == DP both sit in the same lane, KS/2 fragments apart.
// turns[i] = base^(-2i/d) / (2 pi) in double precision (LDS, filled once per workgroup); the
// angle in revolutions is reduced to [-1/2, 1/2] in double (position ids reach 10^6, where an
// fp32 angle is off by 0.05 rad) and only then handed to the fp32 sine / cosine instructions,
// which take revolutions.
template <int DP>
__device__ inline void rope_rotate(bf16x8 (&f)[8 * halves_of(DP)], const double* turns, int pos, int h) {
    constexpr int KS = DP / 16;
#pragma unroll
    for (int ks = 0; ks < KS / 2; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const double t = (double)pos * turns[16 * ks + 8 * h + e];
            const float r = (float)(t - rint(t));
            const float sn = __builtin_amdgcn_sinf(r), cs = __builtin_amdgcn_cosf(r);
            const float lo = (float)f[ks][e], hi = (float)f[ks + KS / 2][e];
            f[ks][e] = (__bf16)fmaf(lo, cs, -hi * sn);
            f[ks + KS / 2][e] = (__bf16)fmaf(hi, cs, lo * sn);
        }
}

// One code path serves every step: a block is walked up to the last key tile that holds an
// allowed pair, and the last BM / 64 tiles of the walk carry the element mask.  For a
// triangular block the mask limit is the query's own position; for a full block (contiguous
// layout, q_dev > kv_dev) it is the last key, c - 1, which for a multiple of 128 masks
// nothing.  RAGGED: c is not a multiple of 128.  The last query tile then holds rows beyond
// the shard (their loads are clamped to the last row, their results are not stored) and the
// last key tiles hold keys beyond it (the tile loads return zeros there and the mask removes
// them).
// (FULL is a template argument rather than a launch argument so that profiler traces name
// triangular and full launches apart; the code is the same.)
// ROPE: the query rows are rotated by their position ids as they are loaded (d == DP).
template <bool RAGGED, bool FULL, int DP, bool PART, bool ROPE = false>
__global__ void __launch_bounds__(64 * NW, DP > 128 ? 1 : 2)
fwd_mfma_kernel(StepArgs p, int n_qtiles) {
    constexpr int NH = halves_of(DP), KS = ksteps_of(DP), MB = halves_of(DP) * blocks_of(DP);      // k-steps per half, column blocks
    __shared__ double rope_turns[ROPE ? DP / 2 : 1];
    // one LDS object per tile buffer (two 128-column halves each when DP = 256)
    __shared__ __attribute__((aligned(1024))) char k_lds0[TILE_BYTES * NH];
    __shared__ __attribute__((aligned(1024))) char k_lds1[TILE_BYTES * NH];
    __shared__ __attribute__((aligned(1024))) char v_lds0[TILE_BYTES * NH];
    __shared__ __attribute__((aligned(1024))) char v_lds1[TILE_BYTES * NH];

    const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform, kept scalar
    int rank, bh;
    decode_block<true>((int)blockIdx.x, n_qtiles, p.B * p.H, rank, bh);
    const int qt = n_qtiles - 1 - rank;      // triangular steps: heaviest query tiles first
    const int b = bh / p.H, hd = bh - b * p.H;
    const int64_t base = b * p.stride_b + hd * p.stride_h;
    // key/value head of this query head's group (the same head when H_kv == H)
    const int64_t kv_base = b * p.kv_stride_b + (hd / (p.H / p.H_kv)) * p.kv_stride_h;
    const __bf16* Q = (const __bf16*)p.q + base;
    const int d = p.d;                                 // d <= DP, zero-padded to DP columns
    const int64_t ss = p.stride_s;                     // elements between consecutive rows of Q and O
    const int pitch = 2 * (int)p.kv_stride_s;          // bytes between consecutive rows of K and V
    const int tile_pitch = TILE_ROWS * pitch;          // bytes between 64-row tiles in global memory
    const dt_rsrc K = dt_make_rsrc((const __bf16*)p.k + kv_base, p.c, pitch, d);
    const dt_rsrc V = dt_make_rsrc((const __bf16*)p.v + kv_base, p.c, pitch, d);
    float* O = p.o + base;
    float* L = p.lse + b * p.stat_stride_b + hd * p.stat_stride_h;

    const int q0 = qt * BM;
    const int a_own = q0 + 32 * wave + n;     // this lane's query row
    const bool row_ok = !RAGGED || a_own < p.c;
    const int a = RAGGED ? min(a_own, p.c - 1) : a_own;      // the row it loads
    constexpr bool full_block = FULL;                // every key allowed: the mask limit is the last key
    // 64-key tiles holding at least one allowed pair for the workgroup.  Triangular: keys
    // b <= a - off, i.e. tiles 0 .. (q0 + 127) / 64.  All four wavefronts walk all 2 n_kt
    // sub-tiles (at most NW - 1 of them are entirely masked for a wavefront); the element
    // mask is applied on the last NW sub-tiles only.
    const int n_kt_fine = full_block ? 2 * n_qtiles : (q0 + BM) / TILE_ROWS;
    int n_kt = n_kt_fine;
    if (!full_block && p.skip_bq > 0) {
        // emulated coarse skipping: up to the last skip_bk-wide key tile that shares an allowed
        // pair with the skip_bq-tall tile these queries belong to
        const int q_hi = (q0 / p.skip_bq + 1) * p.skip_bq - 1;
        n_kt = min(p.c, ((q_hi - p.off) / p.skip_bk + 1) * p.skip_bk) / TILE_ROWS;
    }
    // sub-tile v: register r (key 32 v + 8 (r/4) + 4h + r%4) is allowed iff
    // 8 (r/4) + r%4 <= mask_base - 32 v
    const int mask_base = (full_block ? p.c - 1 : a_own - p.off) - 4 * h;

    // per-lane addresses: K A-operand reads per k-step, V transposing reads per 32-column
    // block (bytes within a 32-row half tile), and the global byte offsets of this lane's
    // direct loads
    uint32_t kaddr[8], vaddr[4], kg0[NH], vg0[NH];
    {
        const int x = n & 15;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) kaddr[ks] = n * 256 + (((2 * ks + h) ^ x) << 4);
        const int i = lane & 15, nh = (lane >> 4) & 1, j4 = i >> 2;
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
            vaddr[mb] = (4 * h + j4) * 256 + ((4 * (mb ^ j4) + 2 * nh + ((i & 3) >> 1)) << 4) + (i & 1) * 8;
        const int lr = lane >> 4, pc = lane & 15;      // row within the 4-row group, physical chunk
#pragma unroll
        for (int hh = 0; hh < NH; ++hh) {
            // row 4 wave + lr of each 16; half hh of the rows starts 256 bytes in
            kg0[hh] = (4 * wave + lr) * pitch + 256 * hh + ((pc ^ (4 * wave + lr)) << 4);
            // V's swizzle depends on the row within the 4-row group only, so its four pieces
            // differ by exactly four rows: one lane offset, the rest goes into the scalar offset
            vg0[hh] = (4 * LPW * wave + lr) * pitch + 256 * hh + ((pc ^ (lr << 2)) << 4);
            // chunks that start at or beyond column d are not fetched: their LDS columns get zeros
            if (128 * hh + 8 * (pc ^ (4 * wave + lr)) >= d) kg0[hh] = DT_OUT_OF_RANGE;
            if (128 * hh + 8 * (pc ^ (lr << 2)) >= d) vg0[hh] = DT_OUT_OF_RANGE;
        }
    }

    auto load_k = [&](int tile_byte_offset, char* buf) {
#pragma unroll
        for (int hh = 0; hh < NH; ++hh)
            load_tile_direct(K, tile_byte_offset, buf + hh * TILE_BYTES, kg0[hh], wave, pitch);
    };
    auto load_v = [&](int tile_byte_offset, char* buf) {
#pragma unroll
        for (int hh = 0; hh < NH; ++hh)
            load_v_tile_direct(V, tile_byte_offset, buf + hh * TILE_BYTES, vg0[hh], wave, pitch);
    };
    // first tiles on their way while the running state is loaded
    load_k(0, k_lds0);
    load_v(0, v_lds0);
    load_k(tile_pitch, k_lds1);     // n_kt >= 2 always

    bf16x8 qf[8 * NH];
    load_b_frags<8 * NH>(qf, Q + (int64_t)a * ss, h, d);
    int q_position = 0;
    if (ROPE) {
        q_position = p.q_pos[b * p.pos_stride_b + a];
        if (tid < DP / 2) rope_turns[tid] = exp2(-2.0 * tid / DP * p.rope_log2_base) * 0.15915494309189535;
    }
    const float kappa = p.scale * LOG2E;
    // This block's own partial result is accumulated from an empty state and folded into the
    // running (O, LSE) in the epilogue, where the running state is read.  Read here instead, it
    // sits in front of the first tile of every workgroup of the launch at once (the fp32 state
    // is the largest tensor of a step), which is what a short step spends a quarter of its time on.
    float m = -INFINITY;                      // no reference yet: the first sub-tile sets it
    float l = 0.f;                            // the two half-waves hold partial row sums
    f32x16 oacc[4 * NH];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[mb][r] = 0.f;

    __builtin_amdgcn_s_waitcnt(0);     // the direct loads have landed (vmcnt) ...
    __syncthreads();                   // ... for every wavefront
    if (ROPE) rope_rotate<DP>(qf, rope_turns, q_position, h);

    // PART: k-step whose fragment, in this half-wave, is the chunk holding column d
    const int part_ks = (PART && ((d >> 3) & 1) == h) ? (d >> 4) : -1;
    f32x16 s_a, s_b;
    bf16x8 p_a[2], p_b[2];
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
        for (int e = 0; e < 8; ++e) p_a[g][e] = p_b[g][e] = (__bf16)0.f;
    // prologue: S(0)
    {
#pragma unroll
        for (int r = 0; r < 16; ++r) s_a[r] = 0.f;
#pragma unroll
        for (int hh = 0; hh < NH; ++hh)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 ka = lds_read_b128(k_lds0 + hh * TILE_BYTES, k_step_addr(kaddr, ks));
                s_a = mfma(PART ? zero_beyond_d(ka, 8 * hh + ks == part_ks) : ka, qf[8 * hh + ks], s_a);
            }
    }

    // Trip t = iterations u = 2t and 2t+1 with barrier t between them.  Iteration u does
    // QK(u+1), softmax(u), PV(u-1); S(even) lives in s_a, S(odd) in s_b, P likewise.
    //   u = 2t:   QK(2t+1): K tile t, second half      PV(2t-1): V tile t-1, second half
    //   barrier t: K tile t and V tile t-1 are free -> load K(t+2), V(t+1); K(t+1), V(t),
    //              requested at barrier t-1, have landed
    //   u = 2t+1: QK(2t+2): K tile t+1, first half     PV(2t): V tile t, first half
    // PAR = t & 1 fixes every LDS offset at compile time.
    // LD: which of the two tile requests of the trip exist: 2 = K(t+2) and V(t+1), 1 = V(t+1)
    // only (the last trip but one), 0 = none (the last trip)
    auto trip = [&](auto first_c, auto last_c, auto mask_c, auto par_c, int t, auto ld_c) __attribute__((always_inline)) {
        constexpr bool FIRST = decltype(first_c)::value, LAST = decltype(last_c)::value;
        constexpr bool MASK = decltype(mask_c)::value;
        constexpr int PAR = decltype(par_c)::value, LD = decltype(ld_c)::value;
        char* const k_cur = PAR ? k_lds1 : k_lds0;
        char* const k_nxt = PAR ? k_lds0 : k_lds1;
        char* const v_cur = PAR ? v_lds1 : v_lds0;
        char* const v_prv = PAR ? v_lds0 : v_lds1;
        step<true, true, !FIRST, MASK, DP, PART>(s_a, s_b, p_a, p_b, oacc, qf, m, l, kappa, kaddr, vaddr,
                                                 k_cur + TILE_BYTES / 2, v_prv + TILE_BYTES / 2,
                                                 mask_base - 64 * t, part_ks);
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (LD >= 2) load_k((t + 2) * tile_pitch, k_cur);
        if (LD >= 1) load_v((t + 1) * tile_pitch, v_prv);
        step<!LAST, true, true, MASK, DP, PART>(s_b, s_a, p_b, p_a, oacc, qf, m, l, kappa, kaddr, vaddr, k_nxt,
                                                v_cur, mask_base - 64 * t - 32, part_ks);
    };
    using T = std::true_type;
    using F = std::false_type;
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    using L0 = std::integral_constant<int, 0>;
    using L1 = std::integral_constant<int, 1>;
    using L2 = std::integral_constant<int, 2>;
    // The number of trips is even (tiles come in pairs of 64 keys per 128-row block), so the
    // walk is a sequence of (even, odd) pairs of fixed form: the first pair, plain pairs (the
    // hot loop), masked pairs, the last pair.  Triangular steps: the trips from t_mask on carry
    // the element mask (the last BM / 64 ones, more under emulated coarse skipping).
    const int t_mask = n_kt_fine - BM / TILE_ROWS;
    if (n_kt == 2) {                   // a single pair (triangular: the first query tile)
        trip(T{}, F{}, T{}, P0{}, 0, L1{});
        trip(F{}, T{}, T{}, P1{}, 1, L0{});
    } else {
        if (t_mask == 0) {      // masked from the start (emulated coarse skipping only)
            trip(T{}, F{}, T{}, P0{}, 0, L2{});
            trip(F{}, F{}, T{}, P1{}, 1, L2{});
        } else {
            trip(T{}, F{}, F{}, P0{}, 0, L2{});
            trip(F{}, F{}, F{}, P1{}, 1, L2{});
        }
        int t = 2;
        const int t_plain = min(t_mask, n_kt - 2);
        for (; t < t_plain; t += 2) {                  // the hot loop: two plain trips per turn
            trip(F{}, F{}, F{}, P0{}, t, L2{});
            trip(F{}, F{}, F{}, P1{}, t + 1, L2{});
        }
        for (; t < n_kt - 2; t += 2) {                 // masked pairs before the last one
            trip(F{}, F{}, T{}, P0{}, t, L2{});
            trip(F{}, F{}, T{}, P1{}, t + 1, L2{});
        }
        trip(F{}, F{}, T{}, P0{}, n_kt - 2, L1{});    // the last pair always carries the mask
        trip(F{}, T{}, T{}, P1{}, n_kt - 1, L0{});
    }
    // final iteration u = 2 n_kt: PV(2 n_kt - 1): V tile n_kt - 1, second half; P in p_b
    {
        const char* v_last = v_lds1 + TILE_BYTES / 2;          // n_kt - 1 is odd
        step<false, false, true, false, DP, PART>(s_a, s_b, p_a, p_b, oacc, qf, m, l, kappa, kaddr, vaddr, v_last,
                                                  v_last, 0, part_ks);
    }

    // epilogue: merge this block's partial (unnormalised oacc against reference m, row sum l)
    // into the running state by log-sum-exp (Alg. 1: accumulate into the output and update the
    // running softmax statistics), everything in base-2 units:
    //   LSE' = log2(2^LSE + 2^(m + log2 l)),  O' = O 2^(LSE - LSE') + oacc 2^(m - LSE')
    // A row that saw no key here (l = 0) keeps its state bit for bit; a row whose state is still
    // empty (LSE = -inf) takes the partial and never looks at the stored O.
    const float l_tot = half_wave_sum(l);
    const float lse_old = L[a] * LOG2E;                                       // -inf stays -inf
    const float lse_part = l_tot > 0.f ? m + __builtin_amdgcn_logf(l_tot) : -INFINITY;
    const float top = fmaxf(lse_old, lse_part);
    const float ref = top == -INFINITY ? 0.f : top;                           // no (-inf) - (-inf)
    const float w_old = __builtin_amdgcn_exp2f(lse_old - ref), w_part = __builtin_amdgcn_exp2f(lse_part - ref);
    const float w_sum = w_old + w_part;
    const float inv = w_sum > 0.f ? 1.f / w_sum : 0.f;
    const float a_old = w_old * inv;
    const float a_part = l_tot > 0.f ? w_part * inv / l_tot : 0.f;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int col = 32 * mb + 8 * g + 4 * h;
            if (col >= d || !row_ok) continue;            // padding columns, rows beyond the shard
            float4* dst = reinterpret_cast<float4*>(O + (int64_t)a * ss + col);
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
            if (a_old != 0.f) {
                x = *dst;
                x.x *= a_old; x.y *= a_old; x.z *= a_old; x.w *= a_old;
            }
            x.x = fmaf(oacc[mb][4 * g + 0], a_part, x.x); x.y = fmaf(oacc[mb][4 * g + 1], a_part, x.y);
            x.z = fmaf(oacc[mb][4 * g + 2], a_part, x.z); x.w = fmaf(oacc[mb][4 * g + 3], a_part, x.w);
            *dst = x;
        }
    if (h == 0 && row_ok) L[a] = (top + __builtin_amdgcn_logf(w_sum)) * LN2;
}

}  // namespace

bool fwd_mfma_supported(const StepArgs& a, int dtype) {
    // the tile loads address a shard through a buffer descriptor with 32-bit byte offsets:
    // the last row of its last (possibly partial) tile pair must end below 2^31 bytes from
    // its first
    const int64_t rows = (int64_t)(a.c + BM - 1) / BM * BM;
    // one workgroup per (128-row tile, batch, head) in a 1-D grid
    if (rows / BM * a.B * a.H >= (int64_t(1) << 31)) return false;
    // head dimensions above 128 (two 128-column halves) in whole 16-byte chunks only
    if (a.d > 2 * D || (a.d > D && a.d % 8)) return false;
    return dtype == SA_BF16 && a.d % 4 == 0 && a.c >= BM &&
           rows * 2 * a.kv_stride_s + 2 * a.d < (int64_t(1) << 31);
}

namespace {
template <int DP, bool PART>
void launch_fwd_variant(const StepArgs& a, hipStream_t st, dim3 grid, dim3 block, int n_qtiles) {
    const bool full = a.kind == MASK_FULL;
    if (a.c % BM) {
        if (full) hipLaunchKernelGGL((fwd_mfma_kernel<true, true, DP, PART>), grid, block, 0, st, a, n_qtiles);
        else hipLaunchKernelGGL((fwd_mfma_kernel<true, false, DP, PART>), grid, block, 0, st, a, n_qtiles);
    } else {
        if (full) hipLaunchKernelGGL((fwd_mfma_kernel<false, true, DP, PART>), grid, block, 0, st, a, n_qtiles);
        else hipLaunchKernelGGL((fwd_mfma_kernel<false, false, DP, PART>), grid, block, 0, st, a, n_qtiles);
    }
}
template <int DP>
void launch_fwd_rope(const StepArgs& a, hipStream_t st, dim3 grid, dim3 block, int n_qtiles) {
    if (a.kind == MASK_FULL) hipLaunchKernelGGL((fwd_mfma_kernel<false, true, DP, false, true>), grid, block, 0, st, a, n_qtiles);
    else hipLaunchKernelGGL((fwd_mfma_kernel<false, false, DP, false, true>), grid, block, 0, st, a, n_qtiles);
}
}  // namespace

// fused query rotation: head dimension 64, 128 or 256 (both halves of a rotation pair in one
// lane) and block sizes that are a multiple of 128
bool fwd_mfma_rope_supported(const StepArgs& a, int dtype) {
    return fwd_mfma_supported(a, dtype) && (a.d == 64 || a.d == 128 || a.d == 256) && a.c % BM == 0;
}

hipError_t launch_fwd_mfma(const StepArgs& a, hipStream_t st) {
    const int n_qtiles = (a.c + BM - 1) / BM;
    const dim3 grid((unsigned)n_qtiles * a.B * a.H), block(64 * NW);
    const bool part = a.d % 8 != 0;
    if (a.q_pos) {
        if (a.d == 64) launch_fwd_rope<64>(a, st, grid, block, n_qtiles);
        else if (a.d == 128) launch_fwd_rope<128>(a, st, grid, block, n_qtiles);
        else launch_fwd_rope<256>(a, st, grid, block, n_qtiles);
    } else if (a.d > 128) {
        launch_fwd_variant<256, false>(a, st, grid, block, n_qtiles);
    } else if (a.d <= 64) {
        if (part) launch_fwd_variant<64, true>(a, st, grid, block, n_qtiles);
        else launch_fwd_variant<64, false>(a, st, grid, block, n_qtiles);
    } else if (a.d <= 112) {
        if (part) launch_fwd_variant<112, true>(a, st, grid, block, n_qtiles);
        else launch_fwd_variant<112, false>(a, st, grid, block, n_qtiles);
    } else {
        if (part) launch_fwd_variant<128, true>(a, st, grid, block, n_qtiles);
        else launch_fwd_variant<128, false>(a, st, grid, block, n_qtiles);
    }
    return hipGetLastError();
}

}  // namespace sa
