// Backward ring step on the CDNA4 matrix cores (bf16 operands, fp32 accumulate),
// head dimension up to 256 (64, 112, 128 or 256 columns computed).  The paper describes no
// backward pass; this is the analytic gradient of causal attention (Sec. 2.1) restricted to the pairs that
// GetMask(j, k) allows, with P recomputed from the saved log-sum-exp:
//   P = exp(scale q.k - LSE),  dV += P^T dO,  dP = dO V^T,
//   dS = P * (dP - delta),     dQ += scale dS K,  dK += scale dS^T Q.
// Two deterministic kernels, no atomics: every output row is read-modify-written
// by exactly one wavefront.
//
//  * dq kernel: a workgroup owns 128 query rows (Q and dO stay in registers as
//    B operands), key tiles stream through LDS.  S^T = K Q^T and dP^T = V dO^T
//    put 16 + 16 keys of ONE query in a lane, so LSE and delta are per-lane
//    scalars and dS^T is already the B operand of dQ^T += K^T dS^T.
//  * dkdv kernel: a workgroup owns 128 key rows (K and V in registers), query
//    tiles stream through LDS.  S = Q K^T and dP = dO V^T put 16 + 16 queries of
//    ONE key in a lane; P and dS are the B operands of dV^T += dO^T P and
//    dK^T += Q^T dS.
// Both skip every tile the mask empties (Sec. 2.2.1) per 32-row wavefront and
// apply the element mask only on the tiles that can cross the diagonal (the dq
// kernel also on the last tile pair of a full block, where it removes nothing
// unless the block size is not a multiple of 128).
#include <hip/hip_bf16.h>

#include <type_traits>

#include "mfma_tiles.h"
#include "sa_internal.h"

namespace sa {

namespace {

constexpr int BM = 128;   // rows owned by a workgroup (queries in dq, keys in dkdv)
constexpr int BN = TR;    // rows streamed per tile
constexpr int D = TD;

__device__ inline bf16x8 pack8(const f32x16& x, int first) {
    bf16x8 r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = (__bf16)x[first + e];
    return r;
}

// ---------------------------------------------------------------- dQ kernel
// K and V tiles (64 key rows) stream global -> LDS directly into swizzled tiles, two
// buffers each.  The loop runs over 32-key sub-tiles u; iteration u issues, interleaved
// slice by slice,
//     S^T(u+1) = K(u+1) Q^T, dP^T(u+1) = V(u+1) dO^T   (16 MFMA)
//     P(u) = exp2(S(u) kappa - LSE), dS(u) = P (dP(u) - delta)   (VALU)
// and then dQ^T += K(u)^T dS(u)^T (8 MFMA, K^T through the transposing LDS read).
// Two barriers per 64-key tile: one makes the tile requested one iteration earlier
// visible, one releases the tile just finished for the next request.

// DP: columns computed.  64 for head dimensions up to 64 (k-steps 4..7 of the S and dP
// products and column blocks 2, 3 of the dQ product do not exist then), 112 for those up to 112
// (no k-step 7), 128, or 256 for head dimensions above 128: the K and V tiles then come as two 128-column halves, DT_BYTES apart in
// LDS, and every slice holds one MFMA of each product per half.  PART: d % 8 == 4, the K and V
// fragments that hold column d are cleared beyond it (part_ks = the k-step, or -1 for the lanes
// of the other half-wave).
template <bool NEXT, bool MASK, int DP, bool PART>
__device__ inline void dq_step(f32x16& s_cur, f32x16& dp_cur, f32x16& s_next, f32x16& dp_next,
                               f32x16 (&acc)[4 * halves_of(DP)], const bf16x8 (&qf)[8 * halves_of(DP)],
                               const bf16x8 (&gf)[8 * halves_of(DP)], float kappa, float lse2, float delta,
                               const uint32_t (&arow)[8], const uint32_t (&tr0)[4], const uint32_t (&tr1)[4],
                               const char* k_next, const char* v_next, const char* k_cur, int mask_lim,
                               int part_ks) {
    constexpr int NH = halves_of(DP), KS = ksteps_of(DP), MB = blocks_of(DP);      // per half
    bf16x8 ka[NH][8], va[NH][8], kt[NH][8], dsb[2];
    auto fetch = [&](int i) {
        if (NEXT && i < KS) {
#pragma unroll
            for (int hh = 0; hh < NH; ++hh) {
                ka[hh][i] = dt_read_row(k_next + hh * DT_BYTES, arow[i]);
                va[hh][i] = dt_read_row(v_next + hh * DT_BYTES, arow[i]);
            }
        }
    };
    auto fetch_t = [&](int i) {
        if (i % 4 < MB) {
#pragma unroll
            for (int hh = 0; hh < NH; ++hh)
                kt[hh][i] = dt_read_tr(k_cur + hh * DT_BYTES + (i / 4) * 16 * 256, tr0[i % 4], tr1[i % 4]);
        }
    };
    fetch(0);
    fetch(1);
    if (NEXT) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s_next[r] = dp_next[r] = 0.f;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_barrier(0);          // slices stay in program order
        if (i + 2 < 8) fetch(i + 2);
        if (i >= 4) fetch_t(i - 4);                 // first half of the K^T operands
        if (NEXT && i < KS) {
#pragma unroll
            for (int hh = 0; hh < NH; ++hh) {
                const bool last_chunk = 8 * hh + i == part_ks;
                s_next = mfma(PART ? zero_beyond_d(ka[hh][i], last_chunk) : ka[hh][i], qf[8 * hh + i], s_next);
                dp_next = mfma(PART ? zero_beyond_d(va[hh][i], last_chunk) : va[hh][i], gf[8 * hh + i], dp_next);
            }
        }
#pragma unroll
        for (int r = 2 * i; r < 2 * i + 2; ++r) {
            float pr = __builtin_amdgcn_exp2f(fmaf(s_cur[r], kappa, -lse2));
            if (MASK && 8 * (r / 4) + (r % 4) > mask_lim) pr = 0.f;
            dsb[r / 8][r % 8] = (__bf16)(pr * (dp_cur[r] - delta));
        }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        if (i + 4 < 8) fetch_t(i + 4);
        if (i % 4 < MB) {
#pragma unroll
            for (int hh = 0; hh < NH; ++hh) acc[4 * hh + i % 4] = mfma(kt[hh][i], dsb[i / 4], acc[4 * hh + i % 4]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// One code path serves triangular and full blocks, as in the forward kernel: the last two
// tiles of the walk carry the element mask, whose limit is the query's own position, or the
// last key (c - 1) for a full block.  RAGGED (c not a multiple of 128): loads of rows beyond
// the shard are clamped, their results are not stored, keys beyond it come in as zero rows
// and are removed by the mask.
// (FULL is a template argument rather than a launch argument so that profiler traces name
// triangular and full launches apart; the code is the same.)
template <bool RAGGED, bool FULL, int DP, bool PART>
__global__ void __launch_bounds__(256, DP > 128 ? 1 : 2)
bwd_dq_mfma_kernel(StepArgs p, int n_tiles) {
    constexpr int NH = halves_of(DP), KS = ksteps_of(DP), MB = halves_of(DP) * blocks_of(DP);      // k-steps per half, column blocks
    // one LDS object per tile buffer (two 128-column halves each when DP = 256)
    __shared__ __attribute__((aligned(1024))) char k_lds0[DT_BYTES * NH];
    __shared__ __attribute__((aligned(1024))) char k_lds1[DT_BYTES * NH];
    __shared__ __attribute__((aligned(1024))) char v_lds0[DT_BYTES * NH];
    __shared__ __attribute__((aligned(1024))) char v_lds1[DT_BYTES * NH];

    const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform, kept scalar
    int rank, bh;
    decode_block<true>((int)blockIdx.x, n_tiles, p.B * p.H, rank, bh);
    const int qt = n_tiles - 1 - rank;      // heaviest query tiles first
    const int b = bh / p.H, hd = bh - b * p.H;
    const int64_t base = b * p.stride_b + hd * p.stride_h;
    // key/value head of this query head's group (the same head when H_kv == H)
    const int64_t kv_base = b * p.kv_stride_b + (hd / (p.H / p.H_kv)) * p.kv_stride_h;
    const int64_t sbase = b * p.stat_stride_b + hd * p.stat_stride_h;
    const __bf16* Q = (const __bf16*)p.q + base;
    const int d = p.d;                                 // d <= DP, zero-padded to DP columns
    const int64_t ss = p.stride_s;                     // elements between consecutive rows of Q, dO, dQ
    const int pitch = 2 * (int)p.kv_stride_s;          // bytes between consecutive rows of K and V
    const int tile_pitch = DT_ROWS * pitch;            // bytes between 64-row tiles in global memory
    const dt_rsrc Kr = dt_make_rsrc((const __bf16*)p.k + kv_base, p.c, pitch, d);
    const dt_rsrc Vr = dt_make_rsrc((const __bf16*)p.v + kv_base, p.c, pitch, d);
    const __bf16* G = (const __bf16*)p.dout + base;
    float* DQ = p.dq + base;

    const int q0 = qt * BM, a_own = q0 + 32 * wave + n;
    const bool row_ok = !RAGGED || a_own < p.c;
    const int a = RAGGED ? min(a_own, p.c - 1) : a_own;      // the row this lane loads
    constexpr bool full_block = FULL;                // every key allowed: the mask limit is the last key
    // all four wavefronts walk the 2 n_kt sub-tiles of the workgroup (at most three are
    // entirely masked for a wavefront); the element mask runs on the last four only
    const int n_kt_fine = full_block ? 2 * n_tiles : (q0 + BM) / DT_ROWS;
    int n_kt = n_kt_fine;
    if (!full_block && p.skip_bq > 0) {       // emulated coarse skipping, as in the forward kernel
        const int q_hi = (q0 / p.skip_bq + 1) * p.skip_bq - 1;
        n_kt = min(p.c, ((q_hi - p.off) / p.skip_bk + 1) * p.skip_bk) / DT_ROWS;
    }
    // sub-tile v: allowed iff 8 (r/4) + r%4 <= mask_base - 32 v
    const int mask_base = (full_block ? p.c - 1 : a_own - p.off) - 4 * h;

    uint32_t arow[8], tr0[4], tr1[4], gl[NH][4];
    dt_row_addrs(arow, n, h);
    dt_tr_addrs(tr0, tr1, lane);
#pragma unroll
    for (int hh = 0; hh < NH; ++hh) dt_load_offsets(gl[hh], lane, wave, pitch, d, hh);
    auto load_tile = [&](dt_rsrc m, int tile_byte_offset, char* buf) {
#pragma unroll
        for (int hh = 0; hh < NH; ++hh) dt_load(m, tile_byte_offset, buf + hh * DT_BYTES, gl[hh], wave);
    };
    load_tile(Kr, 0, k_lds0);
    load_tile(Vr, 0, v_lds0);
    load_tile(Kr, tile_pitch, k_lds1);       // n_kt >= 2 always
    load_tile(Vr, tile_pitch, v_lds1);

    bf16x8 qf[8 * NH], gf[8 * NH];
    load_b_frags<8 * NH>(qf, Q + (int64_t)a * ss, h, d);
    load_b_frags<8 * NH>(gf, G + (int64_t)a * ss, h, d);
    const float kappa = p.scale * LOG2E;
    float lse2 = p.lse[sbase + a] * LOG2E;
    float delta = p.delta[sbase + a];
    f32x16 acc[4 * NH];
#pragma unroll
    for (int mb = 0; mb < 4 * NH; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mb][r] = 0.f;

    // the statistics are complete here: a load left pending into the loop would be waited
    // for there, together with the tile loads just issued
    asm volatile("" : "+v"(lse2), "+v"(delta));
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    // PART: k-step whose fragment, in this half-wave, is the chunk holding column d
    const int part_ks = (PART && ((d >> 3) & 1) == h) ? (d >> 4) : -1;
    f32x16 s_a, s_b, dp_a, dp_b;
    {   // prologue: S(0), dP(0)
#pragma unroll
        for (int r = 0; r < 16; ++r) s_a[r] = dp_a[r] = 0.f;
#pragma unroll
        for (int hh = 0; hh < NH; ++hh)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 ka = dt_read_row(k_lds0 + hh * DT_BYTES, arow[ks]);
                const bf16x8 va = dt_read_row(v_lds0 + hh * DT_BYTES, arow[ks]);
                s_a = mfma(PART ? zero_beyond_d(ka, 8 * hh + ks == part_ks) : ka, qf[8 * hh + ks], s_a);
                dp_a = mfma(PART ? zero_beyond_d(va, 8 * hh + ks == part_ks) : va, gf[8 * hh + ks], dp_a);
            }
    }

    // Trip t = iterations 2t (scores in *_a) and 2t+1 (scores in *_b); PAR = t & 1 selects
    // the buffers of tile t at compile time.
    auto trip = [&](auto last_c, auto mask_c, auto par_c, int t) {
        constexpr bool LAST = decltype(last_c)::value, MASK = decltype(mask_c)::value;
        constexpr int PAR = decltype(par_c)::value;
        char* const k_cur = PAR ? k_lds1 : k_lds0;
        char* const v_cur = PAR ? v_lds1 : v_lds0;
        char* const k_nxt = PAR ? k_lds0 : k_lds1;
        char* const v_nxt = PAR ? v_lds0 : v_lds1;
        dq_step<true, MASK, DP, PART>(s_a, dp_a, s_b, dp_b, acc, qf, gf, kappa, lse2, delta, arow, tr0, tr1,
                                      k_cur + DT_BYTES / 2, v_cur + DT_BYTES / 2, k_cur, mask_base - 64 * t,
                                      part_ks);
        if (!LAST) {
            __builtin_amdgcn_s_waitcnt(0);      // tile t+1, requested one iteration ago, has landed
            __syncthreads();
        }
        dq_step<!LAST, MASK, DP, PART>(s_b, dp_b, s_a, dp_a, acc, qf, gf, kappa, lse2, delta, arow, tr0, tr1,
                                       k_nxt, v_nxt, k_cur + DT_BYTES / 2, mask_base - 64 * t - 32, part_ks);
        if (!LAST) {
            __syncthreads();                    // every wavefront is done with tile t
            if (t + 2 < n_kt) {
                load_tile(Kr, (t + 2) * tile_pitch, k_cur);
                load_tile(Vr, (t + 2) * tile_pitch, v_cur);
            }
        }
    };
    using T = std::true_type;
    using F = std::false_type;
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    // trips before the last tile pair of the fine walk without the element mask, then masked
    // trips: two, more under emulated coarse skipping (n_kt_fine and n_kt are even)
    int t = 0;
    for (; t + 2 < n_kt_fine; t += 2) {
        trip(F{}, F{}, P0{}, t);
        trip(F{}, F{}, P1{}, t + 1);
    }
    for (; t + 2 < n_kt; t += 2) {
        trip(F{}, T{}, P0{}, t);
        trip(F{}, T{}, P1{}, t + 1);
    }
    trip(F{}, T{}, P0{}, t);
    trip(T{}, T{}, P1{}, t + 1);

#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int col = 32 * mb + 8 * g + 4 * h;
            if (col >= d || !row_ok) continue;            // padding columns, rows beyond the shard
            float4* dst = reinterpret_cast<float4*>(DQ + (int64_t)a * ss + col);
            float4 x = *dst;
            x.x = fmaf(p.scale, acc[mb][4 * g + 0], x.x); x.y = fmaf(p.scale, acc[mb][4 * g + 1], x.y);
            x.z = fmaf(p.scale, acc[mb][4 * g + 2], x.z); x.w = fmaf(p.scale, acc[mb][4 * g + 3], x.w);
            *dst = x;
        }
}

// ------------------------------------------------------------- dK/dV kernel
// MFMA whose accumulator is pinned to ordinary VGPRs.  The dK/dV kernel needs more than 256
// registers, and once a kernel uses AGPRs the compiler places EVERY MFMA result there; the
// S / dP tiles are consumed by VALU instructions, so they would be copied back register by
// register.
//
// Issued from inline assembly, these MFMAs are invisible to the compiler's hazard recogniser,
// so the one software-managed hazard they have is kept by hand.  ISA guide, "Manually inserted
// wait states (NOPs)": XDL (matrix core) write of a VGPR followed by a VALU read or write of
// it needs passes + 3 wait states: 11 for this 8-pass instruction (19 for a 16-pass one).
//  * In the loops the distance is structural: the last S / dP MFMA of a pipeline step is
//    followed by that step's dV / dK products, 4 * MB >= 8 further MFMAs of 8 passes each
//    (>= 256 cycles of the same in-order pipeline), before the next step's first VALU read.
//  * In the prologue nothing lies between: mfma_results_to_valu() inserts 32 wait states and
//    ties the two tiles to the asm statement, so no read of them can be scheduled before it.
__device__ inline void mfma_results_to_valu(f32x16& a, f32x16& b) {
    asm volatile("s_nop 15\n\ts_nop 15" : "+v"(a), "+v"(b));
}
// The other software-managed hazard is on the input side: a VALU write of a VGPR followed by
// an MFMA read of it needs 2 wait states (same table).  The operands normally come straight
// from LDS reads (ordered by s_waitcnt, no hazard); only the PART instantiations pass them
// through VALU selects first (zero_beyond_d), and then AFTER_VALU puts the wait in front of
// the instruction.
template <bool AFTER_VALU>
__device__ inline void mfma_vgpr_first(f32x16& acc, bf16x8 a, bf16x8 b) {
    if (AFTER_VALU) asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "v"(b));
    else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "v"(b));
}
template <bool AFTER_VALU>
__device__ inline void mfma_vgpr_acc(f32x16& acc, bf16x8 a, bf16x8 b) {
    if (AFTER_VALU) asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
    else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}

// S / dP product of the dK/dV kernel.  DP <= 128: the asm forms above (results stay in VGPRs).
// DP = 256: the compiler's own MFMA; K and V alone are 128 registers there, the asm forms would
// pin them and the score tiles to VGPRs and spill a hundred registers, while the compiler keeps
// part of them in AGPRs and copies a score tile back when the VALU code wants it (32 copies
// against 48 MFMAs per step, affordable at this head dimension).
template <int DP, bool PART>
__device__ inline void score_mfma(f32x16& acc, bf16x8 a, bf16x8 b, bool first) {
    if (DP > 128) {
        if (first) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        }
        acc = mfma(a, b, acc);
    } else if (first) {
        mfma_vgpr_first<PART>(acc, a, b);
    } else {
        mfma_vgpr_acc<PART>(acc, a, b);
    }
}

// A workgroup owns 128 key rows (K and V rows in registers as B operands, dK^T and
// dV^T accumulators in registers: one wavefront per SIMD with the large register
// budget).  Q and dO tiles (64 query rows) stream global -> LDS directly into swizzled
// tiles, two buffers each; LSE * log2(e) and delta of the tile's rows are staged
// beside them.  Iteration u over 32-query sub-tiles issues, interleaved slice by slice,
//     S(u+1) = Q(u+1) K^T, dP(u+1) = dO(u+1) V^T - delta   (16 MFMA; the dP accumulators
//                              start from -delta, read from LDS, instead of from zero)
//     P(u) = exp2(S(u) kappa - LSE), dS(u) = P dP(u)   (VALU)
// and then dV^T += dO(u)^T P(u), dK^T += Q(u)^T dS(u) (16 MFMA, the transposed
// operands through the transposing LDS read).
constexpr int KV_STAT_FLOATS = 2 * 2 * DT_ROWS;              // [buffer][lse2 | -delta][64]

// -delta of the 32 query rows of a sub-tile as the initial dP^T accumulator: register r holds
// query row 8 (r/4) + 4h + r%4
__device__ inline void load_neg_delta(f32x16& dp, const float* neg_delta, int h) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const float4 x = *reinterpret_cast<const float4*>(neg_delta + 8 * g + 4 * h);
        dp[4 * g + 0] = x.x; dp[4 * g + 1] = x.y; dp[4 * g + 2] = x.z; dp[4 * g + 3] = x.w;
    }
}

// DP = 256 (head dimensions above 128): the Q and dO tiles come as two 128-column halves,
// DT_BYTES apart in LDS.  S and dP contract over both; a workgroup accumulates only ONE half of
// the columns of dK^T and dV^T (256 columns of both do not fit the register file beside K, V and
// the score tiles), so tr0 / tr1 arrive with that half's LDS offset added and the other half is
// another workgroup's, which computes S and dP again.
template <bool NEXT, bool MASK, int DP, bool PART>
__device__ inline void dkdv_step(f32x16& s_cur, f32x16& dp_cur, f32x16& s_next, f32x16& dp_next,
                                 f32x16 (&acck)[4], f32x16 (&accv)[4], const bf16x8 (&kf)[8 * halves_of(DP)],
                                 const bf16x8 (&vf)[8 * halves_of(DP)], float kappa, const uint32_t (&arow)[8],
                                 const uint32_t (&tr0)[4], const uint32_t (&tr1)[4], const char* q_next,
                                 const char* g_next, const char* q_cur, const char* g_cur,
                                 const float* stat_cur, const float* stat_next, int h, int mask_lim,
                                 int part_ks) {
    constexpr int NH = halves_of(DP), KS = ksteps_of(DP), MB = blocks_of(DP);      // per half
    bf16x8 qa[NH][8], ga[NH][8], qt[8], gt[8], pb[2], dsb[2];
    if (NEXT) load_neg_delta(dp_next, stat_next + DT_ROWS, h);
    auto fetch = [&](int i) {
        if (NEXT && i < KS) {
#pragma unroll
            for (int hh = 0; hh < NH; ++hh) {
                qa[hh][i] = dt_read_row(q_next + hh * DT_BYTES, arow[i]);
                ga[hh][i] = dt_read_row(g_next + hh * DT_BYTES, arow[i]);
            }
        }
    };
    auto fetch_t = [&](int i) {
        if (i % 4 < MB) {
            gt[i] = dt_read_tr(g_cur + (i / 4) * 16 * 256, tr0[i % 4], tr1[i % 4]);
            qt[i] = dt_read_tr(q_cur + (i / 4) * 16 * 256, tr0[i % 4], tr1[i % 4]);
        }
    };
    // LSE * log2(e) of this lane's query rows 8 (r/4) + 4h + r%4, two per slice
    float2 lv[8];
    auto fetch_stat = [&](int i) {
        lv[i] = *reinterpret_cast<const float2*>(stat_cur + 8 * (i / 2) + 4 * h + 2 * (i % 2));
    };
    // operands requested this many slices ahead of their use: row reads 2, transposed reads 3
    // (3 / 4 and 4 / 5 measured the same to 1 % at 32768-token shards: LDS latency is covered)
    constexpr int AHEAD = 2, TAHEAD = 3;
#pragma unroll
    for (int i = 0; i < AHEAD; ++i) {
        fetch(i);
        fetch_stat(i);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_barrier(0);          // slices stay in program order
        if (i + AHEAD < 8) {
            fetch(i + AHEAD);
            fetch_stat(i + AHEAD);
        }
        if (i >= 8 - TAHEAD) fetch_t(i - (8 - TAHEAD));     // the first transposed operands ahead of their use
        // One wavefront per SIMD: a second MFMA issued right behind the first stalls the
        // wavefront until the matrix pipeline is free again, and nothing else is issued
        // meanwhile.  So each MFMA is followed by one score's worth of VALU work, which runs
        // while it executes.
        auto score = [&](int r) {
            const float lr = (r & 1) ? lv[i].y : lv[i].x;
            float pr = __builtin_amdgcn_exp2f(fmaf(s_cur[r], kappa, -lr));
            if (MASK && 8 * (r / 4) + (r % 4) < mask_lim) pr = 0.f;
            pb[r / 8][r % 8] = (__bf16)pr;
            dsb[r / 8][r % 8] = (__bf16)(pr * dp_cur[r]);
        };
        if (NEXT && i < KS) {
#pragma unroll
            for (int hh = 0; hh < NH; ++hh) {
                const bf16x8 qx = PART ? zero_beyond_d(qa[hh][i], 8 * hh + i == part_ks) : qa[hh][i];
                const bf16x8 gx = PART ? zero_beyond_d(ga[hh][i], 8 * hh + i == part_ks) : ga[hh][i];
                score_mfma<DP, PART>(s_next, qx, kf[8 * hh + i], i == 0 && hh == 0);
                if (hh == 0) {
                    __builtin_amdgcn_sched_barrier(0);
                    score(2 * i);
                    __builtin_amdgcn_sched_barrier(0);
                }
                score_mfma<DP, PART>(dp_next, gx, vf[8 * hh + i], false);
            }
            score(2 * i + 1);
        } else {
            score(2 * i);
            score(2 * i + 1);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        if (i + TAHEAD < 8) fetch_t(i + TAHEAD);
        if (i % 4 < MB) {
            accv[i % 4] = mfma(gt[i], pb[i / 4], accv[i % 4]);
            acck[i % 4] = mfma(qt[i], dsb[i / 4], acck[i % 4]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// RAGGED (c not a multiple of 128): key rows beyond the shard are loaded from its last row and
// not stored; query rows beyond it come in as zero rows of Q and dO with LSE = +inf, so their
// P and dS are exactly zero.
template <bool TRI, bool RAGGED, int DP, bool PART>
__global__ void __launch_bounds__(256, 1)
bwd_dkdv_mfma_kernel(StepArgs p, int n_tiles) {
    constexpr int NH = halves_of(DP), KS = ksteps_of(DP), MB = blocks_of(DP);      // per half
    // one LDS object per tile buffer (two 128-column halves each when DP = 256)
    __shared__ __attribute__((aligned(1024))) char q_lds0[DT_BYTES * NH];
    __shared__ __attribute__((aligned(1024))) char q_lds1[DT_BYTES * NH];
    __shared__ __attribute__((aligned(1024))) char g_lds0[DT_BYTES * NH];
    __shared__ __attribute__((aligned(1024))) char g_lds1[DT_BYTES * NH];
    __shared__ __attribute__((aligned(16))) float stat[KV_STAT_FLOATS];

    const int tid = threadIdx.x, lane = tid & 63, n = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform, kept scalar
    int ktile, bhh;                               // triangular steps: low key tiles see most queries: first
    // one workgroup per (key tile, batch, key/value head, 128-column half of dK / dV); the query
    // head is this launch's member of the group that shares the key/value head
    decode_block<false>((int)blockIdx.x, n_tiles, p.B * p.H_kv * NH, ktile, bhh);
    const int bh = bhh / NH, ohalf = bhh - bh * NH;
    const int b = bh / p.H_kv, kvh = bh - b * p.H_kv;
    const int hd = kvh * (p.H / p.H_kv) + p.member;
    const int64_t base = b * p.stride_b + hd * p.stride_h;
    const int64_t kv_base = b * p.kv_stride_b + kvh * p.kv_stride_h;
    const int64_t sbase = b * p.stat_stride_b + hd * p.stat_stride_h;
    const int d = p.d;                                 // d <= DP, zero-padded to DP columns
    const int64_t ss = p.kv_stride_s;                  // elements between consecutive rows of K, V, dK, dV
    const int pitch = 2 * (int)p.stride_s;             // bytes between consecutive rows of Q and dO
    const int tile_pitch = DT_ROWS * pitch;            // bytes between 64-row tiles in global memory
    const dt_rsrc Qr = dt_make_rsrc((const __bf16*)p.q + base, p.c, pitch, d);
    const dt_rsrc Gr = dt_make_rsrc((const __bf16*)p.dout + base, p.c, pitch, d);
    const __bf16* K = (const __bf16*)p.k + kv_base;
    const __bf16* V = (const __bf16*)p.v + kv_base;
    const float* LSE = p.lse + sbase;
    const float* DEL = p.delta + sbase;
    float* DK = p.dk + kv_base;
    float* DV = p.dv + kv_base;

    const int k0 = ktile * BM, key_own = k0 + 32 * wave + n;
    const bool key_ok = !RAGGED || key_own < p.c;
    const int key = RAGGED ? min(key_own, p.c - 1) : key_own;     // the row this lane loads
    const int n_qt = RAGGED ? 2 * n_tiles : p.c / DT_ROWS;
    // query tiles holding at least one allowed pair (query a >= key + off): from tile k0 / 64
    // on; only its first four 32-query sub-tiles can cross the diagonal for some wavefront
    const int t_first_fine = TRI ? k0 / DT_ROWS : 0;
    int t_first = t_first_fine;
    if (TRI && p.skip_bq > 0)   // emulated coarse skipping: from the first skip_bq-tall query tile
                                // that shares an allowed pair with these keys' skip_bk-wide tile
        t_first = ((k0 / p.skip_bk * p.skip_bk + p.off) / p.skip_bq) * p.skip_bq / DT_ROWS;
    // sub-tile u: register r (query 32 u + 8 (r/4) + 4h + r%4) is allowed iff
    // 8 (r/4) + r%4 >= mask_base - 32 u
    const int mask_base = key_own + p.off - 4 * h;

    uint32_t arow[8], tr0[4], tr1[4], gl[NH][4];
    dt_row_addrs(arow, n, h);
    dt_tr_addrs(tr0, tr1, lane);
    if (NH > 1) {       // the transposed operands come from this workgroup's half of the columns
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) {
            tr0[mb] += ohalf * DT_BYTES;
            tr1[mb] += ohalf * DT_BYTES;
        }
    }
#pragma unroll
    for (int hh = 0; hh < NH; ++hh) dt_load_offsets(gl[hh], lane, wave, pitch, d, hh);
    auto load_tile = [&](dt_rsrc m, int tile_byte_offset, char* buf) {
#pragma unroll
        for (int hh = 0; hh < NH; ++hh) dt_load(m, tile_byte_offset, buf + hh * DT_BYTES, gl[hh], wave);
    };
    // t_first and n_qt are even (k0 and c are multiples of 128): tile t_first goes to buffer 0
    // and there are always at least two tiles
    load_tile(Qr, t_first * tile_pitch, q_lds0);
    load_tile(Gr, t_first * tile_pitch, g_lds0);
    load_tile(Qr, (t_first + 1) * tile_pitch, q_lds1);
    load_tile(Gr, (t_first + 1) * tile_pitch, g_lds1);
    // statistics of query tile t -> stat[(t & 1)][0 | 1][64]: threads 0..63 LSE * log2(e), 64..127
    // -delta.  The fetch is branch-free (wavefronts 2 and 3 re-read what 0 and 1 read and drop
    // it), so nothing waits for it before the store one trip later.
    const float* stat_src = ((tid & DT_ROWS) ? DEL : LSE) + (tid & (DT_ROWS - 1)) + t_first * DT_ROWS;
    const float stat_mul = (tid & DT_ROWS) ? -1.f : LOG2E;
    int stat_row = (tid & (DT_ROWS - 1)) + t_first * DT_ROWS;      // RAGGED only
    auto stat_fetch = [&]() -> float {          // tiles in order: the pointer walks with them
        float x;
        if (RAGGED) {       // rows beyond the shard: LSE = +inf, delta = 0 (still branch-free)
            x = stat_src[min(stat_row, p.c - 1) - stat_row];
            if (stat_row >= p.c) x = (tid & DT_ROWS) ? 0.f : INFINITY;
            stat_row += DT_ROWS;
        } else {
            x = *stat_src;
        }
        stat_src += DT_ROWS;
        return x;
    };
    auto stat_store = [&](int t, float x) {
        if (tid < 2 * DT_ROWS) stat[(t & 1) * 2 * DT_ROWS + tid] = x * stat_mul;
    };
    stat_store(t_first, stat_fetch());
    stat_store(t_first + 1, stat_fetch());

    bf16x8 kf[8 * NH], vf[8 * NH];
    load_b_frags<8 * NH>(kf, K + (int64_t)key * ss, h, d);
    load_b_frags<8 * NH>(vf, V + (int64_t)key * ss, h, d);
    const float kappa = p.scale * LOG2E;
    f32x16 acck[4], accv[4];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acck[mb][r] = accv[mb][r] = 0.f;

    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    // PART: k-step whose fragment, in this half-wave, is the chunk holding column d
    const int part_ks = (PART && ((d >> 3) & 1) == h) ? (d >> 4) : -1;
    f32x16 s_a, s_b, dp_a, dp_b;
    {   // prologue: S, dP of the first sub-tile
        const char* q0p = q_lds0;
        const char* g0p = g_lds0;
        load_neg_delta(dp_a, stat + DT_ROWS, h);          // tile t_first is in buffer 0
        // same order of the partial products as in dkdv_step (k-step outside, half inside): a
        // sub-tile's scores have the same bits whether this prologue or a step computes them
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int hh = 0; hh < NH; ++hh) {
                bf16x8 qx = dt_read_row(q0p + hh * DT_BYTES, arow[ks]), gx = dt_read_row(g0p + hh * DT_BYTES, arow[ks]);
                if (PART) {
                    qx = zero_beyond_d(qx, 8 * hh + ks == part_ks);
                    gx = zero_beyond_d(gx, 8 * hh + ks == part_ks);
                }
                score_mfma<DP, PART>(s_a, qx, kf[8 * hh + ks], ks == 0 && hh == 0);
                score_mfma<DP, PART>(dp_a, gx, vf[8 * hh + ks], false);
            }
        if (DP <= 128) mfma_results_to_valu(s_a, dp_a);
    }

    float rstat = 0.f;          // statistics of the tile after next, in flight
    // Trip t = iterations 2t (scores in *_a) and 2t+1 (scores in *_b) on query tile t.
    auto trip = [&](auto mask_c, auto par_c, auto last_c, int t) {
        constexpr bool MASK = decltype(mask_c)::value, last = decltype(last_c)::value;
        constexpr int PAR = decltype(par_c)::value;
        char* const q_cur = PAR ? q_lds1 : q_lds0;
        char* const g_cur = PAR ? g_lds1 : g_lds0;
        char* const q_nxt = PAR ? q_lds0 : q_lds1;
        char* const g_nxt = PAR ? g_lds0 : g_lds1;
        const float* st = stat + PAR * 2 * DT_ROWS;
        const float* st_nxt = stat + (1 - PAR) * 2 * DT_ROWS;       // statistics of tile t + 1
        dkdv_step<true, MASK, DP, PART>(s_a, dp_a, s_b, dp_b, acck, accv, kf, vf, kappa, arow, tr0, tr1,
                              q_cur + DT_BYTES / 2, g_cur + DT_BYTES / 2, q_cur, g_cur, st, st + 32, h,
                              mask_base - 64 * t, part_ks);
        if (!last) {
            if (t > t_first) stat_store(t + 1, rstat);     // fetched at the end of trip t-1
            __builtin_amdgcn_s_waitcnt(0);       // tile t+1, requested one iteration ago, has landed
            __syncthreads();
            dkdv_step<true, MASK, DP, PART>(s_b, dp_b, s_a, dp_a, acck, accv, kf, vf, kappa, arow, tr0, tr1, q_nxt,
                                  g_nxt, q_cur + DT_BYTES / 2, g_cur + DT_BYTES / 2, st + 32, st_nxt, h,
                                  mask_base - 64 * t - 32, part_ks);
            __syncthreads();                     // every wavefront is done with tile t
            if (t + 2 < n_qt) {
                load_tile(Qr, (t + 2) * tile_pitch, q_cur);
                load_tile(Gr, (t + 2) * tile_pitch, g_cur);
                rstat = stat_fetch();
            }
        } else {
            dkdv_step<false, MASK, DP, PART>(s_b, dp_b, s_a, dp_a, acck, accv, kf, vf, kappa, arow, tr0, tr1, q_nxt,
                                   g_nxt, q_cur + DT_BYTES / 2, g_cur + DT_BYTES / 2, st + 32, st_nxt, h,
                                   mask_base - 64 * t - 32, part_ks);
        }
    };
    using T = std::true_type;
    using F = std::false_type;
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    // t_first and n_qt are even (c and k0 are multiples of 128): trips come in pairs and the
    // last one has odd parity
    int t = t_first;
    if (TRI && DP > 128) {
        // One masked form for every trip (beyond the diagonal the mask limit is negative and
        // removes nothing).  With a second, unmasked copy of the loop this instantiation,
        // which is over the register budget, kept spilled registers live across its hot loop,
        // and every reload there waits for the tile loads in flight as well.
        for (; t + 2 < n_qt; t += 2) {
            trip(T{}, P0{}, F{}, t);
            trip(T{}, P1{}, F{}, t + 1);
        }
        trip(T{}, P0{}, F{}, t);
        trip(T{}, P1{}, T{}, t + 1);
    } else if (TRI) {
        // the trips up to the diagonal carry the element mask: the first two, more under
        // emulated coarse skipping
        for (; t < t_first_fine + 2; t += 2) {
            trip(T{}, P0{}, F{}, t);
            if (t + 2 < n_qt) trip(T{}, P1{}, F{}, t + 1);
            else trip(T{}, P1{}, T{}, t + 1);
        }
    }
    if (!(TRI && DP > 128)) {
        for (; t + 2 < n_qt; t += 2) {
            trip(F{}, P0{}, F{}, t);
            trip(F{}, P1{}, F{}, t + 1);
        }
        if (t < n_qt) {
            trip(F{}, P0{}, F{}, t);
            trip(F{}, P1{}, T{}, t + 1);
        }
    }

#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int col = 128 * ohalf + 32 * mb + 8 * g + 4 * h;
            if (col >= d || !key_ok) continue;            // padding columns, keys beyond the shard
            const int64_t o = (int64_t)key * ss + col;
            float4 x = *reinterpret_cast<float4*>(DV + o);
            x.x += accv[mb][4 * g + 0]; x.y += accv[mb][4 * g + 1];
            x.z += accv[mb][4 * g + 2]; x.w += accv[mb][4 * g + 3];
            *reinterpret_cast<float4*>(DV + o) = x;
            float4 y = *reinterpret_cast<float4*>(DK + o);
            y.x = fmaf(p.scale, acck[mb][4 * g + 0], y.x); y.y = fmaf(p.scale, acck[mb][4 * g + 1], y.y);
            y.z = fmaf(p.scale, acck[mb][4 * g + 2], y.z); y.w = fmaf(p.scale, acck[mb][4 * g + 3], y.w);
            *reinterpret_cast<float4*>(DK + o) = y;
        }
}

}  // namespace

bool bwd_mfma_supported(const StepArgs& a, int dtype) {
    // the tile loads address a shard through a buffer descriptor with 32-bit byte offsets:
    // the last row of its last (possibly partial) tile pair must end below 2^31 bytes from
    // its first
    const int64_t widest = a.stride_s > a.kv_stride_s ? a.stride_s : a.kv_stride_s;
    const int64_t rows = (int64_t)(a.c + BM - 1) / BM * BM;
    // one workgroup per (128-row tile, batch, head) in a 1-D grid
    if (rows / BM * a.B * a.H >= (int64_t(1) << 31)) return false;
    // head dimensions above 128 (two 128-column halves) in whole 16-byte chunks only
    if (a.d > 2 * D || (a.d > D && a.d % 8)) return false;
    return dtype == SA_BF16 && a.d % 4 == 0 && a.c >= BM &&
           rows * 2 * widest + 2 * a.d < (int64_t(1) << 31);
}

namespace {
template <int DP, bool PART>
hipError_t launch_bwd_variant(const StepArgs& a, hipStream_t st) {
    const int n_tiles = (a.c + BM - 1) / BM;
    const bool ragged = a.c % BM != 0;
    const dim3 grid_q((unsigned)n_tiles * a.B * a.H), block(256);
    const dim3 grid_kv((unsigned)n_tiles * a.B * a.H_kv * (DP > 128 ? 2 : 1));
    const bool full = a.kind == MASK_FULL;
    if (ragged) {
        if (full) hipLaunchKernelGGL((bwd_dq_mfma_kernel<true, true, DP, PART>), grid_q, block, 0, st, a, n_tiles);
        else hipLaunchKernelGGL((bwd_dq_mfma_kernel<true, false, DP, PART>), grid_q, block, 0, st, a, n_tiles);
    } else {
        if (full) hipLaunchKernelGGL((bwd_dq_mfma_kernel<false, true, DP, PART>), grid_q, block, 0, st, a, n_tiles);
        else hipLaunchKernelGGL((bwd_dq_mfma_kernel<false, false, DP, PART>), grid_q, block, 0, st, a, n_tiles);
    }
    hipError_t e = hipGetLastError();
    // dK, dV: the members of a group of query heads one after the other, each adding to the
    // shared head's accumulators in stream order (deterministic)
    StepArgs m = a;
    for (m.member = 0; m.member < a.H / a.H_kv && e == hipSuccess; ++m.member) {
        if (a.kind == MASK_TRI) {
            if (ragged) hipLaunchKernelGGL((bwd_dkdv_mfma_kernel<true, true, DP, PART>), grid_kv, block, 0, st, m, n_tiles);
            else hipLaunchKernelGGL((bwd_dkdv_mfma_kernel<true, false, DP, PART>), grid_kv, block, 0, st, m, n_tiles);
        } else {
            if (ragged) hipLaunchKernelGGL((bwd_dkdv_mfma_kernel<false, true, DP, PART>), grid_kv, block, 0, st, m, n_tiles);
            else hipLaunchKernelGGL((bwd_dkdv_mfma_kernel<false, false, DP, PART>), grid_kv, block, 0, st, m, n_tiles);
        }
        e = hipGetLastError();
    }
    return e;
}
}  // namespace

hipError_t launch_bwd_mfma(const StepArgs& a, hipStream_t st) {
    const bool part = a.d % 8 != 0;
    if (a.d > 128) return launch_bwd_variant<256, false>(a, st);
    if (a.d <= 64) return part ? launch_bwd_variant<64, true>(a, st) : launch_bwd_variant<64, false>(a, st);
    if (a.d <= 112) return part ? launch_bwd_variant<112, true>(a, st) : launch_bwd_variant<112, false>(a, st);
    return part ? launch_bwd_variant<128, true>(a, st) : launch_bwd_variant<128, false>(a, st);
}

}  // namespace sa
