// Forward ring step on the CDNA4 matrix cores (bf16 operands, fp32 accumulate),
// head dimension 128: AccumulateAttentionFragment of Algorithm 1 with the fused
// log-sum-exp merge, skipping every key tile that GetMask(j, k) masks entirely
// (Sec. 2.2.1) at a 64-key granularity per 32-query wavefront.
//
// Work decomposition.  A workgroup of 4 wavefronts owns 128 query rows; each
// wavefront owns 32 of them for the whole kernel.  Key/value tiles of 64 rows
// stream through LDS, double buffered (one barrier per tile).
//
// The scores are computed TRANSPOSED, S^T = K Q^T (A = key rows from LDS, B = the
// query rows, resident in registers), so that a lane holds 16 + 16 keys of ONE
// query: the row max / row sum of the online softmax are in-lane reductions
// plus a single exchange between the two half-waves, and the probabilities
// already sit in the B-operand layout of the second product O^T += V^T P^T.
// Its A operand, V^T, is read from the row-major V tile with the transposing
// LDS read, so both tiles are staged with plain 16-byte copies.
//
// Online softmax in base 2: kappa = scale * log2(e) is folded into the exponent,
// p = exp2(s * kappa - m).  The running state enters as (acc = O, m = LSE *
// log2(e), l = 1) and leaves as O = acc / l, LSE = (m + log2 l) * ln 2, which is
// the log-sum-exp merge of the step's partial result with the running one.
// Row sums are taken over the fp32 probabilities before they are rounded to
// bf16 for the second product (summing the rounded values costs 1e-3 of LSE
// accuracy on rows with few keys).
#include <hip/hip_bf16.h>

#include "mfma_tiles.h"
#include "sa_internal.h"

namespace sa {

namespace {

constexpr int BM = 128;        // query rows per workgroup
constexpr int BN = TR;         // key rows per tile
constexpr int D = TD;          // head dimension
constexpr int K_TILE = ROW_TILE;
constexpr int BUF = ROW_TILE + X_TILE;        // elements per pipeline stage: K rows, V rows

// Global -> registers and registers -> LDS stage for key tile kt.
__device__ inline void load_tile(u32x4 (&rk)[4], u32x4 (&rv)[4], const __bf16* __restrict__ K,
                                 const __bf16* __restrict__ V, int kt, int tid) {
    load_rows(rk, K + (int64_t)kt * BN * D, tid);
    load_rows(rv, V + (int64_t)kt * BN * D, tid);
}
__device__ inline void store_tile(const u32x4 (&rk)[4], const u32x4 (&rv)[4],
                                  __bf16* __restrict__ stage, int tid) {
    store_rows(rk, stage, tid);
    store_rows_x(rv, stage + K_TILE, tid);
}

constexpr float RESCALE_LOG2 = 8.f;

// max over the two half-waves (lanes n and n + 32 hold the same query)
__device__ inline float half_wave_max(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float half_wave_sum(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__global__ void __launch_bounds__(256, 2)
fwd_mfma_kernel(StepArgs p, int n_qtiles) {
    __shared__ __attribute__((aligned(16))) __bf16 lds[2 * BUF];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, h = lane >> 5;
    const bool tri = p.kind == MASK_TRI;
    int rank, bh;
    decode_block((int)blockIdx.x, n_qtiles, p.B * p.H, rank, bh);
    const int qt = tri ? n_qtiles - 1 - rank : rank;      // triangular steps: heaviest query tiles first
    const int b = bh / p.H, hd = bh - b * p.H;
    const int64_t base = b * p.stride_b + hd * p.stride_h;
    const __bf16* Q = (const __bf16*)p.q + base;
    const __bf16* K = (const __bf16*)p.k + base;
    const __bf16* V = (const __bf16*)p.v + base;
    float* O = p.o + base;
    float* L = p.lse + b * p.stat_stride_b + hd * p.stat_stride_h;

    const int q0 = qt * BM;
    const int a_lo = q0 + 32 * wave;          // first query row of this wavefront
    const int a = a_lo + n;                   // this lane's query row
    const int off = p.off;
    // key tiles holding at least one allowed pair: for the workgroup / for this wavefront
    const int n_kt = tri ? min(p.c / BN, (q0 + BM - 1 - off) / BN + 1) : p.c / BN;
    const int wave_last = tri ? (a_lo + 31 - off) / BN : n_kt - 1;

    // query rows as B operands: 8 k-steps of 16
    bf16x8 qf[8];
    load_b_frags(qf, Q + (int64_t)a * D, h);

    // running state -> accumulators
    const float kappa = p.scale * LOG2E;
    float m = L[a] * LOG2E;                   // -inf stays -inf
    float l = (h == 0) ? 1.f : 0.f;           // the two half-waves hold partial row sums
    f32x16 oacc[4];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const float4 x = *reinterpret_cast<const float4*>(O + (int64_t)a * D + 32 * mb + 8 * g + 4 * h);
            oacc[mb][4 * g + 0] = x.x; oacc[mb][4 * g + 1] = x.y;
            oacc[mb][4 * g + 2] = x.z; oacc[mb][4 * g + 3] = x.w;
        }

    u32x4 rk[4];
    u32x4 rv[4];
    const int tr_off = tr_lane_offset(lane);
    load_tile(rk, rv, K, V, 0, tid);
    store_tile(rk, rv, lds, tid);
    __syncthreads();

    for (int kt = 0; kt < n_kt; ++kt) {
        const __bf16* stage = lds + (kt & 1) * BUF;
        // prefetch the next tile into registers (the last iteration re-reads its own
        // tile into the idle stage, which keeps the loop free of branches)
        load_tile(rk, rv, K, V, min(kt + 1, n_kt - 1), tid);

        if (kt <= wave_last) {
            // S^T = K Q^T : two blocks of 32 keys x 32 queries.  All 16 A operands are
            // requested from LDS before the first MFMA so that the matrix pipe is fed
            // back to back instead of paying one LDS round trip per pair of MFMAs.
            f32x16 s[2];
            bf16x8 ka[2][8];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) ka[kb][ks] = read_a_rows(stage, kb * 32 + n, ks, h);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) s[kb] = mfma(ka[kb][ks], qf[ks], s[kb]);
            }
            // the first half of the V operands travels while the softmax runs
            bf16x8 va[4][4];
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int mb = 0; mb < 4; ++mb) va[g][mb] = read_a_tr(stage + K_TILE, tr_off, g, mb);
            __builtin_amdgcn_sched_barrier(0);
            // element mask, only on tiles crossing the diagonal: allowed iff key <= a - off
            if (tri && kt * BN + BN - 1 > a_lo - off) {
                const int lim = a - off - kt * BN - 4 * h;   // allowed iff 8*(r/4) + r%4 + 32 kb <= lim
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (32 * kb + 8 * (r / 4) + (r % 4) > lim) s[kb][r] = -INFINITY;
            }
            // online softmax, base 2, with a lazily updated reference m: the reference
            // moves only when a row's tile maximum exceeds it by more than 2^RESCALE_LOG2,
            // so p <= 2^RESCALE_LOG2 (harmless in bf16 / fp32) and the rescaling of l and
            // of the 64 accumulator registers is skipped on almost every tile.
            float mx = s[0][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[0][r]);
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[1][r]);
            mx = half_wave_max(mx);
            const float cand = mx * kappa;
            if (__builtin_amdgcn_ballot_w64(cand > m + RESCALE_LOG2) != 0) {     // wave-uniform
                const float m_new = fmaxf(m, cand);
                const float alpha = __builtin_amdgcn_exp2f(m - ((m_new == -INFINITY) ? 0.f : m_new));
                m = m_new;
                l *= alpha;
#pragma unroll
                for (int mb = 0; mb < 4; ++mb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[mb][r] *= alpha;
            }
            const float m_use = (m == -INFINITY) ? 0.f : m;       // row with no key so far
            bf16x8 pb[4];
            float rs0 = 0.f, rs1 = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    const float p0 = __builtin_amdgcn_exp2f(fmaf(s[kb][r], kappa, -m_use));
                    const float p1 = __builtin_amdgcn_exp2f(fmaf(s[kb][r + 1], kappa, -m_use));
                    rs0 += p0;                 // row sums in fp32, before the rounding to bf16
                    rs1 += p1;
                    pb[2 * kb + r / 8][r % 8] = (__bf16)p0;
                    pb[2 * kb + r / 8][r % 8 + 1] = (__bf16)p1;
                }
            l += rs0 + rs1;
            // O^T += V^T P^T : 4 blocks of 32 d-rows, 4 k-steps of 16 keys
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int g = 2; g < 4; ++g)
#pragma unroll
                for (int mb = 0; mb < 4; ++mb) va[g][mb] = read_a_tr(stage + K_TILE, tr_off, g, mb);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int mb = 0; mb < 4; ++mb) oacc[mb] = mfma(va[g][mb], pb[g], oacc[mb]);
        }

        store_tile(rk, rv, lds + ((kt + 1) & 1) * BUF, tid);
        __syncthreads();
    }

    // epilogue: normalise, store the merged state
    const float l_tot = half_wave_sum(l);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            float4 x;
            x.x = oacc[mb][4 * g + 0] * inv; x.y = oacc[mb][4 * g + 1] * inv;
            x.z = oacc[mb][4 * g + 2] * inv; x.w = oacc[mb][4 * g + 3] * inv;
            *reinterpret_cast<float4*>(O + (int64_t)a * D + 32 * mb + 8 * g + 4 * h) = x;
        }
    if (h == 0) L[a] = (m + __builtin_amdgcn_logf(l_tot)) * LN2;
}

}  // namespace

bool fwd_mfma_supported(const StepArgs& a, int dtype) {
    return dtype == SA_BF16 && a.d == D && a.c % BM == 0;
}

hipError_t launch_fwd_mfma(const StepArgs& a, hipStream_t st) {
    const int n_qtiles = a.c / BM;
    hipLaunchKernelGGL(fwd_mfma_kernel, dim3(n_qtiles * a.B * a.H), dim3(256), 0, st, a, n_qtiles);
    return hipGetLastError();
}

}  // namespace sa
