// Backward ring step on the CDNA4 matrix cores (bf16 operands, fp32 accumulate),
// head dimension 128.  The paper describes no backward pass; this is the
// analytic gradient of causal attention (Sec. 2.1) restricted to the pairs that
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
// apply the element mask only on tiles that cross the diagonal.
#include <hip/hip_bf16.h>

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
constexpr int DQ_K = 0;                       // K rows
constexpr int DQ_KT = ROW_TILE;               // K transposed
constexpr int DQ_V = ROW_TILE + TRN_TILE;     // V rows
constexpr int DQ_LDS = 2 * ROW_TILE + TRN_TILE;

__global__ void __launch_bounds__(256, 2)
bwd_dq_mfma_kernel(StepArgs p, int n_tiles) {
    __shared__ __attribute__((aligned(16))) __bf16 lds[DQ_LDS];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, h = lane >> 5;
    const bool tri = p.kind == MASK_TRI;
    int rank, bh;
    decode_block((int)blockIdx.x, n_tiles, p.B * p.H, rank, bh);
    const int qt = tri ? n_tiles - 1 - rank : rank;      // heaviest query tiles first
    const int b = bh / p.H, hd = bh - b * p.H;
    const int64_t base = b * p.stride_b + hd * p.stride_h;
    const int64_t sbase = b * p.stat_stride_b + hd * p.stat_stride_h;
    const __bf16* Q = (const __bf16*)p.q + base;
    const __bf16* K = (const __bf16*)p.k + base;
    const __bf16* V = (const __bf16*)p.v + base;
    const __bf16* G = (const __bf16*)p.dout + base;
    float* DQ = p.dq + base;

    const int q0 = qt * BM, a_lo = q0 + 32 * wave, a = a_lo + n, off = p.off;
    const int n_kt = tri ? min(p.c / BN, (q0 + BM - 1 - off) / BN + 1) : p.c / BN;
    const int wave_last = tri ? (a_lo + 31 - off) / BN : n_kt - 1;

    bf16x8 qf[8], gf[8];
    load_b_frags(qf, Q + (int64_t)a * D, h);
    load_b_frags(gf, G + (int64_t)a * D, h);
    const float kappa = p.scale * LOG2E;
    const float lse2 = p.lse[sbase + a] * LOG2E;
    const float delta = p.delta[sbase + a];

    f32x16 acc[4];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mb][r] = 0.f;

    u32x4 rk[4], rvr[4];
    uint32_t rq[16];
    load_rows(rk, K, tid);
    load_quads(rq, K, tid);
    load_rows(rvr, V, tid);

    for (int kt = 0; kt < n_kt; ++kt) {
        store_rows(rk, lds + DQ_K, tid);
        store_transposed(rq, lds + DQ_KT, tid);
        store_rows(rvr, lds + DQ_V, tid);
        __syncthreads();
        {   // prefetch the next tile (the last iteration re-reads its own)
            const int64_t nxt = (int64_t)min(kt + 1, n_kt - 1) * BN * D;
            load_rows(rk, K + nxt, tid);
            load_quads(rq, K + nxt, tid);
            load_rows(rvr, V + nxt, tid);
        }
        if (kt <= wave_last) {
            const bool need_mask = tri && kt * BN + BN - 1 > a_lo - off;
            const int lim = a - off - kt * BN - 4 * h;     // allowed iff 32 kb + 8 (r/4) + r%4 <= lim
            bf16x8 dsb[4];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                f32x16 s, dp;
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    s = mfma(read_a_rows(lds + DQ_K, kb * 32 + n, ks, h), qf[ks], s);
                    dp = mfma(read_a_rows(lds + DQ_V, kb * 32 + n, ks, h), gf[ks], dp);
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float pr = __builtin_amdgcn_exp2f(fmaf(s[r], kappa, -lse2));
                    if (need_mask && 32 * kb + 8 * (r / 4) + (r % 4) > lim) pr = 0.f;
                    s[r] = pr * (dp[r] - delta);
                }
                dsb[2 * kb] = pack8(s, 0);
                dsb[2 * kb + 1] = pack8(s, 8);
            }
            // dQ^T += K^T dS^T
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int mb = 0; mb < 4; ++mb)
                    acc[mb] = mfma(read_a_trn(lds + DQ_KT, 32 * mb + n, g, h), dsb[g], acc[mb]);
        }
        __syncthreads();
    }

#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            float4* dst = reinterpret_cast<float4*>(DQ + (int64_t)a * D + 32 * mb + 8 * g + 4 * h);
            float4 x = *dst;
            x.x = fmaf(p.scale, acc[mb][4 * g + 0], x.x); x.y = fmaf(p.scale, acc[mb][4 * g + 1], x.y);
            x.z = fmaf(p.scale, acc[mb][4 * g + 2], x.z); x.w = fmaf(p.scale, acc[mb][4 * g + 3], x.w);
            *dst = x;
        }
}

// ------------------------------------------------------------- dK/dV kernel
constexpr int KV_Q = 0;                            // Q rows
constexpr int KV_QT = ROW_TILE;                    // Q transposed
constexpr int KV_G = ROW_TILE + TRN_TILE;          // dO rows
constexpr int KV_GT = 2 * ROW_TILE + TRN_TILE;     // dO transposed
constexpr int KV_ELEMS = 2 * ROW_TILE + 2 * TRN_TILE;

__global__ void __launch_bounds__(256, 1)
bwd_dkdv_mfma_kernel(StepArgs p, int n_tiles) {
    __shared__ __attribute__((aligned(16))) __bf16 lds[KV_ELEMS];
    __shared__ __attribute__((aligned(16))) float stat[2][BN];     // LSE * log2(e), delta of the query tile

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, n = lane & 31, h = lane >> 5;
    const bool tri = p.kind == MASK_TRI;
    int ktile, bh;                                // triangular steps: low key tiles see most queries: first
    decode_block((int)blockIdx.x, n_tiles, p.B * p.H, ktile, bh);
    const int b = bh / p.H, hd = bh - b * p.H;
    const int64_t base = b * p.stride_b + hd * p.stride_h;
    const int64_t sbase = b * p.stat_stride_b + hd * p.stat_stride_h;
    const __bf16* Q = (const __bf16*)p.q + base;
    const __bf16* K = (const __bf16*)p.k + base;
    const __bf16* V = (const __bf16*)p.v + base;
    const __bf16* G = (const __bf16*)p.dout + base;
    const float* LSE = p.lse + sbase;
    const float* DEL = p.delta + sbase;
    float* DK = p.dk + base;
    float* DV = p.dv + base;

    const int k0 = ktile * BM, b_lo = k0 + 32 * wave, key = b_lo + n, off = p.off;
    const int n_qt = p.c / BN;
    // query tiles holding at least one allowed pair: query a >= key + off
    const int qt_first = tri ? min(n_qt, (k0 + off) / BN) : 0;
    const int wave_first = tri ? (b_lo + off) / BN : 0;     // tiles before it are empty for this wavefront

    bf16x8 kf[8], vf[8];
    load_b_frags(kf, K + (int64_t)key * D, h);
    load_b_frags(vf, V + (int64_t)key * D, h);
    const float kappa = p.scale * LOG2E;

    f32x16 acck[4], accv[4];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acck[mb][r] = accv[mb][r] = 0.f;

    if (qt_first < n_qt) {
        u32x4 rqr[4], rgr[4];
        uint32_t rqq[16], rgq[16];
        float rstat = 0.f;
        auto prefetch = [&](int qt) {
            const int64_t o = (int64_t)qt * BN * D;
            load_rows(rqr, Q + o, tid);
            load_quads(rqq, Q + o, tid);
            load_rows(rgr, G + o, tid);
            load_quads(rgq, G + o, tid);
            if (tid < BN) rstat = LSE[qt * BN + tid] * LOG2E;
            else if (tid < 2 * BN) rstat = DEL[qt * BN + tid - BN];
        };
        prefetch(qt_first);
        for (int qt = qt_first; qt < n_qt; ++qt) {
            store_rows(rqr, lds + KV_Q, tid);
            store_transposed(rqq, lds + KV_QT, tid);
            store_rows(rgr, lds + KV_G, tid);
            store_transposed(rgq, lds + KV_GT, tid);
            if (tid < 2 * BN) stat[tid >> 6][tid & 63] = rstat;
            __syncthreads();
            prefetch(min(qt + 1, n_qt - 1));
            if (qt >= wave_first) {
                const int a0 = qt * BN;
                // allowed iff key <= a - off; a = a0 + 32 qb + 8 (r/4) + 4h + r%4
                const bool need_mask = tri && a0 < b_lo + 31 + off;
                const int lim = key + off - a0 - 4 * h;     // allowed iff 32 qb + 8 (r/4) + r%4 >= lim
                bf16x8 pb[4], dsb[4];
#pragma unroll
                for (int qb = 0; qb < 2; ++qb) {
                    f32x16 s, dp;
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[r] = dp[r] = 0.f;
#pragma unroll
                    for (int ks = 0; ks < 8; ++ks) {
                        s = mfma(read_a_rows(lds + KV_Q, qb * 32 + n, ks, h), kf[ks], s);
                        dp = mfma(read_a_rows(lds + KV_G, qb * 32 + n, ks, h), vf[ks], dp);
                    }
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const float4 l4 = *reinterpret_cast<const float4*>(&stat[0][32 * qb + 8 * g + 4 * h]);
                        const float4 d4 = *reinterpret_cast<const float4*>(&stat[1][32 * qb + 8 * g + 4 * h]);
                        const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
                        const float dv[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int r = 4 * g + e;
                            float pr = __builtin_amdgcn_exp2f(fmaf(s[r], kappa, -lv[e]));
                            if (need_mask && 32 * qb + 8 * g + e < lim) pr = 0.f;
                            s[r] = pr;
                            dp[r] = pr * (dp[r] - dv[e]);
                        }
                    }
                    pb[2 * qb] = pack8(s, 0);
                    pb[2 * qb + 1] = pack8(s, 8);
                    dsb[2 * qb] = pack8(dp, 0);
                    dsb[2 * qb + 1] = pack8(dp, 8);
                }
                // dV^T += dO^T P ; dK^T += Q^T dS
#pragma unroll
                for (int g = 0; g < 4; ++g)
#pragma unroll
                    for (int mb = 0; mb < 4; ++mb) {
                        accv[mb] = mfma(read_a_trn(lds + KV_GT, 32 * mb + n, g, h), pb[g], accv[mb]);
                        acck[mb] = mfma(read_a_trn(lds + KV_QT, 32 * mb + n, g, h), dsb[g], acck[mb]);
                    }
            }
            __syncthreads();
        }
    }

#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int64_t o = (int64_t)key * D + 32 * mb + 8 * g + 4 * h;
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
    return dtype == SA_BF16 && a.d == D && a.c % BM == 0;
}

hipError_t launch_bwd_mfma(const StepArgs& a, hipStream_t st) {
    const int n_tiles = a.c / BM;
    hipLaunchKernelGGL(bwd_dq_mfma_kernel, dim3(n_tiles * a.B * a.H), dim3(256), 0, st, a, n_tiles);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(bwd_dkdv_mfma_kernel, dim3(n_tiles * a.B * a.H), dim3(256), 0, st, a, n_tiles);
    return hipGetLastError();
}

}  // namespace sa
