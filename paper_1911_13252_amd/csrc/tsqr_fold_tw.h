// One fold step of the tall-skinny QR, [R; B] -> [R'; 0] for a block B of BR rows in LDS (the paper's section
// "Computing beta": H = QR applied to [H | T] a block of rows at a time), for widths of more than one panel,
// with the triangular factor T of the compact-WY form built by a fifth wave while the Householder chain of
// the panel runs.
//
// Waves 0-3 run the chain and the trailing update exactly as fold_block() does.  Wave 4 shares a SIMD with
// wave 0 and turns the Gram entries v_j . v_k and the tau values that the chain publishes in LDS into the
// columns of T, two steps behind the chain, so T is complete when the chain ends instead of costing a serial
// back substitution of 32 steps afterwards (13 % of a block at 544 columns).  The float32 matrix
// instruction occupies the vector ALU of its SIMD while it runs (measured: vector work of another wave on
// that SIMD makes no progress meanwhile), so the trailing update itself cannot be overlapped with the chain
// by giving it waves of its own; only the chain's idle issue slots can be filled, which is what wave 4 does.
#pragma once

#include <hip/hip_runtime.h>

#include "tsqr_fold.h"

namespace elm {
namespace fold {

constexpr int kThreadsTW = 320;
constexpr int kTsTW = 36;     // row stride of the T factor in LDS: 16-byte aligned rows

// LDS floats: the block (row stride np + 1), the Gram rows of the panel, its T factor, cross-wave partial
// sums, the tau values
__host__ __device__ inline size_t lds_floats_tw(int np, int br) {
    return (size_t)((br * (np + 1) + 3) & ~3) + 32 * kGs + 32 * kTsTW + 2 * 4 * 32 + 32;
}

// R: this work-group's np x np upper-triangular factor (global memory); lds: the block at lds[0 .. BR*ldb)
// followed by the scratch areas (lds_floats_tw); p0: first panel that can be non-zero in the block; nreal:
// columns of the matrix proper (the last panel takes no steps for the zero padding beyond them).
// All 320 threads call it; it ends with a barrier.
template <int BR>
__device__ __forceinline__ void fold_block_tw(float* __restrict__ R, float* lds, int np, int ldb, int p0, int nreal) {
    constexpr int RPT = BR / 8;      // rows of a panel column held by one lane
    constexpr int MT = BR / 32;      // 32-row accumulator tiles per block
    // Two waves share a SIMD, so a wave has 256 registers.  The trailing update of a 64-row block keeps the
    // panel's reflectors as operands of both of its products in registers (64) next to T (16); a 128-row block
    // would need 128 + 16, so it keeps those of the first product (64) and reads those of the last from LDS.
    constexpr bool kCacheV3 = BR <= 64;
    const int NP = np / kNB;
    float* Bs = lds;                           // [BR][ldb]
    float* Gt = Bs + ((BR * ldb + 3) & ~3);    // [32][36]: row k = v_j . v_k for the finished reflectors j < k
    float* Ts = Gt + 32 * kGs;                 // [32][36] compact-WY T
    float* red = Ts + 32 * kTsTW;              // [2][32][4] cross-wave partial sums
    float* taus = red + 2 * 4 * 32;            // [32]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5;

    if (wave < 4) {
        const int j = tid & 31;          // panel column of this lane
        const int g = tid >> 5;          // row group: rows RPT*g .. RPT*g + RPT-1
        float rdv[32];
#pragma unroll
        for (int k = 0; k < 32; ++k) rdv[k] = R[(size_t)(p0 * kNB + k) * np + p0 * kNB + j];

        for (int p = p0; p < NP; ++p) {
            const int kp = p * kNB;
            // ================= panel factorisation (see fold_block) =================
            float pv[RPT];
#pragma unroll
            for (int i = 0; i < RPT; ++i) pv[i] = Bs[(RPT * g + i) * ldb + kp + j];
            panel_chain<RPT, kChainPublish | kChainGramByStep>(pv, rdv, nreal - kp, red, Gt, taus, wave, j, g, half);
#pragma unroll
            for (int i = 0; i < RPT; ++i) Bs[(RPT * g + i) * ldb + kp + j] = pv[i];
            if (g == 0) {
#pragma unroll
                for (int k = 0; k < 32; ++k)
                    if (k <= j) R[(size_t)(kp + k) * np + kp + j] = rdv[k];
            }
            __syncthreads();                    // E1: reflectors in the block; tau and Gram rows complete
            if (p + 1 == NP) break;
            // next panel's diagonal block of R: in flight during the trailing update, which never touches
            // the rows of R that the next panel factors
#pragma unroll
            for (int k = 0; k < 32; ++k) rdv[k] = R[(size_t)(kp + kNB + k) * np + kp + kNB + j];
            __syncthreads();                    // E2: wave 4 has stored the last column of T

            // ================= trailing update on the matrix instruction =================
            {
                const int c = lane & 31;
                float va1[BR / 2], va3[kCacheV3 ? MT : 1][16], tq[16];
#pragma unroll
                for (int s = 0; s < BR / 2; ++s) va1[s] = Bs[(2 * s + half) * ldb + kp + c];
                if (kCacheV3) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int q = 0; q < 16; ++q)
                            va3[kCacheV3 ? mt : 0][q] = Bs[(mt * 32 + c) * ldb + kp + rho(q) + 4 * half];
                }
#pragma unroll
                for (int q = 0; q < 16; ++q) tq[q] = Ts[(rho(q) + 4 * half) * kTsTW + c];

                int ct = p + 1 + wave;
                floatx16 crv;
                if (ct < NP) {
#pragma unroll
                    for (int q = 0; q < 16; ++q)
                        crv[q] = R[(size_t)(kp + rho(q) + 4 * half) * np + ct * kNB + c];
                }
                for (; ct < NP; ct += 4) {
                    const int cc = ct * kNB + c;
                    floatx16 acc = crv, acc2, crn;
                    if (ct + 4 < NP) {
#pragma unroll
                        for (int q = 0; q < 16; ++q)
                            crn[q] = R[(size_t)(kp + rho(q) + 4 * half) * np + cc + 4 * kNB];
                    }
#pragma unroll
                    for (int q = 0; q < 16; ++q) acc2[q] = 0.0f;
#pragma unroll
                    for (int s = 0; s < BR / 2; ++s)
                        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(va1[s], Bs[(2 * s + half) * ldb + cc], acc, 0, 0, 0);
#pragma unroll
                    for (int q = 0; q < 16; ++q)
                        acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(tq[q], acc[q], acc2, 0, 0, 0);
#pragma unroll
                    for (int q = 0; q < 16; ++q) {
                        R[(size_t)(kp + rho(q) + 4 * half) * np + cc] = crv[q] - acc2[q];
                        acc2[q] = -acc2[q];
                    }
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        floatx16 cb;
#pragma unroll
                        for (int q = 0; q < 16; ++q)
                            cb[q] = Bs[(mt * 32 + rho(q) + 4 * half) * ldb + cc];
#pragma unroll
                        for (int q = 0; q < 16; ++q) {
                            const float a = kCacheV3 ? va3[kCacheV3 ? mt : 0][q]
                                                     : Bs[(mt * 32 + c) * ldb + kp + rho(q) + 4 * half];
                            cb = __builtin_amdgcn_mfma_f32_32x32x2f32(a, acc2[q], cb, 0, 0, 0);
                        }
#pragma unroll
                        for (int q = 0; q < 16; ++q)
                            Bs[(mt * 32 + rho(q) + 4 * half) * ldb + cc] = cb[q];
                    }
                    crv = crn;
                }
            }
            __syncthreads();                    // E3: the block is ready for the next panel
        }
    } else {
        // ================= wave 4: the T factor, two steps behind the chain =================
        const bool t_lane = lane < 32;                      // lane j owns row j of T
        // stale Gram rows are multiplied by the zeros of unfinished T columns: they must be finite
        for (int idx = lane; idx < 32 * kGs; idx += 64) Gt[idx] = 0.0f;
        // Column kk: T[j][kk] = -tau_kk sum_l T[j][l] (v_l . v_kk) for j < kk, tau_kk on the diagonal (columns
        // right of kk are still zero, rows are zero left of the diagonal)
        auto t_column = [&](int kk) {
            float sum = 0.0f;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const float4 tv = *reinterpret_cast<const float4*>(Ts + lane * kTsTW + 4 * q);
                const float4 gv = *reinterpret_cast<const float4*>(Gt + kk * kGs + 4 * q);
                sum = fmaf(tv.x, gv.x, sum);
                sum = fmaf(tv.y, gv.y, sum);
                sum = fmaf(tv.z, gv.z, sum);
                sum = fmaf(tv.w, gv.w, sum);
            }
            const float tk = taus[kk];
            if (lane <= kk) Ts[lane * kTsTW + kk] = (lane == kk) ? tk : -tk * sum;
        };
        for (int p = p0; p < NP; ++p) {
            if (t_lane) {
#pragma unroll
                for (int q = 0; q < kTsTW / 4; ++q)
                    *reinterpret_cast<float4*>(Ts + lane * kTsTW + 4 * q) = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            }
            const int steps = min(32, nreal - p * kNB);     // one barrier per step of the chain
            for (int k = 0; k < steps; ++k) {
                // the chain writes tau and the Gram row of its step k-2 between the barriers of steps k-2 and
                // k-1: complete once this wave has passed the barrier of step k-1
                if (t_lane && k >= 2) t_column(k - 2);
                lds_barrier();
            }
            if (t_lane) t_column(30);
            __syncthreads();                    // E1
            if (p + 1 == NP) break;
            if (t_lane) t_column(31);
            __syncthreads();                    // E2
            __syncthreads();                    // E3
        }
    }
    __syncthreads();
}

}  // namespace fold
}  // namespace elm
