// One fold step of the tall-skinny QR: [R; B] -> [R'; 0] for a block B of BR rows that already sits in
// LDS (the paper's section "Computing beta": H = QR applied to [H | T] a block of rows at a time).
// Shared by the TSQR kernel, which loads the blocks from memory, and by the fused stage-1 kernel, whose
// blocks are the hidden-matrix tiles it has just computed.
#pragma once

#include <hip/hip_runtime.h>

namespace elm {
namespace fold {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kNB = 32;         // panel width = MFMA tile width

// value of x in lane `src` (compile-time constant), delivered through a scalar register
__device__ __forceinline__ float lane_bcast(float x, int src) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), src));
}

// value of x in the lane 32 positions away (the other half of the wavefront), without an LDS round trip
__device__ __forceinline__ float other_half(float x, int half) {
    const unsigned u = __builtin_bit_cast(unsigned, x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __builtin_bit_cast(float, half ? r[0] : r[1]);
}

// row index inside a 32x32 accumulator tile held in register q by a lane of half h
__device__ __forceinline__ int rho(int q) { return 8 * (q >> 2) + (q & 3); }

constexpr int kTs = 33;      // row stride of the T factor in LDS
constexpr int kGs = 36;      // row stride of the Gram matrix in LDS (16-byte aligned rows)

// LDS floats a fold of BR-row blocks of padded width np needs: the block (row stride np + 1), the Gram
// matrix of the panel's reflectors, the T factor, cross-wave partial sums, the panel's tau values
__host__ __device__ inline size_t lds_floats(int np, int br) {
    return (size_t)((br * (np + 1) + 3) & ~3) + 32 * kGs + 32 * kTs + 2 * 4 * 32 + 32;
}

// Barrier between the column steps of a chain: orders LDS traffic only (nothing in global memory changes hands
// inside a chain), so loads from global memory stay in flight across it
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

enum ChainFlags {
    kChainPublish = 1,      // tau and the Gram entries of the reflectors go to LDS (for the T factor)
    kChainGramByStep = 2,   // Gram entry (j, k) is stored at [k][j] (a row per step) instead of [j][k]
};

// The Householder chain of one 32-column panel of [R; B]: `steps` column steps (32, or fewer when the rest of
// the panel is zero padding), run by the 256 threads of four waves.
//   pv[RPT]   lane (j, g) holds rows RPT g .. RPT g + RPT-1 of panel column j of the block (j = thread % 32,
//             g = thread / 32); replaced by the reflectors v (below the implicit unit entry in R)
//   rdv[32]   column j of the panel's diagonal block of R (every g holds a copy); replaced by the new one
//   red       [2][32][4] floats of LDS for the cross-wave sums;  G [32][kGs], taus [32]: see ChainFlags
// One reduction per step gives the norm of column k and its dot products with every column.  The two
// half-waves of a wave hold different rows, so column k arrives as two scalars per register (lanes k and
// 32 + k); every lane uses both as scalar operands: the dot product is taken with each and the own half's sum
// selected once, and the update adds the other half's term with a zero coefficient.  A finished column keeps
// its unscaled entries x (its coefficient is zero from its own step on) and is scaled to the reflector
// v = x f once, after the last step, by an exactly rounded product (the stored reflector must not lose
// digits); the Gram entries carry both factors.  Columns whose remaining mass is below 1e-30 get the identity
// reflector: they only arise as rounding residue when a block has fewer rows than columns, and the hardware
// square root and reciprocal (1 ulp: a reflector built from them is orthogonal to float32 rounding) flush
// denormals; what those make of such a column is dropped by selects, not branched around.
template <int RPT, int FLAGS>
__device__ __forceinline__ void panel_chain(float (&pv)[RPT], float (&rdv)[32], int steps, float* red, float* G,
                                            float* taus, int wave, int j, int g, int half) {
    float f_own = 0.0f;
    auto step = [&](const int k) {
        float lo[RPT], hi[RPT];
        float s_lo = 0.0f, s_hi = 0.0f;
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
            lo[i] = lane_bcast(pv[i], k);
            hi[i] = lane_bcast(pv[i], 32 + k);
            s_lo = fmaf(lo[i], pv[i], s_lo);
            s_hi = fmaf(hi[i], pv[i], s_hi);
        }
        float s = half ? s_hi : s_lo;
        s += other_half(s, half);
        float* rb = red + (k & 1) * 128;            // [32 columns][4 waves]
        if (half == 0) rb[4 * j + wave] = s;
        const float x0 = lane_bcast(rdv[k], k);     // every copy is identical
        lds_barrier();
        const float4 pj = *reinterpret_cast<const float4*>(rb + 4 * j);
        const float4 pk = *reinterpret_cast<const float4*>(rb + 4 * k);
        const float sj = (pj.x + pj.y) + (pj.z + pj.w);
        const float sigma = (pk.x + pk.y) + (pk.z + pk.w);
        const float nrm2 = fmaf(x0, x0, sigma);
        const bool live = sigma > 0.0f && nrm2 > 1e-30f;
        const float nrm = __builtin_amdgcn_sqrtf(nrm2);
        const float alpha_l = (x0 >= 0.0f) ? -nrm : nrm;
        const float alpha = live ? alpha_l : x0;
        const float tau = live ? (alpha_l - x0) * __builtin_amdgcn_rcpf(alpha_l) : 0.0f;
        const float f = live ? __builtin_amdgcn_rcpf(x0 - alpha_l) : 0.0f;
        // lanes j > k apply the reflector, lane j == k stores alpha
        const float w = (j > k) ? tau * fmaf(f, sj, rdv[k]) : 0.0f;
        rdv[k] = (j == k) ? alpha : rdv[k] - w;
        const float cf = -(f * w);                  // zero for the columns at and left of k
        const float cf_lo = half ? 0.0f : cf, cf_hi = half ? cf : 0.0f;
#pragma unroll
        for (int i = 0; i < RPT; ++i) pv[i] = fmaf(hi[i], cf_hi, fmaf(lo[i], cf_lo, pv[i]));
        if ((FLAGS & kChainPublish) && g == 0) {
            if (j == k) taus[k] = tau;
            // v_j . v_k for the finished reflector j
            if (j < k) G[(FLAGS & kChainGramByStep) ? k * kGs + j : j * kGs + k] = (f * f_own) * sj;
        }
        f_own = (j == k) ? f : f_own;
    };
    // (two copies of the unrolled steps: a per-step test in the common case would end every step's basic block
    // and keep the compiler from overlapping neighbouring steps)
    if (steps >= 32) {
#pragma unroll
        for (int k = 0; k < 32; ++k) step(k);
    } else {
#pragma unroll
        for (int k = 0; k < 32; ++k)
            if (k < steps) step(k);
    }
#pragma unroll
    for (int i = 0; i < RPT; ++i) pv[i] *= f_own;
}

// The triangular factor T of the compact-WY form Q = I - V T V^T of one panel, from
// T^-1 = diag(1/tau) + striu(V^T V): column j of T by back substitution, one lane per column (32 lanes of one
// wave call it with their column j); t[l] = 0 for l > j makes every lane run the same instruction stream.
// Gs: [32][kGs], entry (i, l) = v_i . v_l for i < l; taus: [32]; Ts: [32][kTs], written.
__device__ __forceinline__ void t_factor_backsubst(const float* Gs, const float* taus, float* Ts, int j) {
    float t[32], tv[32];
#pragma unroll
    for (int l = 0; l < 32; ++l) {
        tv[l] = taus[l];
        t[l] = (l == j) ? tv[l] : 0.0f;
    }
    // Row i of the Gram matrix is read in 16-byte pieces starting at the multiple of four at
    // or below i + 1 (the entries at or left of the diagonal in the first piece are skipped);
    // row i - 1 is requested before row i is used, so the LDS latency hides behind the FMAs.
    float4 gq[2][8];
#pragma unroll
    for (int c = 7; c < 8; ++c) gq[0][c] = *reinterpret_cast<const float4*>(Gs + 30 * kGs + 4 * c);
#pragma unroll
    for (int i = 30; i >= 0; --i) {
        const int cur = (30 - i) & 1;
        if (i > 0) {
#pragma unroll
            for (int c = (i >> 2); c < 8; ++c)        // chunks of row i - 1: from i / 4
                gq[cur ^ 1][c] = *reinterpret_cast<const float4*>(Gs + (i - 1) * kGs + 4 * c);
        }
        __builtin_amdgcn_sched_barrier(0);
        float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;      // four short dependency chains
#pragma unroll
        for (int c = ((i + 1) >> 2); c < 8; ++c) {
            const float4 gv = gq[cur][c];
            const int l4 = 4 * c;
            if (l4 + 0 > i) s0 = fmaf(gv.x, t[l4 + 0], s0);
            if (l4 + 1 > i) s1 = fmaf(gv.y, t[l4 + 1], s1);
            if (l4 + 2 > i) s2 = fmaf(gv.z, t[l4 + 2], s2);
            if (l4 + 3 > i) s3 = fmaf(gv.w, t[l4 + 3], s3);
        }
        t[i] = (i < j) ? -tv[i] * ((s0 + s1) + (s2 + s3)) : t[i];
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int i = 0; i < 32; ++i) Ts[i * kTs + j] = t[i];
}

// R: this work-group's np x np upper-triangular factor (global memory); lds: the block at lds[0 .. BR*ldb)
// followed by the scratch areas; p0: first panel that can be non-zero in the block (columns left of it
// are zero); nreal: columns of the matrix proper (the rest of np is zero padding, for which the last panel
// takes no steps).  All 256 threads call it; it ends with a barrier.
// ONE_PANEL: np == 32, the whole width is one panel: no T factor, no trailing update, and far fewer
// registers, so that several work-groups share a compute unit.
template <int BR, bool ONE_PANEL = false>
__device__ __forceinline__ void fold_block(float* __restrict__ R, float* lds, int np, int ldb, int p0, int nreal) {
    constexpr int RPT = BR / 8;      // rows of a panel column held by one lane
    constexpr int MT = BR / 32;      // 32-row accumulator tiles per block
    const int NP = np / kNB;
    float* Bs = lds;                           // [BR][ldb]
    float* Gs = Bs + ((BR * ldb + 3) & ~3);    // [32][36] strict upper part of V_B^T V_B
    float* Ts = Gs + 32 * kGs;                 // [32][33] compact-WY T
    float* red = Ts + 32 * kTs;                // [2][32][4] cross-wave partial sums
    float* taus = red + 2 * 4 * 32;            // [32]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = tid & 31;          // panel column of this lane
    const int g = tid >> 5;          // row group: rows RPT*g .. RPT*g + RPT-1
    const int half = lane >> 5;

    // diagonal block of R for the first panel; later ones are fetched one panel ahead (a
    // panel's trailing update never touches the rows of R that the next panel factors)
    float rdv[32];
#pragma unroll
    for (int k = 0; k < 32; ++k) rdv[k] = R[(size_t)(p0 * kNB + k) * np + p0 * kNB + j];

    for (int p = p0; p < NP; ++p) {
        const int kp = p * kNB;
        // ================= panel factorisation =================
        float pv[RPT];
#pragma unroll
        for (int i = 0; i < RPT; ++i) pv[i] = Bs[(RPT * g + i) * ldb + kp + j];

        panel_chain<RPT, ONE_PANEL ? 0 : kChainPublish>(pv, rdv, nreal - kp, red, Gs, taus, wave, j, g, half);
        if (!ONE_PANEL) {                 // the trailing update reads the reflectors from the block
#pragma unroll
            for (int i = 0; i < RPT; ++i) Bs[(RPT * g + i) * ldb + kp + j] = pv[i];
        }
        if (g == 0) {
#pragma unroll
            for (int k = 0; k < 32; ++k)
                if (k <= j) R[(size_t)(kp + k) * np + kp + j] = rdv[k];
        }
        __syncthreads();
        if (ONE_PANEL || p + 1 == NP) break;       // last panel: nothing to the right

        // next panel's diagonal block of R: in flight during the T factor and trailing update
#pragma unroll
        for (int k = 0; k < 32; ++k) rdv[k] = R[(size_t)(kp + kNB + k) * np + kp + kNB + j];

        // ================= T factor =================
        if (wave == 0 && half == 0) t_factor_backsubst(Gs, taus, Ts, j);
        __syncthreads();

        // ================= trailing update on MFMA =================
        {
            const int c = lane & 31;
            float va1[BR / 2], va3[MT][16], tq[16];
#pragma unroll
            for (int s = 0; s < BR / 2; ++s) va1[s] = Bs[(2 * s + half) * ldb + kp + c];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int q = 0; q < 16; ++q)
                    va3[mt][q] = Bs[(mt * 32 + c) * ldb + kp + rho(q) + 4 * half];
#pragma unroll
            for (int q = 0; q < 16; ++q) tq[q] = Ts[(rho(q) + 4 * half) * kTs + c];

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
                // R tile of this wave's next column tile: its latency hides behind the MFMAs
                if (ct + 4 < NP) {
#pragma unroll
                    for (int q = 0; q < 16; ++q)
                        crn[q] = R[(size_t)(kp + rho(q) + 4 * half) * np + cc + 4 * kNB];
                }
#pragma unroll
                for (int q = 0; q < 16; ++q) acc2[q] = 0.0f;
#pragma unroll
                for (int s = 0; s < BR / 2; ++s)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(va1[s], Bs[(2 * s + half) * ldb + cc],
                                                               acc, 0, 0, 0);
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
                    for (int q = 0; q < 16; ++q)
                        cb = __builtin_amdgcn_mfma_f32_32x32x2f32(va3[mt][q], acc2[q], cb, 0, 0, 0);
#pragma unroll
                    for (int q = 0; q < 16; ++q)
                        Bs[(mt * 32 + rho(q) + 4 * half) * ldb + cc] = cb[q];
                }
                crv = crn;
            }
        }
        __syncthreads();
    }
    __syncthreads();
}

}  // namespace fold
}  // namespace elm
