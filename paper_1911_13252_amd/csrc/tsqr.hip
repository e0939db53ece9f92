// Stage 2a: tall-skinny Householder QR of the augmented matrix [H | T] (the paper's section
// "Computing beta": H = QR, z = Q^T Y; applying the reflectors to [H | T] yields R and z at once).
//
// Every work-group keeps its own upper-triangular R (np x np, global memory, L2 resident) and
// folds 64-row blocks of the input into it, one after the other:  [R; B] -> [R'; 0].  Because R is
// triangular, the reflector that eliminates column k only touches row k of R and the whole block,
// so V = [I; V_B] and one fold costs 2*64*n^2 flops: no work is spent on the zero triangle.
// Per panel of 32 columns:
//   * panel factorisation on the VALU: lanes hold 8 rows of one panel column in registers, the
//     Householder norm and all dot products of a step come from ONE reduction (wavefront shuffle
//     inside a wave, a 4-entry LDS exchange across the 4 waves);
//   * the triangular factor T of the compact-WY form Q = I - V T V^T from the Gram matrix of V_B;
//   * trailing update of the remaining 32-column tiles on fp32 MFMA:
//       Y = C_R + V_B^T C_B,  W = T^T Y,  C_R -= W,  C_B -= V_B W
//     where Y and W never leave the accumulator registers (the MFMA k-slot order is chosen so an
//     accumulator register can be fed back as a B operand).
// The R factors of all work-groups are combined by the same kernel applied to the stacked R's
// (fan-in 4 per level, skipping the panels left of each 64-row slice of a triangular input).

#include "internal.h"

namespace elm {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kRows = 64;       // rows per folded block
constexpr int kNB = 32;         // panel width = MFMA tile width
constexpr int kFan = 4;         // R factors folded by one work-group in a combine level

struct FoldArgs {
    const float* src0;   // level 0: H (ld = nc0 = L); combine: previous R stack (ld = nc0 = np)
    const float* src1;   // level 0: T (ld = nc1 = m); combine: null
    int64_t ld0, ld1;
    int nc0, nc1;
    int64_t nrows;       // level 0: N
    int nblocks;         // level 0: number of 64-row blocks
    int nprev;           // combine: number of R factors in the previous stack
    int combine;         // 0 / 1
    float* Rout;         // [gridDim.x][np][np]
    int np, ldb;
};

// row index inside a 32x32 accumulator tile held in register q by a lane of half h
__device__ __forceinline__ int rho(int q) { return 8 * (q >> 2) + (q & 3); }

__global__ __launch_bounds__(kThreads) void tsqr_fold_kernel(const FoldArgs a) {
    extern __shared__ __align__(16) float lds[];
    const int np = a.np, ldb = a.ldb, NP = np / kNB;
    float* Bs = lds;                           // [64][ldb]
    float* Ts = Bs + kRows * ldb;              // [32][33]  compact-WY T
    float* Gs = Ts + 32 * 33;                  // [32][33]  strict upper part of V_B^T V_B
    float* red = Gs + 32 * 33;                 // [2][4][32] cross-wave partial sums
    float* taus = red + 2 * 4 * 32;            // [32]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = tid & 31;          // panel column of this lane
    const int g = tid >> 5;          // row group: rows 8g .. 8g+7
    const int half = lane >> 5;
    float* R = a.Rout + (size_t)blockIdx.x * np * np;

    for (int idx = tid; idx < np * np; idx += kThreads) R[idx] = 0.0f;

    // ---- which blocks does this work-group fold?
    int blk_begin, blk_end, per_r = 1;
    if (!a.combine) {
        blk_begin = (int)(((int64_t)a.nblocks * blockIdx.x) / gridDim.x);
        blk_end = (int)(((int64_t)a.nblocks * (blockIdx.x + 1)) / gridDim.x);
    } else {
        per_r = (np + kRows - 1) / kRows;                     // 64-row slices per R factor
        const int r_begin = blockIdx.x * kFan;
        const int r_end = min(r_begin + kFan, a.nprev);
        blk_begin = r_begin * per_r;
        blk_end = r_end * per_r;
    }
    __syncthreads();

    for (int blk = blk_begin; blk < blk_end; ++blk) {
        // ---- load the block into LDS (zero padded)
        int p0 = 0;
        if (!a.combine) {
            const int64_t r0 = (int64_t)blk * kRows;
            for (int idx = tid; idx < kRows * np; idx += kThreads) {
                const int r = idx / np, c = idx - r * np;
                const int64_t row = r0 + r;
                float v = 0.0f;
                if (row < a.nrows) {
                    if (c < a.nc0) v = a.src0[row * a.ld0 + c];
                    else if (c < a.nc0 + a.nc1) v = a.src1[row * a.ld1 + (c - a.nc0)];
                }
                Bs[r * ldb + c] = v;
            }
        } else {
            const int ri = blk / per_r, slice = blk - ri * per_r;
            const float* src = a.src0 + (size_t)ri * np * np;
            const int rbase = slice * kRows;
            p0 = rbase / kNB;                                   // columns left of the slice are zero
            for (int idx = tid; idx < kRows * np; idx += kThreads) {
                const int r = idx / np, c = idx - r * np;
                const int row = rbase + r;
                Bs[r * ldb + c] = (row < np) ? src[(size_t)row * np + c] : 0.0f;
            }
        }
        __syncthreads();

        for (int p = p0; p < NP; ++p) {
            const int kp = p * kNB;
            // ================= panel factorisation =================
            float pv[8], rdv[32];
#pragma unroll
            for (int i = 0; i < 8; ++i) pv[i] = Bs[(8 * g + i) * ldb + kp + j];
#pragma unroll
            for (int k = 0; k < 32; ++k) rdv[k] = R[(size_t)(kp + k) * np + kp + j];

#pragma unroll
            for (int k = 0; k < 32; ++k) {
                const int srcl = k + (lane & 32);
                float xk[8];
                float s = 0.0f;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    xk[i] = __shfl(pv[i], srcl);
                    s = fmaf(xk[i], pv[i], s);
                }
                s += __shfl_xor(s, 32);
                float* rb = red + (k & 1) * 128;
                if (half == 0) rb[wave * 32 + j] = s;
                const float x0 = __shfl(rdv[k], srcl);
                __syncthreads();
                const float sj = (rb[j] + rb[32 + j]) + (rb[64 + j] + rb[96 + j]);
                const float sigma = (rb[k] + rb[32 + k]) + (rb[64 + k] + rb[96 + k]);
                float alpha = x0, tau = 0.0f, f = 0.0f;
                if (sigma > 0.0f) {
                    const float nrm = sqrtf(fmaf(x0, x0, sigma));
                    alpha = (x0 >= 0.0f) ? -nrm : nrm;
                    tau = (alpha - x0) / alpha;
                    f = 1.0f / (x0 - alpha);
                }
                if (j == k) {
                    rdv[k] = alpha;
#pragma unroll
                    for (int i = 0; i < 8; ++i) pv[i] = xk[i] * f;
                    if (g == 0) taus[k] = tau;
                } else if (j > k) {
                    const float w = tau * fmaf(f, sj, rdv[k]);
                    rdv[k] -= w;
                    const float fw = f * w;
#pragma unroll
                    for (int i = 0; i < 8; ++i) pv[i] = fmaf(-xk[i], fw, pv[i]);
                } else if (g == 0) {
                    Gs[j * 33 + k] = f * sj;      // v_j . v_k for the finished reflector j < k
                }
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) Bs[(8 * g + i) * ldb + kp + j] = pv[i];
            if (g == 0) {
#pragma unroll
                for (int k = 0; k < 32; ++k)
                    if (k <= j) R[(size_t)(kp + k) * np + kp + j] = rdv[k];
            }
            __syncthreads();
            if (p + 1 == NP) break;       // last panel: nothing to the right

            // ================= T factor (forward, column by column) =================
            if (wave == 0 && half == 0) {
                float trow[32];
#pragma unroll
                for (int k = 0; k < 32; ++k) trow[k] = 0.0f;
#pragma unroll
                for (int k = 0; k < 32; ++k) {
                    float acc = 0.0f;
#pragma unroll
                    for (int l = 0; l < k; ++l) acc = fmaf(trow[l], Gs[l * 33 + k], acc);
                    const float tk = taus[k];
                    trow[k] = (j == k) ? tk : ((j < k) ? -tk * acc : 0.0f);
                }
#pragma unroll
                for (int k = 0; k < 32; ++k) Ts[j * 33 + k] = trow[k];
            }
            __syncthreads();

            // ================= trailing update on MFMA =================
            {
                const int c = lane & 31;
                float va1[32], va3[2][16], tq[16];
#pragma unroll
                for (int s = 0; s < 32; ++s) va1[s] = Bs[(2 * s + half) * ldb + kp + c];
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int q = 0; q < 16; ++q)
                        va3[mt][q] = Bs[(mt * 32 + c) * ldb + kp + rho(q) + 4 * half];
#pragma unroll
                for (int q = 0; q < 16; ++q) tq[q] = Ts[(rho(q) + 4 * half) * 33 + c];

                for (int ct = p + 1 + wave; ct < NP; ct += 4) {
                    const int cc = ct * kNB + c;
                    floatx16 crv, acc, acc2;
#pragma unroll
                    for (int q = 0; q < 16; ++q) {
                        crv[q] = R[(size_t)(kp + rho(q) + 4 * half) * np + cc];
                        acc[q] = crv[q];
                        acc2[q] = 0.0f;
                    }
#pragma unroll
                    for (int s = 0; s < 32; ++s)
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
                    for (int mt = 0; mt < 2; ++mt) {
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
                }
            }
            __syncthreads();
        }
        __syncthreads();
    }
}

size_t fold_lds_bytes(int np) {
    const int ldb = np + 1;
    return ((size_t)kRows * ldb + 2 * 32 * 33 + 2 * 4 * 32 + 32) * sizeof(float);
}

}  // namespace

SolvePlan make_solve_plan(int64_t N, int L, int m) {
    SolvePlan pl{};
    pl.N = N; pl.L = L; pl.m = m;
    pl.n = L + m;
    pl.np = (pl.n + 31) / 32 * 32;
    const int64_t nblocks = (N + kRows - 1) / kRows;
    int64_t g0 = (nblocks + 3) / 4;
    if (g0 < 1) g0 = 1;
    if (g0 > 256) g0 = 256;
    pl.levels = 0;
    pl.groups[pl.levels++] = (int)g0;
    while (pl.groups[pl.levels - 1] > 1) {
        pl.groups[pl.levels] = (pl.groups[pl.levels - 1] + kFan - 1) / kFan;
        ++pl.levels;
    }
    auto align = [](size_t v) { return (v + 255) & ~(size_t)255; };
    const size_t rbytes = (size_t)pl.np * pl.np * sizeof(float);
    size_t off = 0;
    pl.off_R[0] = off; off = align(off + rbytes * pl.groups[0]);
    pl.off_R[1] = off; off = align(off + rbytes * (pl.levels > 1 ? pl.groups[1] : 1));
    pl.off_part = off; off = align(off + (size_t)1024 * ((size_t)L * m + 2) * sizeof(double));
    pl.off_small = off; off = align(off + SmallArea::doubles(L, m) * sizeof(double));
    pl.bytes = off;
    return pl;
}

hipError_t launch_tsqr(const SolvePlan& pl, const float* H, const float* T, void* ws, float** R_final,
                       hipStream_t stream) {
    const size_t lds = fold_lds_bytes(pl.np);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(tsqr_fold_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    char* base = static_cast<char*>(ws);
    FoldArgs a{};
    a.np = pl.np;
    a.ldb = pl.np + 1;
    for (int lvl = 0; lvl < pl.levels; ++lvl) {
        float* out = reinterpret_cast<float*>(base + pl.off_R[lvl & 1]);
        if (lvl == 0) {
            a.src0 = H; a.ld0 = pl.L; a.nc0 = pl.L;
            a.src1 = T; a.ld1 = pl.m; a.nc1 = pl.m;
            a.nrows = pl.N;
            a.nblocks = (int)((pl.N + kRows - 1) / kRows);
            a.combine = 0; a.nprev = 0;
        } else {
            a.src0 = reinterpret_cast<const float*>(base + pl.off_R[(lvl - 1) & 1]);
            a.ld0 = pl.np; a.nc0 = pl.np;
            a.src1 = nullptr; a.ld1 = 0; a.nc1 = 0;
            a.nrows = 0; a.nblocks = 0;
            a.combine = 1; a.nprev = pl.groups[lvl - 1];
        }
        a.Rout = out;
        hipLaunchKernelGGL(tsqr_fold_kernel, dim3(pl.groups[lvl]), dim3(kThreads), lds, stream, a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        *R_final = out;
    }
    return hipSuccess;
}

}  // namespace elm
