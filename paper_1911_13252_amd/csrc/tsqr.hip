// Stage 2a: tall-skinny Householder QR of the augmented matrix [H | T] (the paper's section
// "Computing beta": H = QR, z = Q^T Y; applying the reflectors to [H | T] yields R and z at once).
//
// Every work-group keeps its own upper-triangular R (np x np, global memory) and folds BR-row blocks (64 or 128
// rows) of the input into it, one after the other: [R; B] -> [R'; 0].  Because R is triangular, the reflector
// that eliminates column k only touches row k of R and the whole block, so V = [I; V_B] and one fold costs
// 2*BR*n^2 flops: no work is spent on the zero triangle.
// Per panel of 32 columns:
//   * panel factorisation on the VALU (panel_chain in tsqr_fold.h): lanes hold BR/8 rows of one panel column in
//     registers, the Householder norm and all dot products of a step come from ONE reduction (wavefront shuffle
//     inside a wave, a 16-byte LDS read across the 4 waves);
//   * the triangular factor T of the compact-WY form Q = I - V T V^T from the Gram matrix of V_B;
//   * trailing update of the remaining 32-column tiles on fp32 MFMA:
//       Y = C_R + V_B^T C_B,  W = T^T Y,  C_R -= W,  C_B -= V_B W
//     where Y and W never leave the accumulator registers (the MFMA k-slot order is chosen so an
//     accumulator register can be fed back as a B operand).
// The block lives in LDS (fold_block, fold_block_tw: up to 288 padded columns at 128 rows) or mostly in
// registers (fold_blocks_rr: wider matrices).
// The R factors of all work-groups are combined by the same kernels in a binary tree: a work-group
// starts from a copy of its first R and folds the row slices of the second one into it (skipping the
// panels left of each slice of the triangular input), so a level costs one R fold of serial work.

#include "internal.h"
#include "tsqr_fold.h"
#include "tsqr_fold_tw.h"
#include "tsqr_fold_rr.h"

namespace elm {
namespace {

using namespace fold;

constexpr int kFan = 2;         // R factors merged by one work-group in a combine level

struct FoldArgs {
    const float* src0;   // level 0: H (ld = nc0 = L); combine: previous R stack (ld = nc0 = np)
    const float* src1;   // level 0: T (ld = nc1 = m); combine: null
    int64_t ld0, ld1;
    int nc0, nc1;
    int64_t nrows;       // level 0: N
    int nblocks;         // level 0: number of BR-row blocks
    int nprev;           // combine: number of R factors in the previous stack
    int combine;         // 0 / 1
    int keep;            // level 0: fold into the R factors already in Rout (a later chunk of rows)
    int nreal;           // columns of [H | T]; the rest of np is zero padding
    float* Rout;         // [gridDim.x][np][np]
    int np, ldb;
};

// BR = rows per folded block (64 or 128).  Taller blocks halve the number of sequential
// Householder steps per input row; they are used whenever the block fits in LDS.
// Which fold a kernel variant runs:
//   kOnePanel  np == 32: four waves, no T factor and no trailing update, three work-groups per compute unit;
//   kTWave     every wider matrix: five waves, the T factor built by the fifth while the chain runs
//              (fold_block_tw; 10 % faster than the four-wave fold_block on 64-row blocks at 544 columns, 2 - 4 %
//              on 128-row blocks, where a wave's 256 registers hold only half of the update's operands).
enum FoldMode { kOnePanel = 0, kTWave = 2 };

template <int BR, int MODE>
__global__ __launch_bounds__(MODE == kTWave ? kThreadsTW : kThreads, MODE == kOnePanel ? 3 : 1)
void tsqr_fold_kernel(const FoldArgs a) {
    constexpr int kT = MODE == kTWave ? kThreadsTW : kThreads;  // threads of the work-group
    constexpr int kW = kT / 64;                                 // ... and waves
    extern __shared__ __align__(16) float lds[];
    const int np = a.np, ldb = a.ldb;
    float* Bs = lds;                           // [BR][ldb], then the scratch areas of fold_block
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    float* R = a.Rout + (size_t)blockIdx.x * np * np;

    // ---- which blocks does this work-group fold, and what does its R start from?
    int blk_begin, blk_end, per_r = 1;
    if (!a.combine) {
        if (!a.keep)
            for (int idx = tid; idx < np * np; idx += kT) R[idx] = 0.0f;
        blk_begin = (int)(((int64_t)a.nblocks * blockIdx.x) / gridDim.x);
        blk_end = (int)(((int64_t)a.nblocks * (blockIdx.x + 1)) / gridDim.x);
    } else {
        per_r = (np + BR - 1) / BR;                           // BR-row slices per R factor
        const int r_begin = blockIdx.x * kFan;
        const int r_end = min(r_begin + kFan, a.nprev);
        const float* first = a.src0 + (size_t)r_begin * np * np;
        for (int idx = tid; idx < np * np; idx += kT) R[idx] = first[idx];
        blk_begin = (r_begin + 1) * per_r;
        blk_end = r_end * per_r;
    }
    __syncthreads();

    for (int blk = blk_begin; blk < blk_end; ++blk) {
        // ---- load the block into LDS (zero padded).  A wave takes 8 rows at a time and issues all of
        // their loads before the first LDS store, so a block costs a handful of memory round trips.
        int p0 = 0;
        {
            const float* src0;
            const float* src1 = a.src1;
            int64_t ld0, row_first, row_limit;
            int nc0, nc1;
            if (!a.combine) {
                src0 = a.src0; ld0 = a.ld0; nc0 = a.nc0; nc1 = a.nc1;
                row_first = (int64_t)blk * BR; row_limit = a.nrows;
            } else {
                const int ri = blk / per_r, slice = blk - ri * per_r;
                src0 = a.src0 + (size_t)ri * np * np; ld0 = np; nc0 = np; nc1 = 0;
                row_first = (int64_t)slice * BR; row_limit = np;
                p0 = (slice * BR) / kNB;                        // columns left of the slice are zero
            }
            constexpr int U = 8;
            const bool vec4 = ((nc0 & 3) == 0) && ((ld0 & 3) == 0) &&
                              ((reinterpret_cast<uintptr_t>(src0) & 15) == 0);
            for (int rb = wave * U; rb < BR; rb += kW * U) {
                if (vec4) {
                    for (int c = lane * 4; c < nc0; c += 256) {
                        float4 v[U];
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            const int64_t row = row_first + rb + u;
                            v[u] = (row < row_limit) ? *reinterpret_cast<const float4*>(src0 + row * ld0 + c)
                                                     : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                        }
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            float* dst = Bs + (rb + u) * ldb + c;
                            dst[0] = v[u].x; dst[1] = v[u].y; dst[2] = v[u].z; dst[3] = v[u].w;
                        }
                    }
                } else {
                    for (int c = lane; c < nc0; c += 64) {
                        float v[U];
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            const int64_t row = row_first + rb + u;
                            v[u] = (row < row_limit) ? src0[row * ld0 + c] : 0.0f;
                        }
#pragma unroll
                        for (int u = 0; u < U; ++u) Bs[(rb + u) * ldb + c] = v[u];
                    }
                }
                for (int c = nc0 + lane; c < np; c += 64) {       // targets, then zero padding
                    float v[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int64_t row = row_first + rb + u;
                        v[u] = (row < row_limit && c < nc0 + nc1) ? src1[row * a.ld1 + (c - nc0)] : 0.0f;
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) Bs[(rb + u) * ldb + c] = v[u];
                }
            }
        }
        __syncthreads();

        if constexpr (MODE == kTWave) fold_block_tw<BR>(R, lds, np, ldb, p0, a.nreal);
        else fold_block<BR, MODE == kOnePanel>(R, lds, np, ldb, p0, a.nreal);
    }
}

// The same level-0 / combine fold with most of the block in registers (fold_block_rr): 128-row blocks (MT = 4)
// for the widths whose 128-row block does not fit LDS.
template <int MT>
__global__ __launch_bounds__(kThreads, 1)
void tsqr_fold_rr_kernel(const FoldArgs a) {
    constexpr int BR = 32 * MT;
    extern __shared__ __align__(16) float lds[];
    const int np = a.np;
    const int tid = threadIdx.x;
    float* R = a.Rout + (size_t)blockIdx.x * np * np;

    int blk_begin, blk_end, per_r = 1;
    if (!a.combine) {
        if (!a.keep)
            for (int idx = tid; idx < np * np; idx += kThreads) R[idx] = 0.0f;
        blk_begin = (int)(((int64_t)a.nblocks * blockIdx.x) / gridDim.x);
        blk_end = (int)(((int64_t)a.nblocks * (blockIdx.x + 1)) / gridDim.x);
    } else {
        per_r = (np + BR - 1) / BR;
        const int r_begin = blockIdx.x * kFan;
        const int r_end = min(r_begin + kFan, a.nprev);
        const float* first = a.src0 + (size_t)r_begin * np * np;
        for (int idx = tid; idx < np * np; idx += kThreads) R[idx] = first[idx];
        blk_begin = (r_begin + 1) * per_r;
        blk_end = r_end * per_r;
    }
    __syncthreads();

    FoldInput in;
    in.src0 = a.src0; in.src1 = a.src1; in.ld0 = a.ld0; in.ld1 = a.ld1; in.nc0 = a.nc0; in.nc1 = a.nc1;
    in.nrows = a.nrows; in.combine = a.combine; in.per_r = per_r; in.np = np; in.nreal = a.nreal;
    fold_blocks_rr<MT>(R, in, blk_begin, blk_end, lds, np);
}

size_t fold_lds_bytes(int np, int br) {
    return (np > 32 ? fold::lds_floats_tw(np, br) : fold::lds_floats(np, br)) * sizeof(float);
}

}  // namespace

SolvePlan make_solve_plan(int64_t N, int L, int m, int level0_groups) {
    SolvePlan pl{};
    pl.N = N; pl.L = L; pl.m = m;
    pl.n = L + m;
    pl.np = (pl.n + 31) / 32 * 32;
    // 128-row blocks when there are enough rows for them (in LDS if the padded width allows it, else in
    // registers)
    pl.block_rows = (N >= 128 * 64) ? 128 : 64;
    const int64_t nblocks = (N + pl.block_rows - 1) / pl.block_rows;
    int64_t g0 = (nblocks + 3) / 4;
    if (g0 < 1) g0 = 1;
    // one work-group per compute unit; three where the width is a single panel (np == 32: that kernel
    // needs few registers and little LDS, and its Householder chains then overlap); at most 1024 R factors
    const int cus = device_compute_units();
    int64_t cap = (pl.np == 32) ? 3 * (int64_t)cus : cus;
    if (cap > 1024) cap = 1024;
    if (g0 > cap) g0 = cap;
    if (level0_groups > 0) g0 = level0_groups;      // the fused stage-1 kernel brings its own grid
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

namespace {

struct FoldLaunch {
    void (*kern)(const FoldArgs);
    int br;
    size_t lds;
    int threads;
};

hipError_t fold_launch_config(const SolvePlan& pl, bool combine, FoldLaunch* fl) {
    int dev = 0, lds_max = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    e = hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
    if (e != hipSuccess) return e;
    // 128-row blocks whenever the input is tall enough to keep the grid busy: in LDS if they fit there, else
    // in registers
    const bool fits = fold_lds_bytes(pl.np, 128) <= (size_t)lds_max;
    const bool tall = fits && pl.block_rows == 128;
    fl->br = tall ? 128 : 64;
    fl->lds = fold_lds_bytes(pl.np, fl->br);
    fl->threads = (pl.np > 32) ? kThreadsTW : kThreads;
    if (!fits && pl.block_rows == 128) {
        fl->br = 128;
        fl->lds = fold::lds_floats_rr(pl.np, 128) * sizeof(float);
        if (fl->lds > (size_t)lds_max) return hipErrorInvalidValue;      // np <= 544 fits; the library admits no more
        fl->threads = kThreads;
        fl->kern = tsqr_fold_rr_kernel<4>;
        return hipFuncSetAttribute(reinterpret_cast<const void*>(fl->kern),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)fl->lds);
    }
    if (pl.np == 32 && combine) {
        // a 32 x 32 triangular input is one 32-row block: the shortest Householder steps
        fl->br = 32;
        fl->lds = fold_lds_bytes(pl.np, 32);
        fl->kern = tsqr_fold_kernel<32, kOnePanel>;
    } else if (pl.np == 32) {
        fl->kern = tall ? tsqr_fold_kernel<128, kOnePanel> : tsqr_fold_kernel<64, kOnePanel>;
    } else {
        fl->kern = tall ? tsqr_fold_kernel<128, kTWave> : tsqr_fold_kernel<64, kTWave>;
    }
    return hipFuncSetAttribute(reinterpret_cast<const void*>(fl->kern),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)fl->lds);
}

}  // namespace

// Level 0 over `rows` rows of H and T: every work-group folds its share of the row blocks into its
// own R factor, which starts from zero (keep == 0) or from what earlier calls left there (keep != 0:
// the rows arrive in chunks; the work-group count of the plan is used for every chunk).
hipError_t launch_tsqr_level0(const SolvePlan& pl, const float* H, const float* T, int64_t rows, void* ws,
                              int keep, hipStream_t stream) {
    FoldLaunch fl{};
    hipError_t e = fold_launch_config(pl, false, &fl);
    if (e != hipSuccess) return e;
    FoldArgs a{};
    a.np = pl.np;
    a.ldb = pl.np + 1;
    a.src0 = H; a.ld0 = pl.L; a.nc0 = pl.L;
    a.src1 = T; a.ld1 = pl.m; a.nc1 = pl.m;
    a.nrows = rows;
    a.nblocks = (int)((rows + fl.br - 1) / fl.br);
    a.combine = 0; a.nprev = 0; a.keep = keep;
    a.nreal = pl.n;
    a.Rout = reinterpret_cast<float*>(static_cast<char*>(ws) + pl.off_R[0]);
    hipLaunchKernelGGL(fl.kern, dim3(pl.groups[0]), dim3(fl.threads), fl.lds, stream, a);
    return hipGetLastError();
}

// The combine levels: merge the level-0 R factors pairwise until one is left.
hipError_t launch_tsqr_combine(const SolvePlan& pl, void* ws, float** R_final, hipStream_t stream) {
    FoldLaunch fl{};
    hipError_t e = fold_launch_config(pl, true, &fl);
    if (e != hipSuccess) return e;
    char* base = static_cast<char*>(ws);
    *R_final = reinterpret_cast<float*>(base + pl.off_R[0]);
    FoldArgs a{};
    a.np = pl.np;
    a.ldb = pl.np + 1;
    a.ld0 = pl.np; a.nc0 = pl.np;
    a.combine = 1;
    a.nreal = pl.n;
    for (int lvl = 1; lvl < pl.levels; ++lvl) {
        a.src0 = reinterpret_cast<const float*>(base + pl.off_R[(lvl - 1) & 1]);
        a.nprev = pl.groups[lvl - 1];
        a.Rout = reinterpret_cast<float*>(base + pl.off_R[lvl & 1]);
        hipLaunchKernelGGL(fl.kern, dim3(pl.groups[lvl]), dim3(fl.threads), fl.lds, stream, a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        *R_final = a.Rout;
    }
    return hipSuccess;
}

hipError_t launch_tsqr(const SolvePlan& pl, const float* H, const float* T, void* ws, float** R_final,
                       hipStream_t stream) {
    hipError_t e = launch_tsqr_level0(pl, H, T, pl.N, ws, 0, stream);
    if (e != hipSuccess) return e;
    return launch_tsqr_combine(pl, ws, R_final, stream);
}

}  // namespace elm
