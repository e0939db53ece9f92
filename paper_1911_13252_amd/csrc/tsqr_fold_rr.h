// One fold step of the tall-skinny QR, [R; B] -> [R'; 0] (the paper's section "Computing beta": H = QR applied
// to [H | T] a block of rows at a time), for matrices too wide for a 128-row block in LDS: most of the block
// lives in REGISTERS, in the accumulator layout of the 32x32 matrix instruction.
//
// A compute unit has 512 KB of vector registers against 160 KB of LDS.  Four waves hold the first twelve
// 32-column tiles of a 128-row block in their accumulation registers (wave w owns tiles w, w + 4, w + 8; a tile
// is MT 32x32 accumulators; with Y and W that fills the 256 accumulation registers, the only place the compiler
// puts an accumulator operand), the remaining tiles (five at 544 columns) stay in LDS.  Against the 64-row
// block that fits LDS as a whole at more than 288 columns this halves the number of Householder column steps
// per input row and the traffic of the R factor.  Both products of the trailing update take a register tile
// where it is: an accumulator register holds rows r and r + 4 of the tile in its two half-waves, which is
// exactly a B operand of the matrix instruction for the k-slot (r, r + 4), and C_B -= V_B W accumulates in
// place.  An LDS tile is read into vector registers in the same layout, enters both products as a B operand,
// and is written back after a vector add of the second product.  The panel being factored is staged in LDS
// (the owner of a register tile writes it there before the chain; an LDS tile is factored where it is), and the
// reflectors that replace it serve as A operands.
//
// The T factor is a serial back substitution of one half-wave.  It runs on the wave that owns tile p, which
// has one tile less to update than the busiest wave in three panels out of four, and the other waves start
// the first product of their first tile (which does not need T) meanwhile.
#pragma once

#include <hip/hip_runtime.h>

#include "tsqr_fold_tw.h"

namespace elm {
namespace fold {

constexpr int kLdp = 33;           // row stride of a tile in LDS
constexpr int kSlotsRR = 3;        // register tiles per wave
constexpr int kRegTilesRR = 4 * kSlotsRR;

__host__ __device__ inline int lds_tiles_rr(int np) { return np / kNB > kRegTilesRR ? np / kNB - kRegTilesRR : 0; }

// LDS floats: the staged panel and the LDS tiles (BR x 32 each, row stride 33), the Gram matrix, the T factor,
// cross-wave partial sums, tau
__host__ __device__ inline size_t lds_floats_rr(int np, int br) {
    return (size_t)(1 + lds_tiles_rr(np)) * ((br * kLdp + 3) & ~3) + 32 * kGs + 32 * kTs + 2 * 4 * 32 + 32;
}

// Where the rows of a block come from: columns [0, nc0) from src0, [nc0, nc0 + nc1) from src1, zero beyond;
// rows at or beyond row_limit are zero.
struct BlockSource {
    const float* src0;
    const float* src1;
    int64_t ld0, ld1;
    int nc0, nc1;
    int64_t row_first, row_limit;
};

// One 32-column tile of the block (all zero unless valid) in the accumulator layout: register q of
// accumulator mt holds row 32 mt + rho(q) + 4 half, column lane % 32.
template <int MT>
__device__ __forceinline__ void load_tile_rr(floatx16 (&t)[MT], const BlockSource& b, int tile, bool valid,
                                             int lane) {
    const int c = lane & 31, half = lane >> 5;
    const int col = tile * kNB + c;
    const bool from0 = col < b.nc0;
    const bool colok = valid && col < b.nc0 + b.nc1;
    const float* base = from0 ? b.src0 + col : b.src1 + (col - b.nc0);
    const int64_t ld = from0 ? b.ld0 : b.ld1;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int64_t row = b.row_first + mt * 32 + rho(q) + 4 * half;
            t[mt][q] = (colok && row < b.row_limit) ? base[row * ld] : 0.0f;
        }
}

// Trailing update of one 32-column tile with the panel's reflectors V_B (Vp, BR x 32, row stride 33) and
// factor T (Ts):
//   Y = C_R + V_B^T C_B,  W = T^T Y,  C_R -= W,  C_B -= V_B W.
// cbt: the tile's rows of the block; in_place: the last product accumulates into cbt (register tiles) or into a
// temporary that is then added (tiles that only pass through vector registers); Rrs: buffer descriptor of R;
// rt_lane: byte offset of (row 4 half, column j), one vector register for every access; rt_wave: byte offset of
// the tile's first element (row kp, column 32 ct), scalar; synced: whether this wave has already passed the
// barrier after which T is complete (passed here, after the first product, if not).  A operands are read from
// LDS one group of 16 ahead of the matrix instructions that use them.
template <int MT>
__device__ __forceinline__ void update_tile_rr(floatx16 (&cbt)[MT], const bool in_place, __amdgpu_buffer_rsrc_t Rrs,
                                               unsigned rt_lane, unsigned rt_wave, int np, const float* Vp,
                                               const float* Ts, int j, int half, bool& synced) {
    floatx16 acc, acc2;
    float crv[16], va[2][16];
#pragma unroll
    for (int q = 0; q < 16; ++q)
        crv[q] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                               Rrs, rt_lane, rt_wave + (unsigned)(rho(q) * np) * 4u, 0));
#pragma unroll
    for (int q = 0; q < 16; ++q) va[0][q] = Vp[(rho(q) + 4 * half) * kLdp + j];
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[q] = 0.0f;
    // V_B^T C_B: k-slot (mt, q) pairs rows 32 mt + rho(q) and + 4 of the block
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        if (mt + 1 < MT) {
#pragma unroll
            for (int q = 0; q < 16; ++q)
                va[(mt + 1) & 1][q] = Vp[((mt + 1) * 32 + rho(q) + 4 * half) * kLdp + j];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < 16; ++q)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(va[mt & 1][q], cbt[mt][q], acc, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
    if (!synced) {
        __syncthreads();        // T is complete
        synced = true;
    }
    float tq[16], y[16], w[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) tq[q] = Ts[(rho(q) + 4 * half) * kTs + j];
#pragma unroll
    for (int q = 0; q < 16; ++q) va[0][q] = Vp[j * kLdp + rho(q) + 4 * half];
#pragma unroll
    for (int q = 0; q < 16; ++q) y[q] = acc[q] + crv[q];
#pragma unroll
    for (int q = 0; q < 16; ++q) acc2[q] = 0.0f;
    __builtin_amdgcn_sched_barrier(0);
    // W = T^T Y
#pragma unroll
    for (int q = 0; q < 16; ++q) acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(tq[q], y[q], acc2, 0, 0, 0);
    // C_R -= W
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, crv[q] - acc2[q]), Rrs, rt_lane,
                                              rt_wave + (unsigned)(rho(q) * np) * 4u, 0);
        w[q] = -acc2[q];
    }
    // C_B -= V_B W
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        if (mt + 1 < MT) {
#pragma unroll
            for (int q = 0; q < 16; ++q)
                va[(mt + 1) & 1][q] = Vp[((mt + 1) * 32 + j) * kLdp + rho(q) + 4 * half];
        }
        __builtin_amdgcn_sched_barrier(0);
        if (in_place) {
#pragma unroll
            for (int q = 0; q < 16; ++q)
                cbt[mt] = __builtin_amdgcn_mfma_f32_32x32x2f32(va[mt & 1][q], w[q], cbt[mt], 0, 0, 0);
        } else {
            floatx16 tmp;
#pragma unroll
            for (int q = 0; q < 16; ++q) tmp[q] = 0.0f;
#pragma unroll
            for (int q = 0; q < 16; ++q)
                tmp = __builtin_amdgcn_mfma_f32_32x32x2f32(va[mt & 1][q], w[q], tmp, 0, 0, 0);
#pragma unroll
            for (int q = 0; q < 16; ++q) cbt[mt][q] += tmp[q];
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Loads the block (tiles p0 .. NP-1; the ones left of p0 are zero in the source and never touched) and folds it.
// R: this work-group's np x np upper-triangular factor (global memory); lds: lds_floats_rr(np, 32 MT) floats;
// p0: first panel that can be non-zero in the block.  All 256 threads call it; it ends with a barrier.
// np <= 32 (12 + 5): the LDS tiles of wider matrices would not fit.
template <int MT>
__device__ __forceinline__ void fold_block_rr(float* __restrict__ R, const BlockSource& src, float* lds, int np,
                                              int p0) {
    constexpr int BR = 32 * MT;
    constexpr int RPT = BR / 8;      // rows of a panel column held by one lane during the chain
    constexpr int kTile = (BR * kLdp + 3) & ~3;
    const int NP = np / kNB;
    const int NL = lds_tiles_rr(np);
    float* Pb = lds;                           // [BR][33] staged panel of a register tile
    float* Lt = Pb + kTile;                    // [NL][BR][33] tiles 12 .. NP-1
    float* Gs = Lt + NL * kTile;               // [32][36] strict upper part of V_B^T V_B
    float* Ts = Gs + 32 * kGs;                 // [32][33] compact-WY T
    float* red = Ts + 32 * kTs;                // [2][4][32] cross-wave partial sums
    float* taus = red + 2 * 4 * 32;            // [32]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = tid & 31;          // panel column of this lane (chain) = tile column (update)
    const int g = tid >> 5;          // row group of the chain: rows RPT*g .. RPT*g + RPT-1
    const int half = lane >> 5;
    // the tiles of R go through a buffer descriptor: base and tile offset in scalar registers, one vector
    // register of lane offsets for every access (accesses beyond the np x np floats are dropped)
    const __amdgpu_buffer_rsrc_t Rrs = __builtin_amdgcn_make_buffer_rsrc(R, 0, np * np * 4, 0x00020000);
    const unsigned rt_lane = (unsigned)(4 * half * np + j) * 4u;

    // ---- the block: register tiles of this wave, then its LDS tiles (tile t belongs to wave t % 4)
    floatx16 cb[kSlotsRR][MT];
#pragma unroll
    for (int i = 0; i < kSlotsRR; ++i) {
        const int t = wave + 4 * i;
        load_tile_rr<MT>(cb[i], src, t, t >= p0 && t < NP, lane);
    }
    for (int t = kRegTilesRR + wave; t < NP; t += 4) {
        floatx16 tl[MT];
        load_tile_rr<MT>(tl, src, t, t >= p0, lane);
        float* dst = Lt + (t - kRegTilesRR) * kTile;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int q = 0; q < 16; ++q) dst[(mt * 32 + rho(q) + 4 * half) * kLdp + j] = tl[mt][q];
    }

    float rdv[32];
#pragma unroll
    for (int k = 0; k < 32; ++k) rdv[k] = R[(size_t)(p0 * kNB + k) * np + p0 * kNB + j];
    for (int p = p0; p < NP; ++p) {
        const int kp = p * kNB;
        const int ow = p & 3;                  // the wave that owns tile p
        float* Vp = (p < kRegTilesRR) ? Pb : Lt + (p - kRegTilesRR) * kTile;
        if (p < kRegTilesRR && wave == ow) {
            const int io = p >> 2;
#pragma unroll
            for (int i = 0; i < kSlotsRR; ++i) {
                if (i == io) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int q = 0; q < 16; ++q)
                            Pb[(mt * 32 + rho(q) + 4 * half) * kLdp + j] = cb[i][mt][q];
                }
            }
        }
        __syncthreads();

        // ================= panel factorisation (the chain of fold_block) =================
        float pv[RPT];
#pragma unroll
        for (int i = 0; i < RPT; ++i) pv[i] = Vp[(RPT * g + i) * kLdp + j];
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            float xk[RPT];
            float s = 0.0f;
#pragma unroll
            for (int i = 0; i < RPT; ++i) {
                const float lo = lane_bcast(pv[i], k);
                const float hi = lane_bcast(pv[i], 32 + k);
                xk[i] = half ? hi : lo;
                s = fmaf(xk[i], pv[i], s);
            }
            s += other_half(s, half);
            float* rb = red + (k & 1) * 128;
            if (half == 0) rb[wave * 32 + j] = s;
            const float x0 = lane_bcast(rdv[k], k);
            lds_barrier();
            const float sj = (rb[j] + rb[32 + j]) + (rb[64 + j] + rb[96 + j]);
            const float sigma = (rb[k] + rb[32 + k]) + (rb[64 + k] + rb[96 + k]);
            float alpha = x0, tau = 0.0f, f = 0.0f;
            const float nrm2 = fmaf(x0, x0, sigma);
            if (sigma > 0.0f && nrm2 > 1e-30f) {
                const float nrm = __builtin_amdgcn_sqrtf(nrm2);
                alpha = (x0 >= 0.0f) ? -nrm : nrm;
                tau = (alpha - x0) * __builtin_amdgcn_rcpf(alpha);
                f = __builtin_amdgcn_rcpf(x0 - alpha);
            }
            const float w = (j > k) ? tau * fmaf(f, sj, rdv[k]) : 0.0f;
            rdv[k] = (j == k) ? alpha : rdv[k] - w;
            const float cf = (j == k) ? f : -(f * w);
#pragma unroll
            for (int i = 0; i < RPT; ++i) pv[i] = fmaf(xk[i], cf, (j == k) ? 0.0f : pv[i]);
            if (g == 0) {
                if (j == k) taus[k] = tau;
                if (j < k) Gs[j * kGs + k] = f * sj;      // v_j . v_k for the finished reflector j
            }
        }
#pragma unroll
        for (int i = 0; i < RPT; ++i) Vp[(RPT * g + i) * kLdp + j] = pv[i];
        if (g == 0) {
#pragma unroll
            for (int k = 0; k < 32; ++k)
                if (k <= j) R[(size_t)(kp + k) * np + kp + j] = rdv[k];
        }
        __syncthreads();                    // E1: reflectors in place of the panel; tau and Gram matrix complete
        if (p + 1 == NP) break;
        // next panel's diagonal block of R: in flight during the trailing update, which never touches the
        // rows of R that the next panel factors
#pragma unroll
        for (int k = 0; k < 32; ++k) rdv[k] = R[(size_t)(kp + kNB + k) * np + kp + kNB + j];

        // ================= T factor and trailing update =================
        {
            // Every wave passes E2 exactly once: the owner of tile p after it has built T, the others after the
            // first product of their first tile (or at the end, if they have no tile).
            bool synced = false;
            if (wave == ow) {
                if (half == 0) t_factor_backsubst(Gs, taus, Ts, j);
                __syncthreads();                // E2
                synced = true;
            }
#pragma unroll
            for (int i = 0; i < kSlotsRR; ++i) {
                const int ct = wave + 4 * i;
                if (ct > p && ct < NP)
                    update_tile_rr<MT>(cb[i], true, Rrs, rt_lane, (unsigned)(kp * np + ct * kNB) * 4u, np, Vp, Ts, j,
                                       half, synced);
            }
            for (int ct = kRegTilesRR + wave; ct < NP; ct += 4) {
                if (ct <= p) continue;
                float* tile = Lt + (ct - kRegTilesRR) * kTile;
                floatx16 tl[MT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int q = 0; q < 16; ++q) tl[mt][q] = tile[(mt * 32 + rho(q) + 4 * half) * kLdp + j];
                update_tile_rr<MT>(tl, false, Rrs, rt_lane, (unsigned)(kp * np + ct * kNB) * 4u, np, Vp, Ts, j, half,
                                   synced);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int q = 0; q < 16; ++q) tile[(mt * 32 + rho(q) + 4 * half) * kLdp + j] = tl[mt][q];
            }
            if (!synced) __syncthreads();       // E2
        }
        __syncthreads();                    // E3: the staging area is free for the next panel
    }
    __syncthreads();
}

}  // namespace fold
}  // namespace elm
