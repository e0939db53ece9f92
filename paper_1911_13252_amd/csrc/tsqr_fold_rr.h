// One fold step of the tall-skinny QR, [R; B] -> [R'; 0] (the paper's section "Computing beta": H = QR applied
// to [H | T] a block of rows at a time), for matrices too wide for a 128-row block in LDS: most of the block
// lives in REGISTERS, in the accumulator layout of the 32x32 matrix instruction.
//
// A compute unit has 512 KB of vector registers against 160 KB of LDS.  Four waves hold the LAST twelve
// 32-column tiles of a 128-row block in their accumulation registers (a tile is MT 32x32 accumulators; three
// tiles, Y and W fill the 256 accumulation registers, the only place the compiler puts an accumulator
// operand), the first tiles (five at 544 columns) stay in LDS.  A tile is updated by every panel left of it,
// so the last twelve of seventeen tiles take 126 of the 136 tile updates of a block.  Against the 64-row block
// that fits LDS as a whole at more than 288 columns this halves the number of Householder column steps per
// input row and the traffic of the R factor.  Both products of the trailing update take a register tile where
// it is: an accumulator register holds rows r and r + 4 of the tile in its two half-waves, which is exactly a
// B operand of the matrix instruction for the k-slot (r, r + 4), and C_B -= V_B W accumulates in place.  An LDS
// tile is read into vector registers in the same layout, enters both products as a B operand, and is written
// back after a vector add of the second product.  The panel being factored is staged in LDS (the owner of a
// register tile writes it there right after it has updated it for the panel before; an LDS tile is factored
// where it is), and the reflectors that replace it serve as A operands.
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
constexpr int kRegTilesRR = 4 * kSlotsRR;        // the last twelve tiles of a block

__host__ __device__ inline int lds_tiles_rr(int np) { return np / kNB > kRegTilesRR ? np / kNB - kRegTilesRR : 0; }

// LDS floats: two staging areas for the panels of register tiles and the LDS tiles (BR x 32 each, row stride
// 33), the Gram matrix, the T factor, cross-wave partial sums, tau
__host__ __device__ inline size_t lds_floats_rr(int np, int br) {
    return (size_t)(2 + lds_tiles_rr(np)) * ((br * kLdp + 3) & ~3) + 32 * kGs + 32 * kTs + 2 * 4 * 32 + 32;
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

// What a launch folds: the rows of [src0 | src1] in blocks of BR (level 0), or BR-row slices of the np x np
// factors of the previous level (combine; per_r slices per factor).
struct FoldInput {
    const float* src0;
    const float* src1;
    int64_t ld0, ld1;
    int nc0, nc1;
    int64_t nrows;
    int combine, per_r, np;
    int nreal;      // columns of the matrix proper, the rest of np is zero padding
};

// Block blk of the input, and the first panel that can be non-zero in it
template <int BR>
__device__ __forceinline__ void block_source_rr(const FoldInput& in, int blk, BlockSource* b, int* p0) {
    if (!in.combine) {
        b->src0 = in.src0; b->ld0 = in.ld0; b->nc0 = in.nc0;
        b->src1 = in.src1; b->ld1 = in.ld1; b->nc1 = in.nc1;
        b->row_first = (int64_t)blk * BR; b->row_limit = in.nrows;
        *p0 = 0;
    } else {
        const int ri = blk / in.per_r, slice = blk - ri * in.per_r;
        b->src0 = in.src0 + (size_t)ri * in.np * in.np; b->ld0 = in.np; b->nc0 = in.np;
        b->src1 = nullptr; b->ld1 = 0; b->nc1 = 0;
        b->row_first = (int64_t)slice * BR; b->row_limit = in.np;
        *p0 = (slice * BR) / kNB;                           // columns left of the slice are zero
    }
}

// The rows of one block behind two buffer descriptors (base addresses in scalar registers, 32-bit lane offsets;
// loads beyond the block's last valid row return zero through the descriptor's range check, and so do the lanes
// of columns that belong to the other source or to neither, whose offsets start beyond every range).
struct BlockLoader {
    __amdgpu_buffer_rsrc_t rs0, rs1;
    unsigned row0, row1;      // bytes per row of either source
    int nc0, nc1;
    static constexpr unsigned kNowhere = 0x80000000u;

    template <int BR>
    __device__ __forceinline__ void open(const BlockSource& b) {
        int64_t rows = b.row_limit - b.row_first;
        rows = rows < 0 ? 0 : (rows > BR ? BR : rows);
        row0 = (unsigned)b.ld0 * 4u;
        row1 = (unsigned)b.ld1 * 4u;
        nc0 = b.nc0;
        nc1 = b.nc1;
        rs0 = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(b.src0 + b.row_first * b.ld0), 0,
                                                (int)(rows * row0), 0x00020000);
        rs1 = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float*>(b.nc1 > 0 ? b.src1 + b.row_first * b.ld1 : b.src0), 0,
            b.nc1 > 0 ? (int)(rows * row1) : 0, 0x00020000);
    }

    // One 32-column tile of the block (all zero unless valid) in the accumulator layout: register q of
    // accumulator mt holds row 32 mt + rho(q) + 4 half, column lane % 32.
    template <int MT>
    __device__ __forceinline__ void load_tile(floatx16 (&t)[MT], int tile, bool valid, int lane) const {
        const int c = lane & 31, half = lane >> 5;
        const int col = tile * kNB + c;
        const bool in0 = valid && col < nc0;
        const bool in1 = valid && col >= nc0 && col < nc0 + nc1;
        const unsigned v0 = in0 ? (unsigned)(4 * half) * row0 + (unsigned)col * 4u : kNowhere;
        const unsigned v1 = in1 ? (unsigned)(4 * half) * row1 + (unsigned)(col - nc0) * 4u : kNowhere;
        const bool any1 = valid && tile * kNB + kNB > nc0 && nc1 > 0;      // wave-uniform
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                const unsigned r = (unsigned)(mt * 32 + rho(q));
                unsigned bits = __builtin_amdgcn_raw_buffer_load_b32(rs0, v0 + r * row0, 0, 0);
                if (any1) bits |= __builtin_amdgcn_raw_buffer_load_b32(rs1, v1 + r * row1, 0, 0);
                t[mt][q] = __builtin_bit_cast(float, bits);
            }
    }
};

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
        lds_barrier();          // T is complete
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

// The barriers inside a block order LDS traffic only: the R factor needs no ordering there, because inside a
// block every element of it is touched by one lane only, and the barrier that ends a block is a full one.
template <int MT>
__device__ __forceinline__ void fold_blocks_rr(float* __restrict__ R, const FoldInput& in, int blk_begin,
                                               int blk_end, float* lds, int np) {
    constexpr int BR = 32 * MT;
    constexpr int RPT = BR / 8;      // rows of a panel column held by one lane during the chain
    constexpr int kTile = (BR * kLdp + 3) & ~3;
    const int NP = np / kNB;
    const int t0 = lds_tiles_rr(np);           // tiles 0 .. t0-1 live in LDS, t0 .. NP-1 in registers
    float* Pb = lds;                           // [2][BR][33] staged panels of register tiles (panel p in p & 1)
    float* Lt = Pb + 2 * kTile;                // [t0][BR][33] the LDS tiles
    float* Gs = Lt + t0 * kTile;               // [32][36] strict upper part of V_B^T V_B
    float* Ts = Gs + 32 * kGs;                 // [32][33] compact-WY T
    float* red = Ts + 32 * kTs;                // [2][32][4] cross-wave partial sums
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

    floatx16 cb[kSlotsRR][MT];       // register tiles of this wave: tiles t0 + wave, + 4, + 8
    // stage a register tile of this wave as panel pp
    auto stage = [&](const floatx16 (&tile)[MT], int pp) {
        float* dst = Pb + (pp & 1) * kTile;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int q = 0; q < 16; ++q) dst[(mt * 32 + rho(q) + 4 * half) * kLdp + j] = tile[mt][q];
    };

    for (int blk = blk_begin; blk < blk_end; ++blk) {
        BlockSource src;
        int p0;
        block_source_rr<BR>(in, blk, &src, &p0);
        BlockLoader loader;
        loader.template open<BR>(src);

        // ---- the block: register tiles of this wave, then its LDS tiles (tile t belongs to wave t % 4)
#pragma unroll
        for (int i = 0; i < kSlotsRR; ++i) {
            const int t = t0 + wave + 4 * i;
            loader.template load_tile<MT>(cb[i], t, t >= p0 && t < NP, lane);
        }
        for (int t = wave; t < t0; t += 4) {
            if (t < p0) continue;
            floatx16 tl[MT];
            loader.template load_tile<MT>(tl, t, true, lane);
            float* dst = Lt + t * kTile;
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
            const bool reg_tile = p >= t0;
            const int ow = (reg_tile ? p - t0 : p) & 3;     // the wave that owns tile p
            float* Vp = reg_tile ? Pb + (p & 1) * kTile : Lt + p * kTile;
            if (p == p0) {
                // the first panel of a block is staged here, the later ones by their owners during the update before
                if (reg_tile && wave == ow) {
#pragma unroll
                    for (int i = 0; i < kSlotsRR; ++i)
                        if (i == ((p - t0) >> 2)) stage(cb[i], p);
                }
                lds_barrier();
            }

            // ================= panel factorisation (the chain of fold_block) =================
            float pv[RPT];
#pragma unroll
            for (int i = 0; i < RPT; ++i) pv[i] = Vp[(RPT * g + i) * kLdp + j];
            panel_chain<RPT, kChainPublish>(pv, rdv, in.nreal - kp, red, Gs, taus, wave, j, g, half);
#pragma unroll
            for (int i = 0; i < RPT; ++i) Vp[(RPT * g + i) * kLdp + j] = pv[i];
            if (g == 0) {
#pragma unroll
                for (int k = 0; k < 32; ++k)
                    if (k <= j) R[(size_t)(kp + k) * np + kp + j] = rdv[k];
            }
            lds_barrier();                      // E1: reflectors in place of the panel; tau and Gram matrix complete
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
                    lds_barrier();                  // E2
                    synced = true;
                }
#pragma unroll
                for (int i = 0; i < kSlotsRR; ++i) {
                    const int ct = t0 + wave + 4 * i;
                    if (ct > p && ct < NP) {
                        update_tile_rr<MT>(cb[i], true, Rrs, rt_lane, (unsigned)(kp * np + ct * kNB) * 4u, np, Vp,
                                           Ts, j, half, synced);
                        if (ct == p + 1) stage(cb[i], ct);     // the next panel
                    }
                }
                for (int ct = wave; ct < t0; ct += 4) {
                    if (ct <= p) continue;
                    float* tile = Lt + ct * kTile;
                    floatx16 tl[MT];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int q = 0; q < 16; ++q) tl[mt][q] = tile[(mt * 32 + rho(q) + 4 * half) * kLdp + j];
                    update_tile_rr<MT>(tl, false, Rrs, rt_lane, (unsigned)(kp * np + ct * kNB) * 4u, np, Vp, Ts,
                                       j, half, synced);
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int q = 0; q < 16; ++q) tile[(mt * 32 + rho(q) + 4 * half) * kLdp + j] = tl[mt][q];
                }
                if (!synced) lds_barrier();         // E2
            }
            lds_barrier();                      // E3: the next panel is staged, this one's reflectors are dead
        }
        __syncthreads();                        // R and the LDS tiles change hands between blocks
    }
}

}  // namespace fold
}  // namespace elm
