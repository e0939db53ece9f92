// Device code of stage 1 (the hidden-matrix build H(Q), step 2 of the paper's Algorithm "S-R-ELM"),
// shared by the plain kernel and by the fused one, which hands every finished tile to the TSQR.
#pragma once

#include "internal.h"
#include "tsqr_fold.h"

namespace elm {
namespace hk {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

// 16-byte load through a buffer descriptor: the base and the wave-uniform byte offset stay in
// scalar registers, only the 32-bit lane offset is a vector register (no 64-bit pointer math).
__device__ __forceinline__ floatx4 buffer_load_x4(__amdgpu_buffer_rsrc_t rsrc, unsigned voff, unsigned soff) {
    const uintx4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, soff, 0);
    return __builtin_bit_cast(floatx4, v);
}

constexpr int kThreads = 256;      // 4 wavefronts, one per SIMD
constexpr int kXPT = 4;            // input values a thread can prefetch per step

struct HiddenArgs {
    const float* X;
    int64_t ldx_n, ldx_q;
    const float* Wp;
    const float* h0;
    const float* c0;
    float* H;
    float* C;
    int64_t N;
    int Q_run, d, L, R, KG, nJB;
    unsigned wp_bytes;
    int ring;              // history slots in the operand row (1; Q-1 for the fully connected multi-lag cell)
    unsigned copy_bytes;   // distance between the per-step rotations of the packed weights (ring > 1)
    // fused form only: the tile [H(Q) | T] is folded into this work-group's R factor instead of being stored
    const float* T;        // N x m targets
    int m, np, ldb;        // np = L + m rounded up to 32, ldb = np + 1
    float* Rout;           // [gridDim.x][np][np]
    int64_t tiles;         // tiles of 32*MS rows; work-group b takes tiles b, b + gridDim.x, ...
};

__device__ __forceinline__ float sigmoid_f(float x) {
    return __builtin_amdgcn_rcpf(1.0f + __expf(-x));
}
__device__ __forceinline__ float tanh_f(float x) {
    return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __expf(2.0f * x));
}
// acc[g][ms] += A(ms) . B(g) over all k-groups.
//   A fragment of k-group kg, tile ms: lane (r = lane&31, half = lane>>5) holds
//     Abuf[(ms*32 + r)*R + kg*8 + half*4 + e], e = 0..3      (one ds_read_b128)
//   B fragment of k-group kg, gate slot g (gate GA + g*GSTEP of GT): lane holds the 4 floats at
//     byte wbase + (kg*GT + GA + g*GSTEP)*1024 + 16*lane
//     = weight row kg*8 + half*4 + e, column (lane&31) of that gate's 32-column block.
//   MFMA step e therefore contracts k-slots {kg*8+e, kg*8+4+e}; every k is covered once.
// Fill all PF slots of the weight-fragment queue with k-groups 0..PF-1 of one contraction.
template <int G, int GT, int GA, int GSTEP, int PF>
__device__ __forceinline__ void prefetch_weights(floatx4 (&bq)[PF][G], __amdgpu_buffer_rsrc_t wrs,
                                                 unsigned wbase, int lane) {
    const unsigned voff = (unsigned)lane * 16u;
    // Drain every older vector-memory access first (s_waitcnt vmcnt(0)): the compiler's wait
    // insertion then sees only these loads as pending inside the contraction loop and emits exact
    // vmcnt(n) waits instead of draining the queue once per trip.
    __builtin_amdgcn_s_waitcnt(0x0F70);
#pragma unroll
    for (int u = 0; u < PF; ++u) {
#pragma unroll
        for (int g = 0; g < G; ++g)
            bq[u][g] = buffer_load_x4(wrs, voff, wbase + (unsigned)(u * GT + GA + g * GSTEP) * 1024u);
        __builtin_amdgcn_sched_barrier(0);      // issue order: oldest slot first
    }
}

// The contraction proper; bq must hold k-groups 0..PF-1 (prefetch_weights).
// PF k-groups of weight fragments are in flight.  Slot u is consumed by the MFMAs of group kg+u
// and refilled, in place, with group kg+u+PF right after them, so every load has PF-1 groups of
// matrix work to hide behind and no register copies are needed at the loop edge.
template <int G, int GT, int GA, int GSTEP, int MS, int PF>
__device__ __forceinline__ void contract_main(floatx16 (&acc)[G][MS], floatx4 (&bq)[PF][G],
                                              const float* __restrict__ Abuf, int R,
                                              __amdgpu_buffer_rsrc_t wrs, unsigned wbase, int KG, int lane) {
    const unsigned voff = (unsigned)lane * 16u;   // wbase: wave-uniform byte offset of this block's fragments
    const float* ap = Abuf + (lane & 31) * R + (lane >> 5) * 4;
    floatx4 a[MS];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms) a[ms] = *reinterpret_cast<const floatx4*>(ap + ms * 32 * R);

    auto group = [&](int k, int u, bool refill) {
        floatx4 an[MS];              // activation fragment of the next group
        const int kn = (k + 1 < KG) ? (k + 1) : k;
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
            an[ms] = *reinterpret_cast<const floatx4*>(ap + ms * 32 * R + kn * 8);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int ms = 0; ms < MS; ++ms)
                    acc[g][ms] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ms][e], bq[u][g][e], acc[g][ms],
                                                                      0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (refill) {
#pragma unroll
            for (int g = 0; g < G; ++g)
                bq[u][g] = buffer_load_x4(wrs, voff, wbase + (unsigned)((k + PF) * GT + GA + g * GSTEP) * 1024u);
        }
#pragma unroll
        for (int ms = 0; ms < MS; ++ms) a[ms] = an[ms];
        __builtin_amdgcn_sched_barrier(0);
    };

    int kg = 0;
    for (; kg + 2 * PF <= KG; kg += PF) {       // branch-free body: PF groups, PF refills
#pragma unroll
        for (int u = 0; u < PF; ++u) group(kg + u, u, true);
    }
    for (; kg + PF <= KG; kg += PF) {           // last full trip: refill only what is still needed
#pragma unroll
        for (int u = 0; u < PF; ++u) group(kg + u, u, kg + u + PF < KG);
    }
#pragma unroll
    for (int u = 0; u < PF - 1; ++u)            // remaining KG % PF groups, nothing left to load
        if (kg + u < KG) group(kg + u, u, false);
}

template <int G, int GT, int GA, int GSTEP, int MS, int PF>
__device__ __forceinline__ void contract(floatx16 (&acc)[G][MS], const float* __restrict__ Abuf,
                                         int R, __amdgpu_buffer_rsrc_t wrs, unsigned wbase, int KG, int lane) {
    floatx4 bq[PF][G];
    prefetch_weights<G, GT, GA, GSTEP, PF>(bq, wrs, wbase, lane);
    contract_main<G, GT, GA, GSTEP, MS, PF>(acc, bq, Abuf, R, wrs, wbase, KG, lane);
}

// STAGE > 0: that many of a lane's pending new-h values (those of the first column chunk) wait in
// spare LDS instead of registers; used by the largest LSTM variants, which otherwise spill.
// WR > 1 (narrow layers, L <= 64, one column chunk): the four waves share 4/WR column blocks and split
// the tile's rows into WR groups of 32*MS instead, so that no wave is idle.
// Variants that fit 256 registers (32-row blocks, one column chunk, or two for the cells with at most
// three gates) are compiled for two waves per SIMD: one wave's gate math overlaps another's matrix work.
// FUSE: the finished tile is not stored; together with its rows of T it becomes the next block of the
// work-group's tall-skinny QR (step 3 of the paper's Algorithm "S-R-ELM" needs H(Q) only through H^+ T).

// The final cell state of a tile (LSTM, for callers that ask for it): element (ms, i) of column chunk ch of
// this lane is row rbase + 32 ms + 8 (i / 4) + 4 (lane / 32) + i % 4, column 32 (4 ch + wcol) + lane % 32.
template <int MS, int NCH>
__device__ __forceinline__ void write_cell_state(float* C, const float* st, int64_t row0, int64_t N, int L, int nJB,
                                                 int wcol, int rbase, int lane) {
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
        const int jb = ch * 4 + wcol;
        const int col = jb * 32 + (lane & 31);
        if (jb < nJB && col < L) {
#pragma unroll
            for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int64_t row = row0 + rbase + ms * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
                    if (row < N) C[row * L + col] = st[(ch * MS + ms) * 16 + i];
                }
        }
    }
}
// The same as a call, for the variants that run one work-group per compute unit: inlined, these rarely
// taken stores (128 addresses of 64 bits) made the compiler spill 67 more registers of the headline variant,
// twelve of them stored in every step of the window loop (30 GB of scratch traffic per launch at full size).
template <int MS, int NCH>
__device__ __noinline__ void write_cell_state_call(float* C, const float* st, int64_t row0, int64_t N, int L,
                                                   int nJB, int wcol, int rbase, int lane) {
    write_cell_state<MS, NCH>(C, st, row0, N, L, nJB, wcol, rbase, lane);
}

// The level-0 fold of a finished tile, as a call: the fold's registers are allocated apart from those of the
// step loop (inlined, the fold's code changed which values of the step loop the compiler spilled, and the
// headline variant lost 4 %).
template <int S>
__device__ __noinline__ void fold_tile(float* R, float* lds, int np, int ldb, int nreal) {
    fold::fold_block<S>(R, lds, np, ldb, 0, nreal);
}
template <int CELL, int MS, int NCH, int STAGE, int WR, bool FUSE>
__device__ __forceinline__ void hidden_tile(const HiddenArgs& p, const int64_t tile, float* lds) {
    static_assert(WR == 1 || NCH == 1, "rows are split over the waves only when one column chunk exists");
    static_assert(!FUSE || WR == 1, "the fused form folds tiles of 32 or 64 rows");
    constexpr int G = (CELL == ELM_CELL_ELMAN) ? 1 : (CELL == ELM_CELL_LSTM) ? 4 : 3;
    constexpr int S = 32 * MS * WR;
    constexpr int PF = 4;
    constexpr bool TWOPASS = (CELL == ELM_CELL_LSTM) && (NCH >= 3);

    const int tid = threadIdx.x, lane = tid & 63;
    // wave-uniform values are forced into scalar registers: weight addresses then live in SGPRs
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wcol = (WR == 1) ? wave : wave % (4 / WR);          // column block of this wave in a chunk
    const int rbase = (WR == 1) ? 0 : (wave / (4 / WR)) * 32 * MS;   // first tile row of this wave
    const int L = p.L, R = p.R, d = p.d, KG = p.KG;
    const int64_t row0 = tile * S;
    const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(p.Wp), 0, (int)p.wp_bytes, 0x00020000);   // raw dword buffer, range-checked
    float* A0 = lds;               // [S][R]: x_t | 1 | h_{t-1} | 0...
    float* A1 = lds + S * R;       // GRU only: x_t | 1 | (r*h_{t-1}) | 0...
    float* stage = lds + S * R + tid;   // STAGE > 0: [STAGE][256] behind the operand, one column per thread

    // accumulator element (ms, i) of this lane: sample row, hidden column inside the block
    const int col_in = lane & 31;
    auto acc_row = [&](int ms, int i) { return rbase + ms * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3); };

    // ---- initial contents of the activation operand
    // The operand row is [x_t | 1 | history | 0...]: one slot of L columns (h_{t-1}) for the lag-1
    // cells; for the fully connected multi-lag cell a ring of p.ring slots, h(t') in slot (t'-1) % ring,
    // read with the weights rotated accordingly (copy t % ring of the packed operand at step t).  The
    // history comes last so that the slots not yet written (all zero) are a tail the contraction skips.
    const int hoff = d + 1;                        // first history column
    for (int idx = tid; idx < S * R; idx += kThreads) {
        const int s = idx / R, k = idx - s * R;
        const int64_t row = row0 + s;
        float v = 0.0f;
        if (k >= hoff && k < hoff + L) {
            if (p.h0 != nullptr && row < p.N) v = p.h0[row * L + (k - hoff)];
        } else if (k == d) {
            v = 1.0f;
        }
        A0[idx] = v;
        if (CELL == ELM_CELL_GRU) A1[idx] = (k == d) ? 1.0f : 0.0f;
    }

    const int nx = S * d;                          // input values per step for this tile
    const bool x_prefetch = nx <= kThreads * kXPT;
    float xr[kXPT];
    auto load_x = [&](int t) {
#pragma unroll
        for (int q = 0; q < kXPT; ++q) {
            const int e = tid + q * kThreads;
            xr[q] = 0.0f;
            if (e < nx) {
                const int s = e / d, dd = e - s * d;
                const int64_t row = row0 + s;
                if (row < p.N) xr[q] = p.X[row * p.ldx_n + (int64_t)t * p.ldx_q + dd];
            }
        }
    };
    auto store_x = [&](float* buf) {
#pragma unroll
        for (int q = 0; q < kXPT; ++q) {
            const int e = tid + q * kThreads;
            if (e < nx) {
                const int s = e / d, dd = e - s * d;
                buf[s * R + dd] = xr[q];
            }
        }
    };
    auto copy_x_direct = [&](int t, float* buf) {     // wide inputs: no register staging
        for (int e = tid; e < nx; e += kThreads) {
            const int s = e / d, dd = e - s * d;
            const int64_t row = row0 + s;
            buf[s * R + dd] =
                (row < p.N) ? p.X[row * p.ldx_n + (int64_t)t * p.ldx_q + dd] : 0.0f;
        }
    };

    // ---- register-resident state
    float st[NCH][MS][16];     // LSTM: cell state c; GRU: this lane's own copy of h; Elman: unused
    float hn[NCH][MS][16];     // LSTM/Elman: new h until the old one is dead; GRU: update gate z
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
        const int jb = ch * 4 + wcol;
        const int col = jb * 32 + col_in;
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float v = 0.0f;
                const int64_t row = row0 + acc_row(ms, i);
                const float* src = (CELL == ELM_CELL_LSTM) ? p.c0 : (CELL == ELM_CELL_GRU) ? p.h0 : nullptr;
                if (src != nullptr && row < p.N && col < L) v = src[row * L + col];
                st[ch][ms][i] = v;
                hn[ch][ms][i] = 0.0f;
            }
    }
    __syncthreads();       // A0/A1 constants written before the x slots are filled
    if (x_prefetch) {
        load_x(0);
        store_x(A0);
        // the GRU's second operand gets x_0 at the top of the first step
    } else {
        copy_x_direct(0, A0);
    }
    __syncthreads();

    floatx4 bq2[6][2];         // weight-fragment queue of the two-pass LSTM path (lives across phases)
    if (TWOPASS && wave < p.nJB)
        prefetch_weights<2, 4, 0, 3, 6>(bq2, wrs, (unsigned)(wave * KG * G) * 1024u, lane);

    int slot = 0;                  // t % ring: weight rotation of this step and slot that receives h(t+1)
    for (int t = 0; t < p.Q_run; ++t) {
        if (CELL == ELM_CELL_GRU) {
            if (x_prefetch) store_x(A1); else copy_x_direct(t, A1);
        }
        const bool more = (t + 1 < p.Q_run);
        const unsigned wrot = (unsigned)slot * p.copy_bytes;
        // k-groups that can be non-zero at this step: the input columns and the history slots written so far
        const int KGt = (p.ring > 1) ? min(KG, (hoff + min(t, p.ring) * L + 7) >> 3) : KG;
        if (x_prefetch && more) load_x(t + 1);

        if (CELL != ELM_CELL_GRU) {
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                const int jb = ch * 4 + wcol;
                if (jb < p.nJB) {
                    const unsigned wbase = (unsigned)(jb * KG * G) * 1024u + wrot;
                    if (TWOPASS) {
                        // LSTM with many column chunks: two contractions of two gates each keep the
                        // accumulators at 64 registers so that c and the pending h stay in registers
                        floatx16 acc[2][MS];
                        float ig_gg[MS][16];
#pragma unroll
                        for (int g = 0; g < 2; ++g)
#pragma unroll
                            for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                                for (int i = 0; i < 16; ++i) acc[g][ms][i] = 0.0f;
                        // the weight queue of each contraction is filled one phase early (before the
                        // point-wise work of the previous contraction), so the first MFMA never waits
                        const int jn = ((ch + 1 < NCH) && ((ch + 1) * 4 + wave < p.nJB)) ? jb + 4 : wave;
                        contract_main<2, 4, 0, 3, MS, 6>(acc, bq2, A0 + rbase * R, R, wrs, wbase, KGt, lane);   // gates i, g
                        prefetch_weights<2, 4, 1, 1, 6>(bq2, wrs, wbase, lane);
#pragma unroll
                        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                            for (int i = 0; i < 16; ++i) {
                                ig_gg[ms][i] = sigmoid_f(acc[0][ms][i]) * tanh_f(acc[1][ms][i]);
                                acc[0][ms][i] = 0.0f;
                                acc[1][ms][i] = 0.0f;
                            }
                        contract_main<2, 4, 1, 1, MS, 6>(acc, bq2, A0 + rbase * R, R, wrs, wbase, KGt, lane);   // gates f, o
                        prefetch_weights<2, 4, 0, 3, 6>(bq2, wrs, (unsigned)(jn * KG * G) * 1024u, lane);
#pragma unroll
                        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                            for (int i = 0; i < 16; ++i) {
                                const float c = sigmoid_f(acc[0][ms][i]) * st[ch][ms][i] + ig_gg[ms][i];
                                st[ch][ms][i] = c;
                                const float hv = sigmoid_f(acc[1][ms][i]) * tanh_f(c);
                                if (ch == 0 && ms * 16 + i < STAGE) stage[(ms * 16 + i) * kThreads] = hv;
                                else hn[ch][ms][i] = hv;
                            }
                    } else {
                        floatx16 acc[G][MS];
#pragma unroll
                        for (int g = 0; g < G; ++g)
#pragma unroll
                            for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                                for (int i = 0; i < 16; ++i) acc[g][ms][i] = 0.0f;
                        contract<G, G, 0, 1, MS, PF>(acc, A0 + rbase * R, R, wrs, wbase, KGt, lane);
#pragma unroll
                        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                            for (int i = 0; i < 16; ++i) {
                                if (CELL == ELM_CELL_ELMAN) {
                                    hn[ch][ms][i] = tanh_f(acc[0][ms][i]);
                                } else {
                                    const float ig = sigmoid_f(acc[0][ms][i]);
                                    const float fg = sigmoid_f(acc[G > 1 ? 1 : 0][ms][i]);
                                    const float og = sigmoid_f(acc[G > 2 ? 2 : 0][ms][i]);
                                    const float gg = tanh_f(acc[G > 3 ? 3 : 0][ms][i]);
                                    const float c = fg * st[ch][ms][i] + ig * gg;
                                    st[ch][ms][i] = c;
                                    hn[ch][ms][i] = og * tanh_f(c);
                                }
                            }
                    }
                }
            }
            __syncthreads();          // every wave has finished reading h_{t-1}
            {
                // lane base address, made opaque per step so that the 32*NCH store addresses are
                // recomputed here (scalar row offsets) instead of being kept live across the unroll
                int lane_base = (rbase + 4 * (lane >> 5)) * R + hoff + col_in;
                asm volatile("" : "+v"(lane_base));
#pragma unroll
                for (int ch = 0; ch < NCH; ++ch) {
                    const int jb = ch * 4 + wcol;
                    const int col = jb * 32 + col_in;
                    if (jb < p.nJB && col < L) {
                        float* dst = A0 + lane_base + slot * L + jb * 32;
#pragma unroll
                        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                            for (int i = 0; i < 16; ++i)
                                dst[(ms * 32 + 8 * (i >> 2) + (i & 3)) * R] =
                                    (ch == 0 && ms * 16 + i < STAGE) ? stage[(ms * 16 + i) * kThreads]
                                                                     : hn[ch][ms][i];
                    }
                }
            }
            if (more) {
                if (x_prefetch) store_x(A0); else copy_x_direct(t + 1, A0);
                slot = (slot + 1 == p.ring) ? 0 : slot + 1;
            }
            __syncthreads();
        } else {
            // phase 1: update and reset gates from h_{t-1}; stage r*h_{t-1} as the second operand
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                const int jb = ch * 4 + wcol;
                const int col = jb * 32 + col_in;
                if (jb < p.nJB) {
                    floatx16 acc[2][MS];
#pragma unroll
                    for (int g = 0; g < 2; ++g)
#pragma unroll
                        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                            for (int i = 0; i < 16; ++i) acc[g][ms][i] = 0.0f;
                    contract<2, 3, 0, 1, MS, 4>(acc, A0 + rbase * R, R, wrs, (unsigned)(jb * KG * 3) * 1024u, KG, lane);
#pragma unroll
                    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            hn[ch][ms][i] = sigmoid_f(acc[0][ms][i]);
                            const float r = sigmoid_f(acc[1][ms][i]);
                            if (col < L) A1[acc_row(ms, i) * R + hoff + col] = r * st[ch][ms][i];
                        }
                }
            }
            __syncthreads();
            // phase 2: candidate from r*h_{t-1}; blend; publish h_t into the first operand
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                const int jb = ch * 4 + wcol;
                const int col = jb * 32 + col_in;
                if (jb < p.nJB) {
                    floatx16 acc[1][MS];
#pragma unroll
                    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc[0][ms][i] = 0.0f;
                    contract<1, 3, 2, 1, MS, 4>(acc, A1 + rbase * R, R, wrs, (unsigned)(jb * KG * 3) * 1024u, KG, lane);
#pragma unroll
                    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            const float z = hn[ch][ms][i];
                            const float hv = (1.0f - z) * st[ch][ms][i] + z * tanh_f(acc[0][ms][i]);
                            st[ch][ms][i] = hv;
                            if (col < L) A0[acc_row(ms, i) * R + hoff + col] = hv;
                        }
                }
            }
            if (more) {
                if (x_prefetch) store_x(A0); else copy_x_direct(t + 1, A0);
            }
            __syncthreads();
        }
    }

    if constexpr (FUSE) {
        // ---- the tile [H(Q) | T | 0] replaces the operand in LDS (row stride ldb) and is folded into R.
        // The two layouts overlap, so the values pass through registers; rows past N are zero.
        // wave w moves rows w, w + 4, ...; a lane moves columns lane, lane + 64, ... (L <= 512)
        const int np = p.np, ldb = p.ldb;
        float hv[S / 4][8];
#pragma unroll
        for (int r = 0; r < S / 4; ++r) {
            const int s = 4 * r + wave;
            const bool live = row0 + s < p.N;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int j = lane + 64 * e;
                hv[r][e] = (live && j < L) ? A0[s * R + hoff + j] : 0.0f;
            }
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < S / 4; ++r) {
            const int s = 4 * r + wave;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int j = lane + 64 * e;
                if (j < L) lds[s * ldb + j] = hv[r][e];
            }
        }
        const int extra = np - L;                      // targets, then zero padding
        for (int idx = tid; idx < S * extra; idx += kThreads) {
            const int s = idx / extra, c = idx - s * extra;
            const int64_t row = row0 + s;
            lds[s * ldb + L + c] = (c < p.m && row < p.N) ? p.T[row * p.m + c] : 0.0f;
        }
        __syncthreads();
        // (the variants that share a compute unit between two work-groups keep the fold inline: a call would
        // be compiled for the full register file and halve their occupancy)
        constexpr bool kTwoPerUnit = MS == 1 && (NCH == 1 || (NCH == 2 && CELL != ELM_CELL_LSTM));
        if constexpr (kTwoPerUnit)
            fold::fold_block<S>(p.Rout + (size_t)blockIdx.x * np * np, lds, np, ldb, 0, L + p.m);
        else
            fold_tile<S>(p.Rout + (size_t)blockIdx.x * np * np, lds, np, ldb, L + p.m);
        return;
    }

    // ---- H(Q): the h part of the operand, written row by row (coalesced)
    for (int idx = tid; idx < S * L; idx += kThreads) {
        const int s = idx / L, j = idx - s * L;
        const int64_t row = row0 + s;
        if (row < p.N) p.H[row * L + j] = A0[s * R + hoff + slot * L + j];
    }
    if (CELL == ELM_CELL_LSTM && p.C != nullptr) {
        constexpr bool kTwoPerUnit = MS == 1 && (NCH == 1 || (NCH == 2 && CELL != ELM_CELL_LSTM));
        if constexpr (kTwoPerUnit) {
            write_cell_state<MS, NCH>(p.C, &st[0][0][0], row0, p.N, L, p.nJB, wcol, rbase, lane);
        } else {
            // a copy, so that the state itself never has an address and stays in registers
            float tmp[NCH * MS * 16];
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch)
#pragma unroll
                for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                    for (int i = 0; i < 16; ++i) tmp[(ch * MS + ms) * 16 + i] = st[ch][ms][i];
            write_cell_state_call<MS, NCH>(p.C, tmp, row0, p.N, L, p.nJB, wcol, rbase, lane);
        }
    }
}

template <int CELL, int MS, int NCH, int STAGE, int WR>
__global__ __launch_bounds__(kThreads, (MS == 1 && (NCH == 1 || (NCH == 2 && CELL != ELM_CELL_LSTM))) ? 2 : 1)
void hidden_kernel(const HiddenArgs p) {
    extern __shared__ __align__(16) float lds[];
    hidden_tile<CELL, MS, NCH, STAGE, WR, false>(p, blockIdx.x, lds);
}

}  // namespace hk
}  // namespace elm
