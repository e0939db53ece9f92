// Stage 1 for the paper's fully connected multi-lag cell (section "Fully Connected RNN", Eq. hij_fc)
// when the history of a window does not fit LDS: one launch per step over all rows.
//
//   h(t) = tanh( [h(1) | h(2) | ... | h(t-1) | x_t | 1] . [A_{t-1}; A_{t-2}; ...; A_1; W; b] )
//
// The states of a pass of rows are kept in time order in a device buffer ([slot][row][Lk], one slot of
// Lk = L rounded up to 8 columns per step: a tile's rows of a slot are contiguous in memory), so the
// operand of step t is the first t-1 slots followed by the input, and its weights are a suffix of one
// stack [A_{Q-1}; ...; A_1; W; b]: nothing is shifted or rotated, every step is a plain
// (rows x K_t) . (K_t x L) contraction with K_t growing by Lk per step.  A work-group streams its rows
// of the operand through LDS in chunks of 64 columns (double-buffered, global loads one chunk ahead in
// registers); every wave owns a 32-column block of the output and reads its weight fragments straight
// from L2 in a pre-packed order, eight k-groups ahead.  The history is read once per step ((t-1)*Lk*4
// bytes per row against 2*(t-1)*Lk*L flops), or once per block of steps for layers of at most 64 units.
// Passes of few rows (long windows) split each contraction over slices of the operand (gridDim.z).
//
// The paper's kernel keeps the history of one (sample, neuron) pair per thread (its H_loc) and so
// re-reads every other neuron's past outputs from global memory per thread; here a step is one
// matrix-core contraction shared by the tile.

#include "hidden_kernel.h"

namespace elm {
namespace {

using namespace hk;

constexpr int kBK = 64;            // operand columns per LDS chunk (8 k-groups)
constexpr int kRS = kBK + 4;       // LDS row stride in floats (conflict-free 16-byte reads)
constexpr int kPF = 8;             // weight k-groups in flight per wave = one chunk

struct FcStepArgs {
    const float* hist;     // [slot][row][Lk]: slot s holds h(s+1) of this pass's rows
    unsigned slot_floats;  // distance between slots: rows of a full pass * Lk
    unsigned hist_bytes;   // ring * slot_floats * 4 (below 2^31)
    int Lk;
    const float* X;        // x_t of the chunk's first row
    int64_t ldx_n;
    const float* Wp;       // packed weight stack
    unsigned wp_bytes;
    unsigned kg0;          // first k-group of this step's weights inside a column block
    unsigned jb_stride;    // bytes between the column blocks of the packed stack
    int nchunks;           // chunks of kBK operand columns
    int Kh;                // history columns of this step, (t-1)*Lk
    int d, L, nJB;
    int rows;
    float* out;            // history slot t-1 (ldo = Lk) or H (ldo = L)
    int64_t ldo;
    int ncols;             // columns stored per row; those at or beyond L are zeros
    // Layers of one or two column blocks take the steps in blocks of nsteps = 4 / nJB: one launch
    // contracts the finished slots for all steps of the block at once (wave w: step w / nJB of the block,
    // column block w % nJB; the weights of consecutive steps start one slot apart in the stack) and stores
    // the raw sums; the launch of each step then starts from its sums and adds the block's own slots.
    int block;             // 1: the block launch (no input columns, raw sums out, [row][step][32 nJB])
    int nsteps;            // steps it covers (1 otherwise)
    unsigned slot_groups;  // k-groups per slot, Lk / 8
    const float* acc_in;   // sums the accumulators start from (row stride ldacc), or null
    int64_t ldacc;
    // Launches of few rows split the contraction over gridDim.z slices of the operand chunks; slice z
    // stores its raw sums at out + z * zstride and a second launch adds the slices and applies tanh.
    int raw;               // 1: raw sums out (the split form)
    int64_t zstride;
    // fc_rows_kernel: the stack packed per 16-column unit; the kernel runs the steps t_first .. t_last of a pass
    // itself (a tile's rows depend on no other tile) and derives Kh, kg0, nchunks, X and out per step
    const float* Wp16;
    unsigned wp16_bytes;
    int t_first, t_last, Q_run, ring;
    int64_t ldx_q;         // X: x_1 of the pass's first row
    float* hist_out;       // = hist (written)
    float* H;              // the pass's rows of H (row stride L)
};

// ---- the operand [h(1) | ... | h(t-1) | x_t | 1 | 0 ...] of a tile, streamed in chunks of kBK columns.
// A thread moves NLD 16-byte pieces per chunk: row (tid>>4) + 16*q of the tile, columns 4*(tid&15) .. +3.

// byte offset of the thread's rows inside a slot; rows past the end get an offset that is out of range
template <int NLD>
__device__ __forceinline__ void operand_row_offsets(unsigned (&hoff)[NLD], const FcStepArgs& p, int64_t row0, int lr) {
#pragma unroll
    for (int q = 0; q < NLD; ++q) {
        const int64_t row = row0 + lr + 16 * q;
        hoff[q] = row < p.rows ? (unsigned)(row * p.Lk * 4) : 0xFFFFFFF0u;
    }
}

// operand column k lies in slot k / Lk; Lk and k are multiples of 4, so a piece stays inside a slot
__device__ __forceinline__ unsigned operand_slot_offset(const FcStepArgs& p, int k) {
    const int sl = k / p.Lk;
    return ((unsigned)sl * p.slot_floats + (unsigned)(k - sl * p.Lk)) * 4u;
}

// a chunk that lies inside the history: range-checked loads, rows past the end read as zero
template <int NLD>
__device__ __forceinline__ void operand_load_history(floatx4 (&stage)[NLD], const unsigned (&hoff)[NLD],
                                                     __amdgpu_buffer_rsrc_t hrs, unsigned so) {
#pragma unroll
    for (int q = 0; q < NLD; ++q) {
        const unsigned off = hoff[q] == 0xFFFFFFF0u ? hoff[q] : hoff[q] + so;
        stage[q] = buffer_load_x4(hrs, off, 0);
    }
}

// the same with the offsets rebuilt from the first piece's (rows 16 apart): eight fewer live registers
template <int NLD>
__device__ __forceinline__ void operand_load_history_strided(floatx4 (&stage)[NLD], unsigned hoff0, unsigned step,
                                                             int valid, __amdgpu_buffer_rsrc_t hrs, unsigned so) {
#pragma unroll
    for (int q = 0; q < NLD; ++q)      // pieces q >= valid belong to rows past the end: out of range, read as zero
        stage[q] = buffer_load_x4(hrs, q < valid ? hoff0 + (unsigned)q * step + so : 0xFFFFFFF0u, 0);
}

// a chunk that holds the end of the history, x_t, the constant 1 and the zero padding (no input columns
// when the launch only pre-sums finished slots)
template <int NLD>
__device__ __forceinline__ void operand_load_edge(floatx4 (&stage)[NLD], const unsigned (&hoff)[NLD],
                                                  __amdgpu_buffer_rsrc_t hrs, const FcStepArgs& p, int Kh,
                                                  const float* X, int64_t row0, int lr, int k, bool with_input) {
    const unsigned so = k < Kh ? operand_slot_offset(p, k) : 0u;
#pragma unroll
    for (int q = 0; q < NLD; ++q) {
        const int64_t row = row0 + lr + 16 * q;
        floatx4 v = {0.0f, 0.0f, 0.0f, 0.0f};
        if (row < p.rows) {
            if (k < Kh) {                  // Kh and k are multiples of 4: a piece never straddles the edge
                v = buffer_load_x4(hrs, hoff[q] + so, 0);
            } else if (with_input) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int kk = k + e - Kh;
                    v[e] = kk < p.d ? X[row * p.ldx_n + kk] : (kk == p.d ? 1.0f : 0.0f);
                }
            }
        }
        stage[q] = v;
    }
}

// MS 32-row blocks per wave, CW column blocks per work-group (the other 4/CW waves take further rows);
// EXT: the launch may be a block launch or start from carried sums (layers of at most 64 units only: the
// plain form keeps its registers for four work-groups per compute unit)
template <int MS, int CW, bool EXT>
__global__ __launch_bounds__(kThreads, 2) void fc_step_kernel(const FcStepArgs p) {
    const bool block = EXT && p.block != 0;
    const bool raw = EXT && (p.block != 0 || p.raw != 0);
    // this work-group's slice [c0, c1) of the operand chunks
    const int zs = EXT ? (int)blockIdx.z : 0, nz = EXT ? (int)gridDim.z : 1;
    const int c0 = (int)((int64_t)p.nchunks * zs / nz), c1 = (int)((int64_t)p.nchunks * (zs + 1) / nz);
    constexpr int WR = 4 / CW, S = 32 * MS * WR, NLD = S / 16;
    extern __shared__ float lds[];             // [2][S][kRS]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wcol = wave % CW, rbase = (wave / CW) * 32 * MS;
    const int unit = (int)blockIdx.y * CW + wcol;
    const int jstep = block ? unit / p.nJB : 0;            // step of the block (block launch only)
    const int jb = unit - jstep * p.nJB;
    const bool active = unit < p.nJB * p.nsteps;   // the last group of column blocks may be short
    const int64_t row0 = (int64_t)blockIdx.x * S;
    const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(p.Wp), 0, (int)p.wp_bytes, 0x00020000);   // raw dword buffer, range-checked
    const unsigned wbase = active ? (unsigned)jb * p.jb_stride + (p.kg0 - (unsigned)jstep * p.slot_groups) * 1024u
                                  : p.kg0 * 1024u;
    const unsigned voff = (unsigned)lane * 16u;

    // this thread's NLD 16-byte pieces of a chunk: row (tid>>4) + 16*q, columns 4*(tid&15) .. +3
    const int lr = tid >> 4, lk = (tid & 15) * 4;
    const __amdgpu_buffer_rsrc_t hrs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(p.hist), 0, (int)p.hist_bytes, 0x00020000);
    unsigned hoff[NLD];
    operand_row_offsets<NLD>(hoff, p, row0, lr);
    floatx4 stage[NLD];
    auto load_history = [&](int c) {
        operand_load_history<NLD>(stage, hoff, hrs, operand_slot_offset(p, c * kBK + lk));
    };
    auto load_edge = [&](int c) {
        operand_load_edge<NLD>(stage, hoff, hrs, p, p.Kh, p.X, row0, lr, c * kBK + lk, !block);
    };
    auto store_chunk = [&](float* buf) {
#pragma unroll
        for (int q = 0; q < NLD; ++q)
            *reinterpret_cast<floatx4*>(buf + (lr + 16 * q) * kRS + lk) = stage[q];
    };

    floatx16 acc[MS];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int64_t row = row0 + rbase + ms * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
            acc[ms][i] = (EXT && p.acc_in != nullptr && active && row < p.rows)
                             ? p.acc_in[row * p.ldacc + jb * 32 + (lane & 31)] : 0.0f;
        }

    floatx4 bq[kPF];
#pragma unroll
    for (int u = 0; u < kPF; ++u) bq[u] = buffer_load_x4(wrs, voff, wbase + (unsigned)(c0 * kPF + u) * 1024u);

    // the kPF k-groups of chunk c; every weight slot is refilled with the group one chunk ahead (the
    // stack ends in zero groups, so the look-ahead past the last chunk needs no test)
    auto compute = [&](int c) {
        const float* ap = lds + ((c - c0) & 1) * S * kRS + (rbase + (lane & 31)) * kRS + (lane >> 5) * 4;
        const unsigned wnext = wbase + (unsigned)(c * kPF + kPF) * 1024u;
        floatx4 a[MS];
#pragma unroll
        for (int ms = 0; ms < MS; ++ms) a[ms] = *reinterpret_cast<const floatx4*>(ap + ms * 32 * kRS);
#pragma unroll
        for (int u = 0; u < kPF; ++u) {
            floatx4 an[MS];                         // operand fragment of the next group, read under the MFMAs
#pragma unroll
            for (int ms = 0; ms < MS; ++ms)
                an[ms] = *reinterpret_cast<const floatx4*>(ap + ms * 32 * kRS + (u + 1 < kPF ? u + 1 : u) * 8);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int ms = 0; ms < MS; ++ms)
                    acc[ms] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ms][e], bq[u][e], acc[ms], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);      // the refill is issued here, not at the end of the chunk
            bq[u] = buffer_load_x4(wrs, voff, wnext + (unsigned)u * 1024u);
#pragma unroll
            for (int ms = 0; ms < MS; ++ms) a[ms] = an[ms];
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    const int nfull = p.Kh / kBK;              // chunks that lie inside the history
    if (c0 < nfull) load_history(c0); else load_edge(c0);
    store_chunk(lds);
    __syncthreads();
    int c = c0;
    for (; c + 1 < nfull && c + 1 < c1; ++c) { // chunk c + 1 is fetched while chunk c is contracted
        load_history(c + 1);
        __builtin_amdgcn_sched_barrier(0);          // the operand loads have the whole chunk to arrive
        compute(c);
        store_chunk(lds + ((c + 1 - c0) & 1) * S * kRS);
        __syncthreads();
    }
    for (; c < c1; ++c) {
        const bool more = c + 1 < c1;
        if (more) load_edge(c + 1);
        __builtin_amdgcn_sched_barrier(0);
        compute(c);
        if (more) store_chunk(lds + ((c + 1 - c0) & 1) * S * kRS);
        __syncthreads();
    }

    if (!active) return;
    const int col = jb * 32 + (lane & 31);
    if (raw) {                                 // raw sums (of step jstep of a block), all 32 columns of the block
        float* o = p.out + (int64_t)zs * p.zstride + jstep * 32 * p.nJB + col;
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int64_t row = row0 + rbase + ms * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
                if (row < p.rows) o[row * p.ldo] = acc[ms][i];
            }
        return;
    }
    if (col >= p.ncols) return;
    const bool real = col < p.L;
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int64_t row = row0 + rbase + ms * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
            if (row < p.rows) p.out[row * p.ldo + col] = real ? tanh_f(acc[ms][i]) : 0.0f;
        }
}

typedef float floatx2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ floatx2 buffer_load_x2(__amdgpu_buffer_rsrc_t rsrc, unsigned voff, unsigned soff) {
    typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
    const uintx2 v = __builtin_amdgcn_raw_buffer_load_b64(rsrc, voff, soff, 0);
    return __builtin_bit_cast(floatx2, v);
}

// Layers of 65 to 96 units: three 32-column blocks would leave one wave in four idle.  Here the four
// waves split the rows of a 128-row tile instead and every wave contracts all NU = ceil(L / 16) column
// units for its 32 rows with the 16x16x4 matrix instruction: no idle wave, 16-column granularity.  The
// kernel also runs all steps of a pass itself (a tile's rows depend on no other tile), with a
// work-group-scope fence and a barrier between steps.  Lane (r = lane % 16, q = lane / 16) of an A fragment holds row r, columns
// 8g + 2q + e of k-group g; of a B fragment stack rows 8g + 2q + e, column r of the unit (e = 0, 1: one
// 8-byte load each); accumulator register v of a lane is row 4q + v, column r of the 16 x 16 tile.
// Four k-groups of weight fragments are in flight; the operand loads of the next chunk are issued in
// the middle of a chunk, after the refills this chunk still waits for and before those of the next one,
// so no wait for a weight fragment ever waits for an operand load.
template <int NU>
__global__ __launch_bounds__(kThreads, 2) void fc_rows_kernel(const FcStepArgs args) {
    constexpr int S = 128, NLD = S / 16, PF = 4;
    extern __shared__ float lds[];             // [2][S][kRS]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rbase = wave * 32;
    const int64_t row0 = (int64_t)blockIdx.x * S;
    const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(args.Wp16), 0, (int)args.wp16_bytes, 0x00020000);
    const unsigned voff = (unsigned)lane * 8u;
    const int lr = tid >> 4, lk = (tid & 15) * 4;
    const __amdgpu_buffer_rsrc_t hrs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(args.hist), 0, (int)args.hist_bytes, 0x00020000);
    // rows of this thread's pieces: row0 + lr + 16 q; `valid` of them exist
    const unsigned hoff0 = (unsigned)((row0 + lr) * args.Lk * 4), hstep = (unsigned)(16 * args.Lk * 4);
    const int64_t left = args.rows - (row0 + lr);
    const int valid = left <= 0 ? 0 : (int)((left + 15) / 16 < NLD ? (left + 15) / 16 : NLD);

    for (int t = args.t_first; t <= args.t_last; ++t) {
        // this step's view of the operand and its weights
        const int Kh = (t - 1) * args.Lk;
        const unsigned kg0 = (unsigned)((args.ring - (t - 1)) * (int)args.slot_groups);
        const int nchunks = ((Kh + args.d + 1 + 7) / 8 + 7) / 8;
        const float* Xt = args.X + (int64_t)(t - 1) * args.ldx_q;
        const bool last = t == args.Q_run;
        float* out = last ? args.H : args.hist_out + (int64_t)(t - 1) * args.slot_floats;
        const int64_t ldo = last ? args.L : args.Lk;
        const int ncols = last ? args.L : args.Lk;
        const unsigned wbase = kg0 * (NU * 512u);      // fragments: [k-group][unit][lane][2], 512 bytes each

        floatx4 stage[NLD];
        const int nfull = Kh / kBK;            // chunks that lie inside the history
        auto load_history = [&](int c) {
            operand_load_history_strided<NLD>(stage, hoff0, hstep, valid, hrs,
                                              operand_slot_offset(args, c * kBK + lk));
        };
        auto load_edge = [&](int c) {
            unsigned hoff[NLD];
#pragma unroll
            for (int q = 0; q < NLD; ++q) hoff[q] = hoff0 + (unsigned)q * hstep;     // used for existing rows only
            operand_load_edge<NLD>(stage, hoff, hrs, args, Kh, Xt, row0, lr, c * kBK + lk, true);
        };
        auto store_chunk = [&](float* buf) {
#pragma unroll
            for (int q = 0; q < NLD; ++q)
                *reinterpret_cast<floatx4*>(buf + (lr + 16 * q) * kRS + lk) = stage[q];
        };

        floatx4 acc[2][NU];
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int cu = 0; cu < NU; ++cu) acc[r][cu] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};

        floatx2 bq[PF][NU];
#pragma unroll
        for (int u = 0; u < PF; ++u)
#pragma unroll
            for (int cu = 0; cu < NU; ++cu)
                bq[u][cu] = buffer_load_x2(wrs, voff + (unsigned)cu * 512u, wbase + (unsigned)u * (NU * 512u));

        // k-groups 4h .. 4h+3 of chunk c; slot u is refilled with the group four ahead
        auto half = [&](int c, int h) {
            const float* ap = lds + (c & 1) * S * kRS + (rbase + (lane & 15)) * kRS + (lane >> 4) * 2 + h * 32;
            const unsigned wnext = wbase + (unsigned)(c * 8 + h * 4 + PF) * (NU * 512u);
            floatx2 a0 = *reinterpret_cast<const floatx2*>(ap), a1 = *reinterpret_cast<const floatx2*>(ap + 16 * kRS);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int un = u + 1 < 4 ? u + 1 : u;
                const floatx2 n0 = *reinterpret_cast<const floatx2*>(ap + un * 8);
                const floatx2 n1 = *reinterpret_cast<const floatx2*>(ap + 16 * kRS + un * 8);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int e = 0; e < 2; ++e)
#pragma unroll
                    for (int cu = 0; cu < NU; ++cu) {
                        acc[0][cu] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0[e], bq[u][cu][e], acc[0][cu], 0, 0, 0);
                        acc[1][cu] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1[e], bq[u][cu][e], acc[1][cu], 0, 0, 0);
                    }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int cu = 0; cu < NU; ++cu)
                    bq[u][cu] = buffer_load_x2(wrs, voff + (unsigned)cu * 512u, wnext + (unsigned)u * (NU * 512u));
                a0 = n0;
                a1 = n1;
                __builtin_amdgcn_sched_barrier(0);
            }
        };

        if (nfull > 0) load_history(0); else load_edge(0);
        store_chunk(lds);
        __syncthreads();
        int c = 0;
        for (; c + 1 < nfull; ++c) {           // branch-free body: the waits for weight fragments stay exact
            half(c, 0);
            load_history(c + 1);
            __builtin_amdgcn_sched_barrier(0);
            half(c, 1);
            store_chunk(lds + ((c + 1) & 1) * S * kRS);
            __syncthreads();
        }
        for (; c < nchunks; ++c) {
            const bool more = c + 1 < nchunks;
            half(c, 0);
            if (more) load_edge(c + 1);
            __builtin_amdgcn_sched_barrier(0);
            half(c, 1);
            if (more) store_chunk(lds + ((c + 1) & 1) * S * kRS);
            __syncthreads();
        }

#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int cu = 0; cu < NU; ++cu) {
                const int col = 16 * cu + (lane & 15);
                if (col >= ncols) continue;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int64_t row = row0 + rbase + 16 * r + 4 * (lane >> 4) + v;
                    if (row < args.rows) out[row * ldo + col] = col < args.L ? tanh_f(acc[r][cu][v]) : 0.0f;
                }
            }
        // the next step reads the slot this one wrote: the tile's rows are this work-group's alone (tiles of
        // 128 rows are whole cache lines of a slot), so a fence of work-group scope is enough (a device-scope
        // one writes back and invalidates the whole L2 of the die: measured 213 ms against 176 ms per fit)
        if (t < args.t_last) {
            __threadfence_block();
            __syncthreads();
        }
    }
}

template <int NU>
hipError_t launch_rows(const FcStepArgs& a, hipStream_t stream) {
    constexpr size_t lds = (size_t)2 * 128 * kRS * sizeof(float);
    auto kern = fc_rows_kernel<NU>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)((a.rows + 127) / 128)), dim3(kThreads), lds, stream, a);
    return hipGetLastError();
}

// h = tanh(sum of the nz slices' raw sums), zeros in the padding columns; the slices are added in order
__global__ __launch_bounds__(256) void fc_reduce_kernel(const float* __restrict__ part, int nz, int64_t zstride,
                                                        int ldp, int rows, int L, int ncols,
                                                        float* __restrict__ out, int64_t ldo) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)rows * ncols) return;
    const int row = (int)(idx / ncols), col = (int)(idx - (int64_t)row * ncols);
    float s = 0.0f;
    for (int z = 0; z < nz; ++z) s += part[z * zstride + (int64_t)row * ldp + col];
    out[row * ldo + col] = col < L ? tanh_f(s) : 0.0f;
}

template <int MS, int CW, bool EXT = false>
hipError_t launch_step(const FcStepArgs& a, int ycount, hipStream_t stream, int slices = 1) {
    constexpr int S = 32 * MS * (4 / CW);
    constexpr size_t lds = (size_t)2 * S * kRS * sizeof(float);
    auto kern = fc_step_kernel<MS, CW, EXT>;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    const unsigned tiles = (unsigned)((a.rows + S - 1) / S);
    hipLaunchKernelGGL(kern, dim3(tiles, (unsigned)ycount, (unsigned)(EXT ? slices : 1)), dim3(kThreads), lds,
                       stream, a);
    return hipGetLastError();
}

}  // namespace

bool fc_step_layout(int Q, int d, int L, FcStepLayout* out) {
    FcStepLayout lay{};
    lay.Q = Q; lay.d = d; lay.L = L;
    lay.ring = Q > 1 ? Q - 1 : 1;
    lay.Lk = (L + 7) / 8 * 8;
    lay.nJB = (L + 31) / 32;
    const int64_t Kall = (int64_t)lay.ring * lay.Lk + d + 1;
    const int64_t KGtot = (Kall + 7) / 8;
    // a step runs whole chunks of kPF groups and looks kPF groups ahead: both land in the zero tail
    const int64_t KGpad = KGtot + 2 * kPF;
    const int64_t bytes = (int64_t)lay.nJB * KGpad * 1024;
    const int64_t row_bytes = (int64_t)lay.ring * lay.Lk * (int64_t)sizeof(float);
    // 256 rows of history must stay below 2^31 bytes (32-bit offsets into a range-checked buffer)
    if (bytes >= ((int64_t)1 << 32) || row_bytes >= ((int64_t)8 << 20)) return false;
    lay.KGtot = (int)KGtot;
    lay.KGpad = (int)KGpad;
    lay.floats = (size_t)bytes / sizeof(float);
    int64_t rows = ((((int64_t)2 << 30) - 1) / row_bytes) / 256 * 256;      // the buffer stays below 2^31 bytes
    // 65,536 rows are two full rounds of 64-row work-groups at two per compute unit; larger passes measured
    // slower (100,096 rows: three rounds and a fraction), and so did 49,152 (one and a half)
    lay.chunk_rows = rows < 256 ? 256 : rows > 65536 ? 65536 : rows;
    // 97 to 112 units would take 7 units: measured 1.6 % faster than four 32-column blocks, with 22 registers
    // spilled; those layers keep the 32-column kernel
    lay.NU = (L > 64 && L <= 96) ? (L + 15) / 16 : 0;
    lay.floats16 = (size_t)lay.NU * KGpad * 128;
    if (out != nullptr) *out = lay;
    return true;
}

FcScratch fc_scratch(const FcStepLayout& lay, int64_t N) {
    FcScratch sc{};
    const int64_t n256 = (N + 255) / 256 * 256;
    sc.pass_rows = n256 < lay.chunk_rows ? n256 : lay.chunk_rows;
    sc.hist_floats = (size_t)sc.pass_rows * lay.ring * lay.Lk;
    // scratch sums: a block of steps carried for layers of at most 64 units ([row][128]); eight slices of raw
    // sums for launches of fewer than 128 work-groups ([slice][row][32 nJB])
    const int cw = lay.nJB >= 3 ? 4 : lay.nJB;
    const int64_t few_rows = (int64_t)128 * 32 * (4 / cw) < sc.pass_rows ? (int64_t)128 * 32 * (4 / cw) : sc.pass_rows;
    const size_t carried = lay.nJB <= 2 ? (size_t)sc.pass_rows * 128 : 0;
    const size_t split = (size_t)8 * few_rows * 32 * lay.nJB;
    sc.sums_floats = carried > split ? carried : split;
    sc.off_sums = (sc.hist_floats * sizeof(float) + 255) & ~(size_t)255;
    sc.bytes = (sc.off_sums + sc.sums_floats * sizeof(float) + 255) & ~(size_t)255;
    return sc;
}

// Stack rows: slot s = 0 .. ring-1 holds lag ring - s (Lk rows, those beyond L zero), then W, b, zeros.
// Fragment order: [column block][k-group][lane][e] with row = 8*group + 4*(lane>>5) + e, column = lane&31.
void pack_weights_fc_steps(const FcStepLayout& lay, const float* W, const float* A, const float* b, float* out) {
    const int L = lay.L, d = lay.d, Lk = lay.Lk;
    const int64_t hist_rows = (int64_t)lay.ring * Lk;
    for (size_t i = 0; i < lay.floats; ++i) out[i] = 0.0f;
    for (int jb = 0; jb < lay.nJB; ++jb)
        for (int kg = 0; kg < lay.KGtot; ++kg)
            for (int lane = 0; lane < 64; ++lane)
                for (int e = 0; e < 4; ++e) {
                    const int64_t k = (int64_t)kg * 8 + (lane >> 5) * 4 + e;
                    const int j = jb * 32 + (lane & 31);
                    if (j >= L) continue;
                    float v = 0.0f;
                    if (k < hist_rows) {
                        const int s = (int)(k / Lk), mm = (int)(k - (int64_t)s * Lk);
                        const int lag = lay.ring - s;
                        if (mm < L) v = A[((size_t)(lag - 1) * L + mm) * L + j];
                    } else if (k - hist_rows < d) {
                        v = W[(size_t)(k - hist_rows) * L + j];
                    } else if (k - hist_rows == d) {
                        v = b[j];
                    }
                    out[(((size_t)jb * lay.KGpad + kg) * 64 + lane) * 4 + e] = v;
                }
}

// The same stack per 16-column unit: [k-group][unit][lane][e], row = 8*group + 2*(lane>>4) + e, column = lane&15.
void pack_weights_fc_rows(const FcStepLayout& lay, const float* W, const float* A, const float* b, float* out) {
    const int L = lay.L, d = lay.d, Lk = lay.Lk;
    const int64_t hist_rows = (int64_t)lay.ring * Lk;
    for (size_t i = 0; i < lay.floats16; ++i) out[i] = 0.0f;
    for (int cu = 0; cu < lay.NU; ++cu)
        for (int kg = 0; kg < lay.KGtot; ++kg)
            for (int lane = 0; lane < 64; ++lane)
                for (int e = 0; e < 2; ++e) {
                    const int64_t k = (int64_t)kg * 8 + (lane >> 4) * 2 + e;
                    const int j = cu * 16 + (lane & 15);
                    if (j >= L) continue;
                    float v = 0.0f;
                    if (k < hist_rows) {
                        const int s = (int)(k / Lk), mm = (int)(k - (int64_t)s * Lk);
                        if (mm < L) v = A[((size_t)(lay.ring - s - 1) * L + mm) * L + j];
                    } else if (k - hist_rows < d) {
                        v = W[(size_t)(k - hist_rows) * L + j];
                    } else if (k - hist_rows == d) {
                        v = b[j];
                    }
                    out[(((size_t)kg * lay.NU + cu) * 64 + lane) * 2 + e] = v;
                }
}

hipError_t launch_hidden_fc_steps(const FcStepLayout& lay, const float* Wp, const float* Wp16, void* scratch,
                                  const float* X, int64_t ldx_n, int64_t ldx_q, int64_t N, int Q_run, float* H,
                                  hipStream_t stream) {
    if (Q_run < 1 || Q_run > lay.Q || N < 1 || scratch == nullptr) return hipErrorInvalidValue;
    const FcScratch scr = fc_scratch(lay, N);
    float* hist = static_cast<float*>(scratch);
    float* sums = reinterpret_cast<float*>(static_cast<char*>(scratch) + scr.off_sums);
    const int cw = lay.nJB >= 3 ? 4 : lay.nJB;
    const int ycount = (lay.nJB + cw - 1) / cw;
    const int ldsums = 128;                    // carried sums of a block of steps: [row][B][32 nJB]
    const int ldp = 32 * lay.nJB;              // raw sums of a split launch: [slice][row][32 nJB]
    const int S1 = 32 * (4 / cw);              // rows of the smallest tile
    // passes of equal size (a multiple of 256 rows) rather than full buffers and a short last one
    const int64_t passes = (N + lay.chunk_rows - 1) / lay.chunk_rows;
    const int64_t per_pass = ((N + passes - 1) / passes + 255) / 256 * 256;
    const int64_t slot_floats = per_pass * lay.Lk;
    for (int64_t r0 = 0; r0 < N; r0 += per_pass) {
        const int64_t rows = (N - r0 < per_pass) ? N - r0 : per_pass;
        FcStepArgs base{};
        base.Lk = lay.Lk; base.slot_floats = (unsigned)slot_floats; base.slot_groups = (unsigned)(lay.Lk / 8);
        base.ldx_n = ldx_n; base.Wp = Wp; base.wp_bytes = (unsigned)(lay.floats * sizeof(float));
        base.jb_stride = (unsigned)lay.KGpad * 1024u;
        base.d = lay.d; base.L = lay.L; base.nJB = lay.nJB; base.rows = (int)rows;
        base.nsteps = 1; base.ldacc = ldsums;
        base.Wp16 = Wp16; base.wp16_bytes = (unsigned)(lay.floats16 * sizeof(float));

        // a pass of few rows (long windows: the history of 1,000 rows can be 1 GB) leaves compute units idle:
        // its launches split the contraction over up to 8 slices of the operand chunks instead
        const int64_t wgs = (rows + S1 - 1) / S1 * ycount;
        const bool few = sums != nullptr && wgs < 128 && (size_t)8 * rows * ldp <= scr.sums_floats;
        // steps per block: the waves that a layer of one or two column blocks leaves free take further steps
        const int B = (sums != nullptr && lay.nJB <= 2 && !few) ? 4 / lay.nJB : 1;
        if (Wp16 != nullptr && lay.NU > 0 && (rows + 127) / 128 >= 256) {       // every compute unit gets a tile
            FcStepArgs a = base;
            a.hist = hist; a.hist_out = hist;
            a.hist_bytes = (unsigned)(lay.ring * slot_floats * (int64_t)sizeof(float));
            a.X = X + r0 * ldx_n; a.ldx_q = ldx_q;
            a.H = H + r0 * lay.L;
            a.t_first = 1; a.t_last = Q_run; a.Q_run = Q_run; a.ring = lay.ring;
            const hipError_t e = lay.NU == 5 ? launch_rows<5>(a, stream) : launch_rows<6>(a, stream);
            if (e != hipSuccess) return e;
            continue;
        }
        for (int t0 = 0; t0 < Q_run; t0 += B) {
            const int nb = Q_run - t0 < B ? Q_run - t0 : B;
            const bool carried = B > 1 && t0 > 0;
            if (carried) {
                // the finished slots 0 .. t0-1 into the sums of steps t0+1 .. t0+nb
                FcStepArgs a = base;
                a.hist = hist; a.hist_bytes = (unsigned)(lay.ring * slot_floats * (int64_t)sizeof(float));
                a.X = X;                                   // not read
                a.Kh = t0 * lay.Lk;
                a.kg0 = (unsigned)((lay.ring - t0) * (lay.Lk / 8));      // step t0+1; step t0+j starts j-1 slots earlier
                a.nchunks = (a.Kh + kBK - 1) / kBK;
                a.block = 1; a.nsteps = nb;
                a.out = sums; a.ldo = ldsums; a.ncols = ldsums;
                const hipError_t e = (rows + 63) / 64 >= 512 ? launch_step<2, 4, true>(a, 1, stream)
                                                             : launch_step<1, 4, true>(a, 1, stream);
                if (e != hipSuccess) return e;
            }
            for (int j = 1; j <= nb; ++j) {
                const int t = t0 + j;
                const int own = carried ? j - 1 : t - 1;   // slots this launch contracts itself: t-1-own .. t-2
                const int first = t - 1 - own;
                FcStepArgs a = base;
                a.hist = hist + (int64_t)first * slot_floats;
                a.hist_bytes = (unsigned)((lay.ring - first) * slot_floats * (int64_t)sizeof(float));
                a.X = X + r0 * ldx_n + (int64_t)(t - 1) * ldx_q;
                a.Kh = own * lay.Lk;
                a.kg0 = (unsigned)((lay.ring - own) * (lay.Lk / 8));
                const int groups = (a.Kh + lay.d + 1 + 7) / 8;
                a.nchunks = (groups + kPF - 1) / kPF;
                a.acc_in = carried ? sums + (j - 1) * 32 * lay.nJB : nullptr;
                if (t == Q_run) {
                    a.out = H + r0 * lay.L; a.ldo = lay.L; a.ncols = lay.L;
                } else {
                    a.out = hist + (int64_t)(t - 1) * slot_floats; a.ldo = lay.Lk; a.ncols = lay.Lk;
                }
                int slices = 1;
                if (few) {
                    slices = (int)(256 / wgs) < 8 ? (int)(256 / wgs) : 8;
                    if (slices > a.nchunks / 4) slices = a.nchunks / 4;      // at least four chunks per slice
                }
                if (slices >= 2) {
                    float* out = a.out;
                    const int64_t ldo = a.ldo;
                    a.raw = 1; a.out = sums; a.ldo = ldp; a.zstride = rows * ldp;
                    hipError_t e = cw == 4   ? launch_step<1, 4, true>(a, ycount, stream, slices)
                                   : cw == 2 ? launch_step<1, 2, true>(a, ycount, stream, slices)
                                             : launch_step<1, 1, true>(a, ycount, stream, slices);
                    if (e != hipSuccess) return e;
                    const int64_t total = rows * a.ncols;
                    hipLaunchKernelGGL(fc_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                                       sums, slices, a.zstride, ldp, (int)rows, lay.L, a.ncols, out, ldo);
                    e = hipGetLastError();
                    if (e != hipSuccess) return e;
                    continue;
                }
                // 64-row blocks per wave while they still give every compute unit two work-groups
                const bool big = cw > 1 && (rows + 64 * (4 / cw) - 1) / (64 * (4 / cw)) >= 512;
                hipError_t e;
                if (cw == 4) e = big ? launch_step<2, 4>(a, ycount, stream) : launch_step<1, 4>(a, ycount, stream);
                else if (cw == 2) e = big ? launch_step<2, 2, true>(a, ycount, stream) : launch_step<1, 2, true>(a, ycount, stream);
                else e = launch_step<1, 1, true>(a, ycount, stream);
                if (e != hipSuccess) return e;
            }
        }
    }
    return hipSuccess;
}

}  // namespace elm
