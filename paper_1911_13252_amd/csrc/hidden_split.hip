// Stage 1, fast contraction mode: the same hidden-matrix build as hidden.hip (step 2 of the paper's
// Algorithm "S-R-ELM"), with the recurrent contraction h_{t-1} U carried by fp16 matrix
// instructions at float32-equivalent accuracy.
//
// Every float32 operand value v of the recurrent part is split as v*s = hi + lo with hi = fp16(v*s)
// and lo = fp16(v*s - hi) (s a power of two: 2^13 for h, which lies in [-1, 1], and the power of two
// that brings max|U| into [2^13, 2^14) for the weights).  hi + lo carries 22 significant bits, and
//     A B  ~  Ahi Bhi + Ahi Blo + Alo Bhi        (three v_mfma_f32_32x32x16_f16, fp32 accumulate)
// drops only the lo*lo term (2^-22 relative).  The input and bias part [x_t | 1] . [W; b] has no
// bounded range, so it is split exactly into three bf16 pieces per value (x = p1 + p2 + p3 by
// truncation) and contracted with six v_mfma_f32_32x32x16_bf16 (all products above 2^-24 relative).
// The accumulators hold P = 2^13 * s_U times the pre-activation; W and b are pre-multiplied by P.
//
// Work decomposition, register-resident state and the LDS-resident operand are those of hidden.hip;
// the operand row holds, per group of 16 recurrent columns, [hi(8) lo(8)] fp16 for each half-group
// of 8 (64 bytes), then one group of 16 input columns as [p1(8) p2(8) p3(8)] bf16 per half (96 bytes).

#include <algorithm>
#include <cmath>
#include <cstring>

#include "internal.h"

namespace elm {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ uintx4 buffer_load_x4(__amdgpu_buffer_rsrc_t rsrc, unsigned voff, unsigned soff) {
    return __builtin_amdgcn_raw_buffer_load_b128(rsrc, voff, soff, 0);
}
__device__ __forceinline__ floatx16 mfma_f16(uintx4 a, uintx4 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(halfx8, a), __builtin_bit_cast(halfx8, b),
                                                  c, 0, 0, 0);
}
__device__ __forceinline__ floatx16 mfma_bf16(uintx4 a, uintx4 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                   c, 0, 0, 0);
}

constexpr int kThreads = 256;      // 4 wavefronts, one per SIMD
constexpr int kXPT = 4;            // input values a thread can prefetch per step
constexpr float kHScale = 8192.0f; // 2^13: scale of h before the fp16 split

struct SplitArgs {
    const float* X;
    int64_t ldx_n, ldx_q;
    const void* Wp;
    const float* h0;
    const float* c0;
    float* H;
    float* C;
    int64_t N;
    int Q_run, d, L, KGs, nJB;
    int stride, xoff;          // operand row stride and offset of the input group, in bytes
    unsigned wp_bytes;
    float inv_scale;           // 1 / P
};

// v * 2^13 = hi + lo in fp16; hi goes to p[0], lo 16 bytes further (the lo block of the half-group)
__device__ __forceinline__ void store_split_h(char* p, float v) {
    const float s = v * kHScale;
    const _Float16 hi = (_Float16)s;
    const _Float16 lo = (_Float16)(s - (float)hi);
    *reinterpret_cast<_Float16*>(p) = hi;
    *reinterpret_cast<_Float16*>(p + 16) = lo;
}
// four consecutive recurrent columns of one row (first column a multiple of 4): 8-byte stores
typedef _Float16 halfx4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_split_h4(char* p, float v0, float v1, float v2, float v3) {
    const float s[4] = {v0 * kHScale, v1 * kHScale, v2 * kHScale, v3 * kHScale};
    halfx4 hi, lo;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        hi[e] = (_Float16)s[e];
        lo[e] = (_Float16)(s[e] - (float)hi[e]);
    }
    *reinterpret_cast<halfx4*>(p) = hi;
    *reinterpret_cast<halfx4*>(p + 16) = lo;
}
// x = p1 + p2 + p3 exactly, each piece a bf16 (truncation keeps 8 significant bits per piece)
__device__ __forceinline__ void store_split_x(char* p, float x) {
    const unsigned u1 = __builtin_bit_cast(unsigned, x) & 0xFFFF0000u;
    const float r1 = x - __builtin_bit_cast(float, u1);
    const unsigned u2 = __builtin_bit_cast(unsigned, r1) & 0xFFFF0000u;
    const float r2 = r1 - __builtin_bit_cast(float, u2);
    const unsigned u3 = __builtin_bit_cast(unsigned, r2) & 0xFFFF0000u;
    *reinterpret_cast<unsigned short*>(p) = (unsigned short)(u1 >> 16);
    *reinterpret_cast<unsigned short*>(p + 16) = (unsigned short)(u2 >> 16);
    *reinterpret_cast<unsigned short*>(p + 32) = (unsigned short)(u3 >> 16);
}
// byte offset of recurrent column k / input column k inside an operand row
__device__ __forceinline__ int h_col_off(int k) { return (k >> 4) * 64 + ((k >> 3) & 1) * 32 + (k & 7) * 2; }
__device__ __forceinline__ int x_col_off(int k) { return ((k >> 3) & 1) * 48 + (k & 7) * 2; }

// Activations of a scaled accumulator v = P * a: the factor 1/P is folded into the exponent
// constants k1 = -log2(e)/P and k2 = 2 log2(e)/P, so sigmoid(a) = 1/(1 + 2^(k1 v)) and
// tanh(a) = 1 - 2/(1 + 2^(k2 v)) cost one multiply, one v_exp and one v_rcp each.
__device__ __forceinline__ float sigmoid_s(float v, float k1) {
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(v * k1));
}
__device__ __forceinline__ float tanh_s(float v, float k2) {
    return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(v * k2));
}
__device__ __forceinline__ float tanh_f(float x) {
    return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(x * 2.885390081777927f));
}
// acc[g][ms] += A(ms) . B(g) over the whole weight stream of one column block.
//   Stream position 0 and 1: the input group.  Slot 0 holds bf16 pieces (p1, p2) of [W; b] * P, slot 1
//   holds (p3, unused).  Position p >= 2: recurrent group kg = p - 2, the slot holds (hi, lo) of U * s_U.
//   Fragment of position p, gate slot g (gate GA + g*GSTEP of GT): two 1 KB blocks at byte
//     wbase + (p*GT + GA + g*GSTEP)*2048 (+1024), lane l reads 16 bytes at 16*l = 8 consecutive k
//     (k = 8*(l>>5) + j inside the group) of column l&31.
//   A fragment: lane (r = l&31, half = l>>5) reads 16 bytes of row ms*32 + r at
//     kg*64 + half*32 (hi), +16 (lo);  input group at xoff + half*48 (+16, +32).
// Fill all PF slots of the weight-fragment queue with stream positions 0..PF-1.
template <int G, int GT, int GA, int GSTEP, int PF>
__device__ __forceinline__ void prefetch_weights(uintx4 (&bq)[PF][G][2], __amdgpu_buffer_rsrc_t wrs,
                                                 unsigned wbase, int lane) {
    const unsigned voff = (unsigned)lane * 16u;
    // Drain every older vector-memory access first (s_waitcnt vmcnt(0)): the compiler's wait
    // insertion then sees only these loads as pending inside the contraction loop and emits exact
    // vmcnt(n) waits instead of draining the queue once per trip.
    __builtin_amdgcn_s_waitcnt(0x0F70);
#pragma unroll
    for (int u = 0; u < PF; ++u) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const unsigned off = wbase + (unsigned)(u * GT + GA + g * GSTEP) * 2048u;
            bq[u][g][0] = buffer_load_x4(wrs, voff, off);
            bq[u][g][1] = buffer_load_x4(wrs, voff, off + 1024u);
        }
        __builtin_amdgcn_sched_barrier(0);      // issue order: oldest slot first
    }
}

// The contraction proper; bq must hold stream positions 0..PF-1 (prefetch_weights).  Slot p % PF is
// consumed by the MFMAs of position p and refilled, in place, with position p + PF right after them.
template <int G, int GT, int GA, int GSTEP, int MS, int PF>
__device__ __forceinline__ void contract_main(floatx16 (&acc)[G][MS], uintx4 (&bq)[PF][G][2],
                                              const char* __restrict__ Abuf, int stride, int xoff,
                                              __amdgpu_buffer_rsrc_t wrs, unsigned wbase, int KGs, int lane) {
    static_assert(PF >= 3, "the input group occupies two slots");
    const unsigned voff = (unsigned)lane * 16u;
    const char* ap = Abuf + (lane & 31) * stride + (lane >> 5) * 32;
    auto refill = [&](int u, int p) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const unsigned off = wbase + (unsigned)(p * GT + GA + g * GSTEP) * 2048u;
            bq[u][g][0] = buffer_load_x4(wrs, voff, off);
            bq[u][g][1] = buffer_load_x4(wrs, voff, off + 1024u);
        }
    };

    // Register economy: every A fragment is loaded as late as its first use allows and the products
    // are ordered so that fragments die early (the x pieces one after the other, then per recurrent
    // group hi before lo), which keeps at most three 4-register fragments per row block live.
    uintx4 a[MS][2];              // (hi, lo) fragment of the current recurrent group
    {
        const char* axp = ap + xoff + (lane >> 5) * 16;      // half*48 in total
        uintx4 x[MS][3];
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int q = 0; q < 3; ++q)
                x[ms][q] = *reinterpret_cast<const uintx4*>(axp + ms * 32 * stride + q * 16);
        __builtin_amdgcn_sched_barrier(0);
        // products kept (smallest first): p3p1, p2p2, p2p1, p1p3, p1p2, p1p1 -- everything above
        // 2^-24 relative
#pragma unroll
        for (int c = 0; c < 6; ++c) {
            const int xa = (c == 0) ? 2 : (c <= 2) ? 1 : 0;
            const int wslot = (c == 3) ? 1 : 0;
            const int wpiece = (c == 1 || c == 4) ? 1 : 0;
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int ms = 0; ms < MS; ++ms)
                    acc[g][ms] = mfma_bf16(bq[wslot][g][wpiece], x[ms][xa], acc[g][ms]);
            if (c == 2) {             // pieces 3 and 2 are dead: fetch hi of the first recurrent group
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int ms = 0; ms < MS; ++ms)
                    a[ms][0] = *reinterpret_cast<const uintx4*>(ap + ms * 32 * stride);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
            a[ms][1] = *reinterpret_cast<const uintx4*>(ap + ms * 32 * stride + 16);
        if (PF < KGs) refill(0, PF);
        if (PF + 1 < KGs) refill(1, PF + 1);
        __builtin_amdgcn_sched_barrier(0);
    }

    const int KGh = KGs - 2;
    auto group = [&](int p, int u, bool do_refill) {
        const int kg = p - 2;
        const int kn = (kg + 1 < KGh) ? (kg + 1) : kg;
        uintx4 an[MS];               // hi fragment of the next recurrent group
#pragma unroll
        for (int c = 0; c < 2; ++c) {          // hi*lo, hi*hi
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int ms = 0; ms < MS; ++ms)
                    acc[g][ms] = mfma_f16(bq[u][g][c == 0 ? 1 : 0], a[ms][0], acc[g][ms]);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
            an[ms] = *reinterpret_cast<const uintx4*>(ap + ms * 32 * stride + kn * 64);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < G; ++g)            // lo*hi
#pragma unroll
            for (int ms = 0; ms < MS; ++ms)
                acc[g][ms] = mfma_f16(bq[u][g][0], a[ms][1], acc[g][ms]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ms = 0; ms < MS; ++ms) {
            a[ms][1] = *reinterpret_cast<const uintx4*>(ap + ms * 32 * stride + kn * 64 + 16);
            a[ms][0] = an[ms];
        }
        if (do_refill) refill(u, p + PF);
        __builtin_amdgcn_sched_barrier(0);
    };

    int p = 2;
    for (; p + 2 * PF <= KGs; p += PF) {        // branch-free body: PF groups, PF refills
#pragma unroll
        for (int u = 0; u < PF; ++u) group(p + u, (2 + u) % PF, true);
    }
    for (; p + PF <= KGs; p += PF) {            // last full trip: refill only what is still needed
#pragma unroll
        for (int u = 0; u < PF; ++u) group(p + u, (2 + u) % PF, p + u + PF < KGs);
    }
#pragma unroll
    for (int u = 0; u < PF - 1; ++u)            // remaining groups, nothing left to load
        if (p + u < KGs) group(p + u, (2 + u) % PF, false);
}

template <int G, int GT, int GA, int GSTEP, int MS, int PF>
__device__ __forceinline__ void contract(floatx16 (&acc)[G][MS], const char* __restrict__ Abuf, int stride,
                                         int xoff, __amdgpu_buffer_rsrc_t wrs, unsigned wbase, int KGs,
                                         int lane) {
    uintx4 bq[PF][G][2];
    prefetch_weights<G, GT, GA, GSTEP, PF>(bq, wrs, wbase, lane);
    contract_main<G, GT, GA, GSTEP, MS, PF>(acc, bq, Abuf, stride, xoff, wrs, wbase, KGs, lane);
}

// STAGE > 0: that many of a lane's pending new-h values (those of the first column chunk) wait in
// spare LDS instead of registers; used by the largest LSTM variants, which otherwise spill.
// In the LSTM variants with three or four column chunks the pending new-h values of the middle
// chunks (1 .. NCH-2) do not wait in registers either: they are parked in the tile's own rows of H (private to the
// work-group until the last step, which writes them in place) and read back, all loads in flight at
// once, when the operand is rebuilt.
// WR > 1 (narrow layers, L <= 64, one column chunk): the four waves share 4/WR column blocks and split
// the tile's rows into WR groups of 32*MS instead, so that no wave is idle.
// Variants that fit 256 registers (32-row blocks, one column chunk) are compiled for two waves per
// SIMD: one wave's gate math overlaps another's matrix work.
template <int CELL, int MS, int NCH, int STAGE, int WR>
__global__ __launch_bounds__(kThreads, (MS == 1 && NCH == 1) ? 2 : 1)
void hidden_split_kernel(const SplitArgs p) {
    static_assert(WR == 1 || NCH == 1, "rows are split over the waves only when one column chunk exists");
    constexpr int G = (CELL == ELM_CELL_ELMAN) ? 1 : (CELL == ELM_CELL_LSTM) ? 4 : 3;
    constexpr int S = 32 * MS * WR;
    // fragment-queue depth; the widest LSTM variants have 24 matrix instructions per group and
    // the fewest spare registers: three groups in flight cover the L2 latency there
    constexpr int PF = (CELL == ELM_CELL_LSTM && NCH >= 3) ? 3 : 4;
    constexpr bool GSTAGE = (CELL == ELM_CELL_LSTM) && (NCH >= 3);   // middle chunks parked in H
    extern __shared__ __align__(16) char lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    // wave-uniform values are forced into scalar registers: weight addresses then live in SGPRs
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wcol = (WR == 1) ? wave : wave % (4 / WR);          // column block of this wave in a chunk
    const int rbase = (WR == 1) ? 0 : (wave / (4 / WR)) * 32 * MS;   // first tile row of this wave
    const int L = p.L, d = p.d, KGs = p.KGs, stride = p.stride, xoff = p.xoff;
    const float k1 = -1.4426950408889634f * p.inv_scale, k2 = 2.885390081777927f * p.inv_scale;
    const int64_t row0 = (int64_t)blockIdx.x * S;
    const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void*>(p.Wp), 0, (int)p.wp_bytes, 0x00020000);   // raw dword buffer, range-checked
    const int nbuf = (CELL == ELM_CELL_GRU) ? 2 : 1;
    char* A0 = lds;                     // [S][stride]: h_{t-1} | x_t | 1, split
    char* A1 = lds + S * stride;        // GRU only: (r*h_{t-1}) | x_t | 1, split
    float* stage = reinterpret_cast<float*>(lds + nbuf * S * stride) + tid;   // STAGE > 0: [STAGE][256]

    // The weights sit on the M side of the matrix instruction and the samples on the N side, so
    // accumulator element (ms, i) of this lane belongs to sample row ms*32 + (lane & 31) and to
    // hidden column 8*(i>>2) + 4*(lane>>5) + (i&3) of the 32-column block: every group of four
    // elements i = 4q..4q+3 is four consecutive columns of one row (8-byte operand stores).
    const int samp_in = lane & 31;
    const int unit0 = 4 * (lane >> 5);
    auto acc_unit = [&](int i) { return 8 * (i >> 2) + unit0 + (i & 3); };
    const int Lp = p.KGs * 16 - 32;      // recurrent columns the operand row has room for

    // ---- initial contents of the activation operand: h = 0, x = 0, the bias column = 1 (piece 1)
    {
        unsigned* w = reinterpret_cast<unsigned*>(lds);
        const int words = nbuf * S * stride / 4;
        for (int idx = tid; idx < words; idx += kThreads) w[idx] = 0u;
    }
    __syncthreads();
    for (int s = tid; s < nbuf * S; s += kThreads)
        *reinterpret_cast<unsigned short*>(lds + s * stride + xoff + x_col_off(d)) = 0x3F80;   // bf16 1.0
    if (p.h0 != nullptr) {
        for (int idx = tid; idx < S * L; idx += kThreads) {
            const int s = idx / L, k = idx - s * L;
            const int64_t row = row0 + s;
            if (row < p.N) store_split_h(A0 + s * stride + h_col_off(k), p.h0[row * L + k]);
        }
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
    auto store_x = [&](char* buf) {
#pragma unroll
        for (int q = 0; q < kXPT; ++q) {
            const int e = tid + q * kThreads;
            if (e < nx) {
                const int s = e / d, dd = e - s * d;
                store_split_x(buf + s * stride + xoff + x_col_off(dd), xr[q]);
            }
        }
    };
    auto copy_x_direct = [&](int t, char* buf) {     // wide tiles: no register staging
        for (int e = tid; e < nx; e += kThreads) {
            const int s = e / d, dd = e - s * d;
            const int64_t row = row0 + s;
            store_split_x(buf + s * stride + xoff + x_col_off(dd),
                          (row < p.N) ? p.X[row * p.ldx_n + (int64_t)t * p.ldx_q + dd] : 0.0f);
        }
    };

    // ---- register-resident state
    float st[NCH][MS][16];     // LSTM: cell state c; GRU: this lane's own copy of h; Elman: unused
    float hn[NCH][MS][16];     // LSTM/Elman: new h until the old one is dead; GRU: update gate z
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
        const int jb = ch * 4 + wcol;
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float v = 0.0f;
                const int64_t row = row0 + rbase + ms * 32 + samp_in;
                const int col = jb * 32 + acc_unit(i);
                const float* src = (CELL == ELM_CELL_LSTM) ? p.c0 : (CELL == ELM_CELL_GRU) ? p.h0 : nullptr;
                if (src != nullptr && row < p.N && col < L) v = src[row * L + col];
                st[ch][ms][i] = v;
                hn[ch][ms][i] = 0.0f;
            }
    }
    __syncthreads();       // operand constants written before the x slots are filled
    if (x_prefetch) {
        load_x(0);
        store_x(A0);
        // the GRU's second operand gets x_0 at the top of the first step
    } else {
        copy_x_direct(0, A0);
    }
    __syncthreads();

    // lane part of the operand address of this lane's accumulator elements: row samp_in, first
    // column unit0 of the block; element group (ms, q) adds ms*32*stride + jb*128 + h_col_off(8q)
    const int lane_base0 = (rbase + samp_in) * stride + unit0 * 2;
    // the tile's rows of H as a range-checked buffer (rows past N are dropped by the hardware);
    // element group (ms, q) of column block jb sits at hvoff + (ms*32*L + jb*32 + 8q)*4
    const int64_t rows_here = (p.N - row0 < S) ? (p.N - row0) : S;
    const __amdgpu_buffer_rsrc_t hrs = __builtin_amdgcn_make_buffer_rsrc(
        p.H + row0 * L, 0, (int)(rows_here * L * 4), 0x00020000);
    const unsigned hvoff = (unsigned)((rbase + samp_in) * L + unit0) * 4u;
    // Between steps a full tile keeps the staged values in a packed order instead (value e of
    // thread tid at e*1024 + tid*4: every wave store is one contiguous 256 bytes); the last step and
    // a ragged last tile use the true H layout.  (NCH-2)*MS*16 KB always fit the tile's S*L*4 bytes.
    const bool packed_stage = GSTAGE && rows_here == S;

    for (int t = 0; t < p.Q_run; ++t) {
        if (CELL == ELM_CELL_GRU) {
            if (x_prefetch) store_x(A1); else copy_x_direct(t, A1);
        }
        const bool more = (t + 1 < p.Q_run);
        if (x_prefetch && more) load_x(t + 1);

        if (CELL != ELM_CELL_GRU) {
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                const int jb = ch * 4 + wcol;
                if (jb < p.nJB) {
                    const unsigned wbase = (unsigned)(jb * KGs * G) * 2048u;
                    {
                        floatx16 acc[G][MS];
#pragma unroll
                        for (int g = 0; g < G; ++g)
#pragma unroll
                            for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                                for (int i = 0; i < 16; ++i) acc[g][ms][i] = 0.0f;
                        contract<G, G, 0, 1, MS, PF>(acc, A0 + rbase * stride, stride, xoff, wrs, wbase, KGs, lane);
#pragma unroll
                        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                            for (int i = 0; i < 16; ++i) {
                                if (CELL == ELM_CELL_ELMAN) {
                                    hn[ch][ms][i] = tanh_s(acc[0][ms][i], k2);
                                } else {
                                    const float ig = sigmoid_s(acc[0][ms][i], k1);
                                    const float fg = sigmoid_s(acc[G > 1 ? 1 : 0][ms][i], k1);
                                    const float og = sigmoid_s(acc[G > 2 ? 2 : 0][ms][i], k1);
                                    const float gg = tanh_s(acc[G > 3 ? 3 : 0][ms][i], k2);
                                    const float c = fg * st[ch][ms][i] + ig * gg;
                                    st[ch][ms][i] = c;
                                    const float hv = og * tanh_f(c);
                                    if (ch == 0 && ms * 16 + i < STAGE) {
                                        stage[(ms * 16 + i) * kThreads] = hv;
                                    } else if (GSTAGE && ch >= 1 && ch < NCH - 1) {
                                        const bool packed = packed_stage && more;     // uniform
                                        __builtin_amdgcn_raw_buffer_store_b32(
                                            __builtin_bit_cast(unsigned, hv), hrs, packed ? tid * 4u : hvoff,
                                            packed ? (unsigned)((ch - 1) * MS * 16 + ms * 16 + i) * 1024u
                                                   : (unsigned)(ms * 32 * L + jb * 32 + 8 * (i >> 2) + (i & 3)) * 4u, 0);
                                    } else {
                                        hn[ch][ms][i] = hv;
                                    }
                                }
                            }
                    }
                }
            }
            __syncthreads();          // every wave has finished reading h_{t-1}
            if (more) {
                // lane base address, made opaque per step so that the store addresses are recomputed
                // here (scalar row offsets) instead of being kept live across the unroll
                int lane_base = lane_base0;
                asm volatile("" : "+v"(lane_base));
#pragma unroll
                for (int ch = 0; ch < NCH; ++ch) {
                    const int jb = ch * 4 + wcol;
                    if (jb < p.nJB) {
                        char* dst = A0 + lane_base + jb * 128;
                        float v[MS][16];
#pragma unroll
                        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                            for (int i = 0; i < 16; ++i) {
                                if (GSTAGE && ch >= 1 && ch < NCH - 1)
                                    v[ms][i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                                        hrs, packed_stage ? tid * 4u : hvoff,
                                        packed_stage ? (unsigned)((ch - 1) * MS * 16 + ms * 16 + i) * 1024u
                                                     : (unsigned)(ms * 32 * L + jb * 32 + 8 * (i >> 2) + (i & 3)) * 4u, 0));
                                else
                                    v[ms][i] = (ch == 0 && ms * 16 + i < STAGE) ? stage[(ms * 16 + i) * kThreads]
                                                                                : hn[ch][ms][i];
                            }
#pragma unroll
                        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                if (jb * 32 + 8 * q < Lp)
                                    store_split_h4(dst + ms * 32 * stride + h_col_off(8 * q), v[ms][4 * q],
                                                   v[ms][4 * q + 1], v[ms][4 * q + 2], v[ms][4 * q + 3]);
                    }
                }
                if (x_prefetch) store_x(A0); else copy_x_direct(t + 1, A0);
            }
            __syncthreads();
        } else {
            // phase 1: update and reset gates from h_{t-1}; stage r*h_{t-1} as the second operand
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                const int jb = ch * 4 + wcol;
                if (jb < p.nJB) {
                    floatx16 acc[2][MS];
#pragma unroll
                    for (int g = 0; g < 2; ++g)
#pragma unroll
                        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                            for (int i = 0; i < 16; ++i) acc[g][ms][i] = 0.0f;
                    contract<2, 3, 0, 1, MS, PF>(acc, A0 + rbase * stride, stride, xoff, wrs, (unsigned)(jb * KGs * 3) * 2048u, KGs, lane);
                    char* dst = A1 + lane_base0 + jb * 128;
#pragma unroll
                    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            float rh[4];
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const int i = 4 * q + e;
                                hn[ch][ms][i] = sigmoid_s(acc[0][ms][i], k1);
                                rh[e] = sigmoid_s(acc[1][ms][i], k1) * st[ch][ms][i];
                            }
                            if (jb * 32 + 8 * q < Lp)
                                store_split_h4(dst + ms * 32 * stride + h_col_off(8 * q), rh[0], rh[1], rh[2], rh[3]);
                        }
                }
            }
            __syncthreads();
            // phase 2: candidate from r*h_{t-1}; blend; publish h_t into the first operand
#pragma unroll
            for (int ch = 0; ch < NCH; ++ch) {
                const int jb = ch * 4 + wcol;
                if (jb < p.nJB) {
                    floatx16 acc[1][MS];
#pragma unroll
                    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc[0][ms][i] = 0.0f;
                    contract<1, 3, 2, 1, MS, PF>(acc, A1 + rbase * stride, stride, xoff, wrs, (unsigned)(jb * KGs * 3) * 2048u, KGs, lane);
                    char* dst = A0 + lane_base0 + jb * 128;
#pragma unroll
                    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const int i = 4 * q + e;
                                const float z = hn[ch][ms][i];
                                st[ch][ms][i] = (1.0f - z) * st[ch][ms][i] + z * tanh_s(acc[0][ms][i], k2);
                            }
                            if (more && jb * 32 + 8 * q < Lp)
                                store_split_h4(dst + ms * 32 * stride + h_col_off(8 * q), st[ch][ms][4 * q],
                                               st[ch][ms][4 * q + 1], st[ch][ms][4 * q + 2], st[ch][ms][4 * q + 3]);
                        }
                }
            }
            if (more) {
                if (x_prefetch) store_x(A0); else copy_x_direct(t + 1, A0);
            }
            __syncthreads();
        }
    }

    // ---- H(Q) (and the LSTM cell state) straight from the float32 registers
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
        const int jb = ch * 4 + wcol;
        if (jb < p.nJB) {
            const bool in_place = GSTAGE && ch >= 1 && ch < NCH - 1;      // H already holds these
#pragma unroll
            for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int64_t row = row0 + rbase + ms * 32 + samp_in;
                    const int col = jb * 32 + acc_unit(i);
                    if (row < p.N && col < L) {
                        if (!in_place) {
                            float hv;
                            if (CELL == ELM_CELL_GRU) hv = st[ch][ms][i];
                            else hv = (ch == 0 && ms * 16 + i < STAGE) ? stage[(ms * 16 + i) * kThreads] : hn[ch][ms][i];
                            p.H[row * L + col] = hv;
                        }
                        if (CELL == ELM_CELL_LSTM && p.C != nullptr) p.C[row * L + col] = st[ch][ms][i];
                    }
                }
        }
    }
}

template <int CELL, int MS, int NCH, int STAGE, int WR = 1>
hipError_t launch_variant(const SplitArgs& a, int64_t tiles, size_t lds_bytes, hipStream_t stream) {
    auto kern = hidden_split_kernel<CELL, MS, NCH, STAGE, WR>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(kThreads), lds_bytes, stream, a);
    return hipGetLastError();
}

constexpr int kStage = 24;      // staged values per lane: 24 KB of LDS per work-group

template <int CELL, int MS>
hipError_t launch_nch(int nch, const SplitArgs& a, int64_t tiles, size_t lds, size_t lds_max,
                      hipStream_t s) {
    // the widest LSTM variants take the LDS staging when the operand leaves room for it
    const size_t staged = lds + (size_t)kStage * kThreads * sizeof(float);
    const bool stage = (CELL == ELM_CELL_LSTM) && MS == 2 && nch >= 3 && staged <= lds_max;
    switch (nch) {
        case 1: return launch_variant<CELL, MS, 1, 0>(a, tiles, lds, s);
        case 2: return launch_variant<CELL, MS, 2, 0>(a, tiles, lds, s);
        case 3:
            if (stage) return launch_variant<CELL, MS, 3, (CELL == ELM_CELL_LSTM && MS == 2) ? kStage : 0>(a, tiles, staged, s);
            return launch_variant<CELL, MS, 3, 0>(a, tiles, lds, s);
        case 4:
            if (stage) return launch_variant<CELL, MS, 4, (CELL == ELM_CELL_LSTM && MS == 2) ? kStage : 0>(a, tiles, staged, s);
            return launch_variant<CELL, MS, 4, 0>(a, tiles, lds, s);
        default: return hipErrorInvalidValue;
    }
}

template <int CELL>
hipError_t launch_cell(int ms, int nch, const SplitArgs& a, int64_t N, size_t lds_per_row,
                       size_t lds_max, hipStream_t s) {
    // narrow layers: one or two column blocks only, so the waves split the rows of a larger tile
    int wr = (a.nJB == 1) ? 4 : (a.nJB == 2) ? 2 : 1;
    if (lds_per_row * 32 * ms * wr > lds_max) wr = 1;
    // fewer tiles than compute units: halve the tile so that twice as many work-groups run; layers of
    // one column chunk (L <= 128) also run 32-row blocks per wave: those variants fit 256 registers,
    // so two waves share a SIMD
    if (ms == 2 && ((N + 64 * wr - 1) / (64 * wr) < 256 || nch == 1)) ms = 1;
    if (wr > 1) {
        const int Sw = 32 * ms * wr;
        const int64_t tiles = (N + Sw - 1) / Sw;
        const size_t lds = lds_per_row * Sw;
        if (ms == 2) {
            if (wr == 4) return launch_variant<CELL, 2, 1, 0, 4>(a, tiles, lds, s);
            return launch_variant<CELL, 2, 1, 0, 2>(a, tiles, lds, s);
        }
        if (wr == 4) return launch_variant<CELL, 1, 1, 0, 4>(a, tiles, lds, s);
        return launch_variant<CELL, 1, 1, 0, 2>(a, tiles, lds, s);
    }
    const int S = 32 * ms;
    const int64_t tiles = (N + S - 1) / S;
    const size_t lds = lds_per_row * S;
    if (ms == 2) return launch_nch<CELL, 2>(nch, a, tiles, lds, lds_max, s);
    return launch_nch<CELL, 1>(nch, a, tiles, lds, lds_max, s);
}

// x = p1 + p2 + p3, bf16 pieces by truncation (host side, same rule as store_split_x)
void split_bf16x3(float x, uint16_t (&piece)[3]) {
    for (int q = 0; q < 3; ++q) {
        uint32_t u;
        std::memcpy(&u, &x, sizeof u);
        u &= 0xFFFF0000u;
        float f;
        std::memcpy(&f, &u, sizeof f);
        piece[q] = (uint16_t)(u >> 16);
        x -= f;
    }
}

uint16_t half_bits(_Float16 h) {
    uint16_t u;
    std::memcpy(&u, &h, sizeof u);
    return u;
}

}  // namespace

SplitLayout split_layout(int cell, int d, int L, const float* W, const float* U, const float* b) {
    SplitLayout lay{};
    lay.cell = cell;
    lay.d = d;
    lay.L = L;
    lay.G = gates_of(cell);
    lay.KGh = (L + 15) / 16;
    lay.KGs = lay.KGh + 2;
    lay.nJB = (L + 31) / 32;
    lay.xoff = lay.KGh * 64;
    lay.stride = lay.xoff + 96 + 16;          // stride / 16 is odd: conflict-free 16-byte row reads
    // 8 padding positions: the first fill of the fragment queue may read past a short stream
    lay.bytes = ((size_t)lay.nJB * lay.KGs + 8) * lay.G * 2048;
    lay.ok = false;
    if (cell == ELM_CELL_ELMAN_DIAG || d > 15) return lay;       // one input group of 16 columns: d + 1 <= 16
    const size_t GL = (size_t)lay.G * L;
    float umax = 0.0f, wmax = 0.0f;
    for (size_t i = 0; i < (size_t)L * GL; ++i) {
        if (!std::isfinite(U[i])) return lay;
        umax = std::fmax(umax, std::fabs(U[i]));
    }
    for (size_t i = 0; i < (size_t)d * GL; ++i) {
        if (!std::isfinite(W[i])) return lay;
        wmax = std::fmax(wmax, std::fabs(W[i]));
    }
    for (size_t i = 0; i < GL; ++i) {
        if (!std::isfinite(b[i])) return lay;
        wmax = std::fmax(wmax, std::fabs(b[i]));
    }
    int e = 0;
    if (umax > 0.0f) (void)std::frexp(umax, &e);     // umax = f * 2^e, f in [0.5, 1)
    e = std::min(std::max(e, -60), 60);
    lay.log2_su = 14 - e;                            // max|U| * 2^log2_su in [2^13, 2^14)
    const double P = std::ldexp(1.0, 13 + lay.log2_su);
    if (!(wmax * P < 1e37)) return lay;
    lay.inv_scale = (float)(1.0 / P);
    lay.ok = true;
    return lay;
}

void pack_weights_split(const SplitLayout& lay, const float* W, const float* U, const float* b, void* out) {
    const int L = lay.L, d = lay.d, G = lay.G, GL = G * L;
    uint16_t* o = static_cast<uint16_t*>(out);
    std::memset(out, 0, lay.bytes);
    const float su = std::ldexp(1.0f, lay.log2_su);
    const float P = std::ldexp(1.0f, 13 + lay.log2_su);
    for (int jb = 0; jb < lay.nJB; ++jb)
        for (int g = 0; g < G; ++g)
            for (int lane = 0; lane < 64; ++lane) {
                const int j = jb * 32 + (lane & 31);
                if (j >= L) continue;
                const int col = g * L + j;
                auto block = [&](int pos, int second) {      // 16-bit index of this lane's 8 values
                    return ((((size_t)jb * lay.KGs + pos) * G + g) * 2048 + (size_t)second * 1024 + lane * 16) / 2;
                };
                for (int e = 0; e < 8; ++e) {
                    const int kx = (lane >> 5) * 8 + e;                  // input group: x columns, then the bias
                    const float v = (kx < d) ? W[(size_t)kx * GL + col] * P : (kx == d) ? b[col] * P : 0.0f;
                    uint16_t piece[3];
                    split_bf16x3(v, piece);
                    o[block(0, 0) + e] = piece[0];
                    o[block(0, 1) + e] = piece[1];
                    o[block(1, 0) + e] = piece[2];
                    for (int kg = 0; kg < lay.KGh; ++kg) {
                        const int k = kg * 16 + (lane >> 5) * 8 + e;
                        if (k >= L) continue;
                        const float sv = U[(size_t)k * GL + col] * su;   // exact: power-of-two scale
                        const _Float16 hi = (_Float16)sv;
                        const _Float16 lo = (_Float16)(sv - (float)hi);
                        o[block(2 + kg, 0) + e] = half_bits(hi);
                        o[block(2 + kg, 1) + e] = half_bits(lo);
                    }
                }
            }
}

hipError_t launch_hidden_split(const SplitLayout& lay, const void* Wp, const float* X, int64_t ldx_n,
                               int64_t ldx_q, int64_t N, int Q_run, const float* h0, const float* c0,
                               float* H, float* C, hipStream_t stream) {
    if (!lay.ok) return hipErrorInvalidValue;
    int dev = 0, lds_max = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    e = hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
    if (e != hipSuccess) return e;

    const int nbuf = (lay.cell == ELM_CELL_GRU) ? 2 : 1;
    const size_t lds_per_row = (size_t)nbuf * lay.stride;
    int ms = 2;
    if (lds_per_row * 64 > (size_t)lds_max) ms = 1;
    if (lds_per_row * 32 > (size_t)lds_max) return hipErrorInvalidValue;
    const int nch = (lay.nJB + 3) / 4;

    SplitArgs a{};
    a.X = X; a.ldx_n = ldx_n; a.ldx_q = ldx_q; a.Wp = Wp; a.h0 = h0; a.c0 = c0; a.H = H; a.C = C; a.N = N; a.Q_run = Q_run;
    a.d = lay.d; a.L = lay.L; a.KGs = lay.KGs; a.nJB = lay.nJB; a.stride = lay.stride; a.xoff = lay.xoff;
    a.wp_bytes = (unsigned)lay.bytes; a.inv_scale = lay.inv_scale;
    switch (lay.cell) {
        case ELM_CELL_ELMAN: return launch_cell<ELM_CELL_ELMAN>(ms, nch, a, N, lds_per_row, (size_t)lds_max, stream);
        case ELM_CELL_LSTM:  return launch_cell<ELM_CELL_LSTM>(ms, nch, a, N, lds_per_row, (size_t)lds_max, stream);
        case ELM_CELL_GRU:   return launch_cell<ELM_CELL_GRU>(ms, nch, a, N, lds_per_row, (size_t)lds_max, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace elm
