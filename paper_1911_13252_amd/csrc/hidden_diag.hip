// Stage 1 for the paper's own Elman cell (section "Elman", Eq. hij_elman): every neuron feeds back
// on itself only, from all earlier steps of the window,
//     h_j(t) = tanh( x(t) W[:, j] + b_j + sum_{k=1}^{t-1} alpha[j][k-1] h_j(t-k) ),   t = 1..Q,
// and row i of H is h(Q) of sample i.  There is no contraction across neurons, so this is plain
// vector arithmetic: Q(Q-1)/2 + Q d fused multiply-adds per (sample, neuron).
//
// Mapping: a lane owns one sample, a wave owns JT neurons at a time, so W, alpha and b are
// wave-uniform (scalar registers) and the inner loop is one vector FMA per term with the history
// held in registers (both loops fully unrolled up to QMAX steps, left early when Q is reached).
// A work-group of four waves walks over the neurons of its 64-sample tile; the tile's windows are
// staged once in LDS (transposed, coalesced global reads) and results leave through an LDS tile
// so that H is written in 128-byte row segments.  Windows too large for LDS are read directly.
// Q above 64 takes a one-wave kernel that keeps the history in LDS; Q above 128 (the paper's longest
// windows have 3,197 steps) a kernel that spreads the time axis of one (sample, neuron) pair over the
// lanes of a wave instead (measured: equal at 128 steps, 14 times faster at 512).

#include "internal.h"

namespace elm {
namespace {

__device__ __forceinline__ float tanh_d(float x) {
    return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __expf(2.0f * x));
}

constexpr int TILE = 64;        // samples per work-group = lanes of a wave
constexpr int XS_STRIDE = 65;   // LDS row stride of the transposed window tile
constexpr int OT_STRIDE = 33;   // LDS row stride of the 64 x 32 output tile

// X window of sample i, element e = t*d + s.
__device__ __forceinline__ float load_x(const float* __restrict__ X, int64_t ldx_n, int64_t ldx_q,
                                        int64_t i, int t, int s) {
    return X[i * ldx_n + (int64_t)t * ldx_q + s];
}

// Steps T..QMAX of one pass, unrolled by template recursion so that every index into the history
// is a compile-time constant (the history stays in registers); leaves at the first step past Q.
template <int T, int QMAX, int JT, bool XLDS>
struct DiagSteps {
    static __device__ __forceinline__ void run(float (&hist)[JT][QMAX], float (&last)[JT], const int (&jr)[JT],
                                               int Q, int d, int lda, int lane, const float* xs,
                                               const float* __restrict__ X, int64_t ldx_n, int64_t ldx_q,
                                               int64_t irow, const float* __restrict__ Wt,
                                               const float* __restrict__ alpha,
                                               const float* __restrict__ bias) {
        if (T > Q) return;
        float a[JT];
#pragma unroll
        for (int r = 0; r < JT; ++r) a[r] = bias[jr[r]];
        for (int s = 0; s < d; ++s) {
            const float xv = XLDS ? xs[((T - 1) * d + s) * XS_STRIDE + lane]
                                  : load_x(X, ldx_n, ldx_q, irow, T - 1, s);
#pragma unroll
            for (int r = 0; r < JT; ++r) a[r] = fmaf(xv, Wt[(size_t)jr[r] * d + s], a[r]);
        }
#pragma unroll
        for (int k = 1; k < T; ++k) {
#pragma unroll
            for (int r = 0; r < JT; ++r)
                a[r] = fmaf(alpha[(size_t)jr[r] * lda + (k - 1)], hist[r][T - k - 1], a[r]);
        }
#pragma unroll
        for (int r = 0; r < JT; ++r) {
            last[r] = tanh_d(a[r]);
            hist[r][T - 1] = last[r];
        }
        DiagSteps<T + 1, QMAX, JT, XLDS>::run(hist, last, jr, Q, d, lda, lane, xs, X, ldx_n, ldx_q, irow, Wt,
                                              alpha, bias);
    }
};
template <int QMAX, int JT, bool XLDS>
struct DiagSteps<QMAX + 1, QMAX, JT, XLDS> {
    static __device__ __forceinline__ void run(float (&)[JT][QMAX], float (&)[JT], const int (&)[JT], int, int,
                                               int, int, const float*, const float*, int64_t, int64_t,
                                               int64_t, const float*, const float*, const float*) {}
};

template <int QMAX, int JT, bool XLDS>
__global__ __launch_bounds__(256) void diag_reg_kernel(
    const float* __restrict__ X, int64_t ldx_n, int64_t ldx_q, int64_t N, int Q, int d, int L,
    const float* __restrict__ Wt,      // [L][d]
    const float* __restrict__ alpha,   // [L][lda], lag k in column k-1
    const float* __restrict__ bias,    // [L]
    int lda, float* __restrict__ H, int jchunk) {
    extern __shared__ float lds[];
    float* ot = lds;                              // [TILE][OT_STRIDE]
    float* xs = lds + TILE * OT_STRIDE;           // [Q*d][XS_STRIDE] when XLDS

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t i0 = (int64_t)blockIdx.x * TILE;
    const int64_t irow = i0 + lane < N ? i0 + lane : N - 1;      // clamped: tail lanes repeat the last row
    const int j_begin = blockIdx.y * jchunk;
    const int j_end = min(L, j_begin + jchunk);

    if (XLDS) {
        const int E = Q * d;
        for (int r = wave; r < TILE; r += 4) {
            const int64_t i = i0 + r < N ? i0 + r : N - 1;
            for (int e = lane; e < E; e += 64) {
                const int t = e / d, s = e - t * d;
                xs[e * XS_STRIDE + r] = load_x(X, ldx_n, ldx_q, i, t, s);
            }
        }
        __syncthreads();
    }

    constexpr int NJ = 4 * JT;                    // neurons per pass of the work-group
    for (int jb = j_begin; jb < j_end; jb += 32) {
        for (int jp = 0; jp < 32; jp += NJ) {
            const int jw = jb + jp + wave * JT;   // first neuron of this wave in this pass
            int jr[JT];
#pragma unroll
            for (int r = 0; r < JT; ++r) jr[r] = min(jw + r, L - 1);
            if (jb + jp < j_end) {                // uniform over the work-group
                float hist[JT][QMAX];
                float last[JT];
#pragma unroll
                for (int r = 0; r < JT; ++r) last[r] = 0.0f;
                DiagSteps<1, QMAX, JT, XLDS>::run(hist, last, jr, Q, d, lda, lane, xs, X, ldx_n, ldx_q, irow,
                                                  Wt, alpha, bias);
#pragma unroll
                for (int r = 0; r < JT; ++r) ot[lane * OT_STRIDE + jp + wave * JT + r] = last[r];
            }
        }
        __syncthreads();
        {   // flush 64 rows x 32 neurons: a lane group of 32 writes one 128-byte row segment
            const int col = threadIdx.x & 31, r0 = threadIdx.x >> 5;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int row = r0 + 8 * q;
                if (i0 + row < N && jb + col < j_end)
                    H[(size_t)(i0 + row) * L + jb + col] = ot[row * OT_STRIDE + col];
            }
        }
        __syncthreads();
    }
}

// Any Q up to the LDS capacity: one wave per work-group, history of the current neuron in LDS
// as hs[t][lane].
__global__ __launch_bounds__(64) void diag_lds_kernel(
    const float* __restrict__ X, int64_t ldx_n, int64_t ldx_q, int64_t N, int Q, int d, int L,
    const float* __restrict__ Wt, const float* __restrict__ alpha, const float* __restrict__ bias,
    int lda, float* __restrict__ H, int jchunk) {
    extern __shared__ float hs[];                 // [Q][64]
    const int lane = threadIdx.x;
    const int64_t i = (int64_t)blockIdx.x * TILE + lane;
    const int64_t irow = i < N ? i : N - 1;
    const int j_begin = blockIdx.y * jchunk;
    const int j_end = min(L, j_begin + jchunk);
    for (int j = j_begin; j < j_end; ++j) {
        const float bj = bias[j];
        float last = 0.0f;
        for (int t = 1; t <= Q; ++t) {
            float a = bj;
            for (int s = 0; s < d; ++s)
                a = fmaf(load_x(X, ldx_n, ldx_q, irow, t - 1, s), Wt[(size_t)j * d + s], a);
            for (int k = 1; k < t; ++k) a = fmaf(alpha[(size_t)j * lda + (k - 1)], hs[(t - k - 1) * 64 + lane], a);
            last = tanh_d(a);
            hs[(t - 1) * 64 + lane] = last;       // a lane reads back only its own column: no barrier
        }
        if (i < N) H[(size_t)i * L + j] = last;
    }
}

// Sum over the 64 lanes, returned in every lane.  Inside a row of 16 lanes the partial sums move
// through the data-parallel lane permutations of the vector ALU (two quad swaps, two row rotations:
// a few cycles each, no trip through the LDS crossbar); the four row sums are then read through scalar
// registers.  This chain sits on the critical path of every step of the long-window kernel.
template <int CTRL>
__device__ __forceinline__ float add_dpp(float v) {
    const int moved = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false);
    return v + __builtin_bit_cast(float, moved);
}
__device__ __forceinline__ float lane_value(float v, int src) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), src));
}
__device__ __forceinline__ float wave_sum(float v) {
    v = add_dpp<0xB1>(v);        // quad_perm [1,0,3,2]: lanes 1 apart
    v = add_dpp<0x4E>(v);        // quad_perm [2,3,0,1]: lanes 2 apart
    v = add_dpp<0x124>(v);       // row_ror 4
    v = add_dpp<0x128>(v);       // row_ror 8: every lane of a row holds the row's sum
    return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}

// The steps of slot I (64 I .. 64 I + 63) of the long-window kernel below, then those of the later slots:
// template recursion, so that every index into the history registers is a compile-time constant.
template <int I, int SLOTS, int SPW>
struct LongSlots {
    static constexpr int OFF = 64 * SLOTS;
    static __device__ __forceinline__ void run(float (&hist)[SPW][SLOTS], const float* P, int Q, int lane) {
        if (64 * I >= Q) return;                  // uniform
        const int tend = min(64, Q - 64 * I);
        for (int tt = 0; tt < tend; ++tt) {
            const float* pp = P + OFF + 64 * I + tt - lane;
            float acc[SPW];
#pragma unroll
            for (int s = 0; s < SPW; ++s) acc[s] = 0.0f;
#pragma unroll
            for (int ip = 0; ip <= I; ++ip) {
                const float pv = pp[-64 * ip];
#pragma unroll
                for (int s = 0; s < SPW; ++s) acc[s] = fmaf(pv, hist[s][ip], acc[s]);
            }
#pragma unroll
            for (int s = 0; s < SPW; ++s) {
                const float h = tanh_d(lane_value(hist[s][I], tt) + wave_sum(acc[s]));
                hist[s][I] = (lane == tt) ? h : hist[s][I];
            }
        }
        LongSlots<I + 1, SLOTS, SPW>::run(hist, P, Q, lane);
    }
};
template <int SLOTS, int SPW>
struct LongSlots<SLOTS, SLOTS, SPW> {
    static __device__ __forceinline__ void run(float (&)[SPW][SLOTS], const float*, int, int) {}
};

// Long windows (Q <= 64*SLOTS).  A wave owns SPW = 2 (sample, neuron) pairs of one neuron; lane l, slot i
// of `hist` belongs to step tau = 64 i + l (counted from 0).  Before step tau is taken the entry holds the
// input part u(tau) = x(tau) W[:, j] + b_j, afterwards h(tau).  The feedback sum of step tau is a dot
// product over all lanes and slots with the lag weights read from LDS at index OFF + tau - tau': the
// table is zero at and below OFF, so entries of steps not yet taken (tau' >= tau) drop out by themselves
// and the sum is one wavefront reduction per step and pair.  Q(Q-1)/2 multiply-adds per pair, as the cell
// defines it.  A step is a dependent chain (table reads, multiply-adds, reduction, tanh, write-back), so
// the rate comes from the number of waves a SIMD can interleave: the history registers (2 x SLOTS) are
// sized to the window.  The four waves of a work-group share the neuron, hence the lag table.
template <int SLOTS>
__device__ __forceinline__ void diag_long_body(
    const float* __restrict__ X, int64_t ldx_n, int64_t ldx_q, int64_t N, int Q, int d, int L,
    const float* __restrict__ Wt, const float* __restrict__ alpha, const float* __restrict__ bias,
    int lda, float* __restrict__ H) {
    constexpr int SPW = 2;
    constexpr int OFF = 64 * SLOTS;
    extern __shared__ float P[];                  // [OFF + Q]: P[OFF + k] = alpha[j][k-1], k = 1..Q-1, else 0
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = blockIdx.y;
    for (int idx = threadIdx.x; idx < OFF + Q; idx += 256) {
        const int k = idx - OFF;
        P[idx] = (k >= 1 && k <= Q - 1) ? alpha[(size_t)j * lda + (k - 1)] : 0.0f;
    }
    __syncthreads();

    const int64_t i0 = ((int64_t)blockIdx.x * 4 + wave) * SPW;
    const float bj = bias[j];
    float hist[SPW][SLOTS];
#pragma unroll
    for (int s = 0; s < SPW; ++s) {
        const int64_t irow = i0 + s < N ? i0 + s : N - 1;        // tail pairs repeat the last row
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) {
            const int tau = 64 * i + lane;
            float a = 0.0f;
            if (tau < Q) {
                a = bj;
                for (int c = 0; c < d; ++c) a = fmaf(load_x(X, ldx_n, ldx_q, irow, tau, c), Wt[(size_t)j * d + c], a);
            }
            hist[s][i] = a;
        }
    }

    LongSlots<0, SLOTS, SPW>::run(hist, P, Q, lane);

    // h(Q - 1) sits in lane (Q-1) % 64 of slot (Q-1) / 64
    const int qi = (Q - 1) >> 6, ql = (Q - 1) & 63;
#pragma unroll
    for (int s = 0; s < SPW; ++s) {
        float v = 0.0f;
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) v = (i == qi) ? hist[s][i] : v;
        v = lane_value(v, ql);
        if (lane == 0 && i0 + s < N) H[(size_t)(i0 + s) * L + j] = v;
    }
}

#define ELM_DIAG_LONG_ARGS                                                                              \
    const float *__restrict__ X, int64_t ldx_n, int64_t ldx_q, int64_t N, int Q, int d, int L,              \
        const float *__restrict__ Wt, const float *__restrict__ alpha, const float *__restrict__ bias, int lda, \
        float *__restrict__ H
__global__ __launch_bounds__(256) void diag_long16_kernel(ELM_DIAG_LONG_ARGS) {
    diag_long_body<16>(X, ldx_n, ldx_q, N, Q, d, L, Wt, alpha, bias, lda, H);
}
__global__ __launch_bounds__(256) void diag_long32_kernel(ELM_DIAG_LONG_ARGS) {
    diag_long_body<32>(X, ldx_n, ldx_q, N, Q, d, L, Wt, alpha, bias, lda, H);
}
// the paper's longest windows (3,197 steps)
__global__ __launch_bounds__(256) void diag_long52_kernel(ELM_DIAG_LONG_ARGS) {
    diag_long_body<52>(X, ldx_n, ldx_q, N, Q, d, L, Wt, alpha, bias, lda, H);
}
__global__ __launch_bounds__(256) void diag_long64_kernel(ELM_DIAG_LONG_ARGS) {
    diag_long_body<64>(X, ldx_n, ldx_q, N, Q, d, L, Wt, alpha, bias, lda, H);
}
#undef ELM_DIAG_LONG_ARGS

template <int SLOTS>
hipError_t launch_long(const float* X, int64_t ldx_n, int64_t ldx_q, int64_t N, int Q, int d, int L,
                       const float* Wt, const float* alpha, const float* bias, int lda, float* H,
                       hipStream_t stream) {
    const int64_t groups = (N + 7) / 8;           // 4 waves x 2 samples per work-group
    if (groups > 0x7fffffff || L > 65535) return hipErrorInvalidValue;
    const size_t lds = (size_t)(64 * SLOTS + Q) * sizeof(float);
    auto kern = SLOTS == 16 ? diag_long16_kernel : SLOTS == 32 ? diag_long32_kernel
              : SLOTS == 52 ? diag_long52_kernel : diag_long64_kernel;
    kern<<<dim3((unsigned)groups, (unsigned)L), 256, lds, stream>>>(X, ldx_n, ldx_q, N, Q, d, L, Wt, alpha, bias,
                                                                    lda, H);
    return hipGetLastError();
}

template <int QMAX, int JT>
hipError_t launch_reg(const float* X, int64_t ldx_n, int64_t ldx_q, int64_t N, int Q, int d, int L,
                      const float* Wt, const float* alpha, const float* bias, int lda, float* H,
                      dim3 grid, int jchunk, hipStream_t stream) {
    const size_t ot_bytes = (size_t)TILE * OT_STRIDE * sizeof(float);
    const size_t xs_bytes = (size_t)Q * d * XS_STRIDE * sizeof(float);
    if (ot_bytes + xs_bytes <= 144 * 1024) {
        auto kern = diag_reg_kernel<QMAX, JT, true>;
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)(ot_bytes + xs_bytes));
        if (e != hipSuccess) return e;
        kern<<<grid, 256, ot_bytes + xs_bytes, stream>>>(X, ldx_n, ldx_q, N, Q, d, L, Wt, alpha, bias, lda,
                                                         H, jchunk);
    } else {
        diag_reg_kernel<QMAX, JT, false><<<grid, 256, ot_bytes, stream>>>(X, ldx_n, ldx_q, N, Q, d, L, Wt,
                                                                          alpha, bias, lda, H, jchunk);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_hidden_diag(const float* Wt, const float* alpha, const float* bias, int lda,
                              const float* X, int64_t ldx_n, int64_t ldx_q, int64_t N, int Q, int d, int L,
                              float* H, hipStream_t stream) {
    if (N < 1 || Q < 1 || Q > kDiagMaxQ || Q > lda || d < 1 || L < 1) return hipErrorInvalidValue;
    const int64_t tiles = (N + TILE - 1) / TILE;
    if (tiles > 0x7fffffff) return hipErrorInvalidValue;
    // split the neurons over gridDim.y (in chunks of 32) until the launch has a few waves per CU
    const int jblocks = (L + 31) / 32;
    int64_t want = (2048 + tiles - 1) / tiles;
    int ysplit = (int)(want < 1 ? 1 : want > jblocks ? jblocks : want);
    const int jchunk = 32 * ((jblocks + ysplit - 1) / ysplit);
    ysplit = (L + jchunk - 1) / jchunk;
    const dim3 grid((unsigned)tiles, (unsigned)ysplit);
    if (Q <= 8) return launch_reg<8, 4>(X, ldx_n, ldx_q, N, Q, d, L, Wt, alpha, bias, lda, H, grid, jchunk, stream);
    if (Q <= 16) return launch_reg<16, 4>(X, ldx_n, ldx_q, N, Q, d, L, Wt, alpha, bias, lda, H, grid, jchunk, stream);
    if (Q <= 32) return launch_reg<32, 2>(X, ldx_n, ldx_q, N, Q, d, L, Wt, alpha, bias, lda, H, grid, jchunk, stream);
    if (Q <= 64) return launch_reg<64, 1>(X, ldx_n, ldx_q, N, Q, d, L, Wt, alpha, bias, lda, H, grid, jchunk, stream);
    if (Q > 3328) return launch_long<64>(X, ldx_n, ldx_q, N, Q, d, L, Wt, alpha, bias, lda, H, stream);
    if (Q > 2048) return launch_long<52>(X, ldx_n, ldx_q, N, Q, d, L, Wt, alpha, bias, lda, H, stream);
    if (Q > 1024) return launch_long<32>(X, ldx_n, ldx_q, N, Q, d, L, Wt, alpha, bias, lda, H, stream);
    if (Q > 128) return launch_long<16>(X, ldx_n, ldx_q, N, Q, d, L, Wt, alpha, bias, lda, H, stream);
    const size_t hs_bytes = (size_t)Q * 64 * sizeof(float);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(diag_lds_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)hs_bytes);
    if (e != hipSuccess) return e;
    diag_lds_kernel<<<grid, 64, hs_bytes, stream>>>(X, ldx_n, ldx_q, N, Q, d, L, Wt, alpha, bias, lda, H,
                                                    jchunk);
    return hipGetLastError();
}

}  // namespace elm
