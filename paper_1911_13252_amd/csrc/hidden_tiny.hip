// Stage 1 for layers of a few units (the paper's own experiments use M = 5 ... 20 hidden neurons): the
// recurrences of the paper's sections "Elman" / "Fully Connected RNN" (dense lag-1 form), "LSTM" and
// "GRU" on the vector ALU.
//
// A 32-column matrix-instruction tile is mostly padding for such layers and, worse, the point-wise gate
// math then runs on the padded columns too (at L = 10 only 10 of 32 lanes of a tile row are real units).
// Here a lane owns one sample: its state h (and c) lives in registers, the weights are wave-uniform and
// arrive as scalar operands of the multiply-adds, and all 64 lanes do useful work whatever L is.
// Measured against the matrix-instruction kernel at N = 10^6, Q = 50 (stage-1 ms, this kernel / that one):
// LSTM L = 5: 0.75 / 2.8, 10: 1.76 / 3.5, 20: 5.8 / 4.2; GRU 0.53 / 1.9, 1.55 / 2.4, 4.9 / 3.0; Elman
// 0.14 / 0.6, 0.36 / 0.8, 1.3 / 1.0 -- so it serves layers of up to 12 units.
// Weights are packed on the host as rows [b; W(0..d-1); U(0..LM-1)] of G*LM columns, zero padded from L to
// LM units (a padded unit stays exactly zero in all three cells and feeds nothing).

#include "internal.h"

namespace elm {
namespace {

__device__ __forceinline__ float sigmoid_t(float x) { return __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }
__device__ __forceinline__ float tanh_t(float x) { return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __expf(2.0f * x)); }

struct TinyArgs {
    const float* X;
    int64_t ldx_n, ldx_q;
    const float* Wp;      // [1 + d + LM][G*LM]
    const float* h0;
    const float* c0;
    float* H;
    float* C;
    int64_t N;
    int Q_run, d, L;
};

// pre[0 .. NC) += v * row[0 .. NC), row wave-uniform
template <int NC>
__device__ __forceinline__ void axpy_row(float (&pre)[NC], float v, const float* __restrict__ row) {
#pragma unroll
    for (int c = 0; c < NC; ++c) pre[c] = fmaf(v, row[c], pre[c]);
}

template <int CELL, int LM>
__global__ __launch_bounds__(256) void tiny_kernel(const TinyArgs p) {
    constexpr int G = (CELL == ELM_CELL_ELMAN) ? 1 : (CELL == ELM_CELL_LSTM) ? 4 : 3;
    constexpr int NC = G * LM;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t irow = i < p.N ? i : p.N - 1;          // tail lanes repeat the last sample
    const int d = p.d, L = p.L;
    const float* __restrict__ wb = p.Wp;                  // bias row
    const float* __restrict__ wx = p.Wp + NC;             // d input rows
    const float* __restrict__ wu = p.Wp + (size_t)(1 + d) * NC;   // LM recurrent rows
    const float* __restrict__ xrow = p.X + irow * p.ldx_n;

    float h[LM], c[LM];
#pragma unroll
    for (int k = 0; k < LM; ++k) {
        h[k] = (p.h0 != nullptr && k < L) ? p.h0[irow * L + k] : 0.0f;
        c[k] = (CELL == ELM_CELL_LSTM && p.c0 != nullptr && k < L) ? p.c0[irow * L + k] : 0.0f;
    }
    for (int t = 0; t < p.Q_run; ++t) {
        float pre[NC];
#pragma unroll
        for (int q = 0; q < NC; ++q) pre[q] = wb[q];
        const float* __restrict__ xt = xrow + (int64_t)t * p.ldx_q;
        for (int s = 0; s < d; ++s) axpy_row<NC>(pre, xt[s], wx + (size_t)s * NC);
        if (CELL == ELM_CELL_ELMAN) {
#pragma unroll
            for (int k = 0; k < LM; ++k) axpy_row<NC>(pre, h[k], wu + (size_t)k * NC);
#pragma unroll
            for (int j = 0; j < LM; ++j) h[j] = tanh_t(pre[j]);
        } else if (CELL == ELM_CELL_LSTM) {
#pragma unroll
            for (int k = 0; k < LM; ++k) axpy_row<NC>(pre, h[k], wu + (size_t)k * NC);
#pragma unroll
            for (int j = 0; j < LM; ++j) {                // column blocks (i, f, o, g)
                const float ig = sigmoid_t(pre[j]), fg = sigmoid_t(pre[LM + j]), og = sigmoid_t(pre[2 * LM + j]);
                const float gg = tanh_t(pre[3 * LM + j]);
                c[j] = fg * c[j] + ig * gg;
                h[j] = og * tanh_t(c[j]);
            }
        } else {
            // GRU, column blocks (z, r, n): z and r read h, the candidate reads r*h
#pragma unroll
            for (int k = 0; k < LM; ++k) {
                const float* __restrict__ row = wu + (size_t)k * NC;
#pragma unroll
                for (int q = 0; q < 2 * LM; ++q) pre[q] = fmaf(h[k], row[q], pre[q]);
            }
            float rh[LM];
#pragma unroll
            for (int j = 0; j < LM; ++j) rh[j] = sigmoid_t(pre[LM + j]) * h[j];
#pragma unroll
            for (int k = 0; k < LM; ++k) {
                const float* __restrict__ row = wu + (size_t)k * NC + 2 * LM;
#pragma unroll
                for (int j = 0; j < LM; ++j) pre[2 * LM + j] = fmaf(rh[k], row[j], pre[2 * LM + j]);
            }
#pragma unroll
            for (int j = 0; j < LM; ++j) {
                const float z = sigmoid_t(pre[j]);
                h[j] = (1.0f - z) * h[j] + z * tanh_t(pre[2 * LM + j]);
            }
        }
    }
    if (i < p.N) {
#pragma unroll
        for (int j = 0; j < LM; ++j)
            if (j < L) {
                p.H[i * L + j] = h[j];
                if (CELL == ELM_CELL_LSTM && p.C != nullptr) p.C[i * L + j] = c[j];
            }
    }
}

template <int CELL, int LM>
hipError_t launch_lm(const TinyArgs& a, hipStream_t stream) {
    const int64_t groups = (a.N + 255) / 256;
    if (groups > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL((tiny_kernel<CELL, LM>), dim3((unsigned)groups), dim3(256), 0, stream, a);
    return hipGetLastError();
}

template <int CELL>
hipError_t launch_cell(int lm, const TinyArgs& a, hipStream_t stream) {
    switch (lm) {
        case 2: return launch_lm<CELL, 2>(a, stream);
        case 4: return launch_lm<CELL, 4>(a, stream);
        case 6: return launch_lm<CELL, 6>(a, stream);
        case 8: return launch_lm<CELL, 8>(a, stream);
        case 10: return launch_lm<CELL, 10>(a, stream);
        case 12: return launch_lm<CELL, 12>(a, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

int tiny_padded_units(int cell, int L) {
    if (cell != ELM_CELL_ELMAN && cell != ELM_CELL_LSTM && cell != ELM_CELL_GRU) return 0;
    if (L > kTinyMaxL) return 0;
    return (L + 1) / 2 * 2;
}

size_t tiny_packed_floats(int cell, int d, int L) {
    const int lm = tiny_padded_units(cell, L);
    return lm == 0 ? 0 : (size_t)(1 + d + lm) * gates_of(cell) * lm;
}

void pack_weights_tiny(int cell, int d, int L, const float* W, const float* U, const float* b, float* out) {
    const int G = gates_of(cell), lm = tiny_padded_units(cell, L), NC = G * lm, GL = G * L;
    for (size_t q = 0; q < tiny_packed_floats(cell, d, L); ++q) out[q] = 0.0f;
    for (int g = 0; g < G; ++g)
        for (int j = 0; j < L; ++j) {
            out[g * lm + j] = b[g * L + j];
            for (int s = 0; s < d; ++s) out[(size_t)(1 + s) * NC + g * lm + j] = W[(size_t)s * GL + g * L + j];
            for (int k = 0; k < L; ++k) out[(size_t)(1 + d + k) * NC + g * lm + j] = U[(size_t)k * GL + g * L + j];
        }
}

hipError_t launch_hidden_tiny(int cell, int d, int L, const float* Wp, const float* X, int64_t ldx_n, int64_t ldx_q,
                              int64_t N, int Q_run, const float* h0, const float* c0, float* H, float* C,
                              hipStream_t stream) {
    const int lm = tiny_padded_units(cell, L);
    if (lm == 0 || N < 1) return hipErrorInvalidValue;
    TinyArgs a{X, ldx_n, ldx_q, Wp, h0, c0, H, C, N, Q_run, d, L};
    switch (cell) {
        case ELM_CELL_ELMAN: return launch_cell<ELM_CELL_ELMAN>(lm, a, stream);
        case ELM_CELL_LSTM:  return launch_cell<ELM_CELL_LSTM>(lm, a, stream);
        case ELM_CELL_GRU:   return launch_cell<ELM_CELL_GRU>(lm, a, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace elm
