// Stage 1: the hidden-matrix build H(Q) (step 2 of the paper's Algorithm "S-R-ELM").
//
// One work-group owns a tile of S = 32*MS windows for all Q steps.  Per step it evaluates the
// gate pre-activations  A_t = [x_t | 1 | h_{t-1}] . [W; b; U]  as a dense fp32 MFMA contraction
// (samples x K) . (K x G*L), then the cell's point-wise update (the paper's sections "Elman",
// "LSTM", "GRU").  The activation operand [x | 1 | h] lives in LDS for the whole unroll, the cell
// state c (and the freshly computed h until every wave has finished reading the old one) lives
// in registers, the weights stream from L2 in a pre-packed fragment order.  HBM is read once per
// window element and written once per H row.
//
// Differences from the paper's Opt-PR-ELM kernel (Algorithm "Opt-PR-ELM", one thread per
// (sample, neuron) with BSxBS shared-memory tiles): the per-step H(t) is never stored, the
// recurrence is a dense L x L lag-1 matrix (or, for the paper's fully connected cell, one dense matrix
// per lag over a ring of past states), and the tiling is by 64-lane wavefront MFMA tiles.

#include "hidden_kernel.h"

namespace elm {
namespace {

using namespace hk;

template <int CELL, int MS, int NCH, int STAGE, int WR = 1>
hipError_t launch_variant(const HiddenArgs& a, int64_t tiles, size_t lds_bytes, hipStream_t stream) {
    auto kern = hidden_kernel<CELL, MS, NCH, STAGE, WR>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(kThreads), lds_bytes, stream, a);
    return hipGetLastError();
}

// staged values per lane (1 KB of LDS per work-group each): 27 where the operand leaves that much room (the
// headline shape fills LDS to the byte with them), else 24
constexpr int kStage = 24, kStageMore = 27;

template <int CELL, int MS>
hipError_t launch_nch(int nch, const HiddenArgs& a, int64_t tiles, size_t lds, size_t lds_max,
                      hipStream_t s) {
    // the two-pass LSTM variants take the LDS staging when the operand leaves room for it
    constexpr bool kStaged = (CELL == ELM_CELL_LSTM) && MS == 2;
    const size_t staged = lds + (size_t)kStage * kThreads * sizeof(float);
    const size_t staged_more = lds + (size_t)kStageMore * kThreads * sizeof(float);
    const bool stage = kStaged && nch >= 3 && staged <= lds_max;
    const bool more = stage && staged_more <= lds_max;
    switch (nch) {
        case 1: return launch_variant<CELL, MS, 1, 0>(a, tiles, lds, s);
        case 2: return launch_variant<CELL, MS, 2, 0>(a, tiles, lds, s);
        case 3:
            if (stage) return launch_variant<CELL, MS, 3, kStaged ? kStage : 0>(a, tiles, staged, s);
            return launch_variant<CELL, MS, 3, 0>(a, tiles, lds, s);
        case 4:
            if (more) return launch_variant<CELL, MS, 4, kStaged ? kStageMore : 0>(a, tiles, staged_more, s);
            if (stage) return launch_variant<CELL, MS, 4, kStaged ? kStage : 0>(a, tiles, staged, s);
            return launch_variant<CELL, MS, 4, 0>(a, tiles, lds, s);
        default: return hipErrorInvalidValue;
    }
}

template <int CELL>
hipError_t launch_cell(int ms, int nch, const HiddenArgs& a, int64_t N, size_t lds_per_row,
                       size_t lds_max, hipStream_t s) {
    // narrow layers: one or two column blocks only, so the waves split the rows of a larger tile
    int wr = (a.nJB == 1) ? 4 : (a.nJB == 2) ? 2 : 1;
    if (lds_per_row * 32 * ms * wr > lds_max) wr = 1;
    // fewer tiles than compute units: halve the tile so that twice as many work-groups run; layers of
    // one column chunk (L <= 128; two chunks for Elman and GRU) also run 32-row blocks per wave: those
    // variants fit 256 registers, so two or more waves share a SIMD
    const bool two_waves = nch == 1 || (nch == 2 && CELL != ELM_CELL_LSTM);
    if (ms == 2 && ((N + 64 * wr - 1) / (64 * wr) < device_compute_units() || two_waves)) ms = 1;
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

}  // namespace

PackedLayout packed_layout(int cell, int d, int L, int ring) {
    PackedLayout lay{};
    lay.cell = cell;
    lay.d = d;
    lay.L = L;
    lay.G = gates_of(cell);
    lay.ring = ring;
    lay.K = ring * L + d + 1;
    lay.KG = (lay.K + 7) / 8;
    lay.R = 8 * lay.KG + 4;
    lay.nJB = (L + 31) / 32;
    // 4 extra k-groups: the contraction's look-ahead loads read (harmlessly) past the last group
    lay.copy_floats = ((size_t)lay.nJB * lay.KG + 4) * lay.G * 256;
    lay.floats = lay.copy_floats * ring;
    return lay;
}

// Fully connected multi-lag cell: `ring` rotations of the packed operand [W; b; A_k(0); A_k(1); ...].
// Rotation c is used at the steps t with t % ring == c, when history slot s holds the state of
// 1 + (c - 1 - s) mod ring steps ago; A is [Q][L][L] (lag k in block k-1).
void pack_weights_fc(const PackedLayout& lay, const float* W, const float* A, const float* b, float* out) {
    const int L = lay.L, d = lay.d, ring = lay.ring;
    for (size_t i = 0; i < lay.floats; ++i) out[i] = 0.0f;
    for (int c = 0; c < ring; ++c) {
        float* oc = out + (size_t)c * lay.copy_floats;
        for (int jb = 0; jb < lay.nJB; ++jb)
            for (int kg = 0; kg < lay.KG; ++kg)
                for (int lane = 0; lane < 64; ++lane)
                    for (int e = 0; e < 4; ++e) {
                        const int k = kg * 8 + (lane >> 5) * 4 + e;
                        const int j = jb * 32 + (lane & 31);
                        if (k >= lay.K || j >= L) continue;
                        float v;                      // operand rows: input, bias, history slots
                        if (k < d) {
                            v = W[(size_t)k * L + j];
                        } else if (k == d) {
                            v = b[j];
                        } else {
                            const int s = (k - d - 1) / L, m = (k - d - 1) - s * L;
                            const int lag = 1 + (((c - 1 - s) % ring) + ring) % ring;
                            v = A[((size_t)(lag - 1) * L + m) * L + j];
                        }
                        oc[(((size_t)jb * lay.KG + kg) * 64 + lane) * 4 + e] = v;
                    }
    }
}

void pack_weights(const PackedLayout& lay, const float* W, const float* U, const float* b, float* out) {
    const int L = lay.L, d = lay.d, G = lay.G, GL = G * L;
    for (size_t i = 0; i < lay.floats; ++i) out[i] = 0.0f;
    for (int jb = 0; jb < lay.nJB; ++jb)
        for (int kg = 0; kg < lay.KG; ++kg)
            for (int g = 0; g < G; ++g)
                for (int lane = 0; lane < 64; ++lane)
                    for (int e = 0; e < 4; ++e) {
                        const int k = kg * 8 + (lane >> 5) * 4 + e;
                        const int j = jb * 32 + (lane & 31);
                        if (k >= lay.K || j >= L) continue;
                        const int col = g * L + j;
                        float v;                      // operand rows: input, bias, recurrent
                        if (k < d) v = W[(size_t)k * GL + col];
                        else if (k == d) v = b[col];
                        else v = U[(size_t)(k - d - 1) * GL + col];
                        out[((((size_t)jb * lay.KG + kg) * G + g) * 64 + lane) * 4 + e] = v;
                    }
}

hipError_t launch_hidden(const PackedLayout& lay, const float* Wp, const float* X, int64_t ldx_n,
                         int64_t ldx_q, int64_t N, int Q_run, const float* h0, const float* c0,
                         float* H, float* C, hipStream_t stream) {
    int dev = 0, lds_max = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    e = hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
    if (e != hipSuccess) return e;

    const int nbuf = (lay.cell == ELM_CELL_GRU) ? 2 : 1;
    const size_t lds_per_row = (size_t)nbuf * lay.R * sizeof(float);
    int ms = 2;
    if (lds_per_row * 64 > (size_t)lds_max) ms = 1;
    if (lds_per_row * 32 > (size_t)lds_max) return hipErrorInvalidValue;
    const int nch = (lay.nJB + 3) / 4;

    HiddenArgs a{};
    a.X = X; a.ldx_n = ldx_n; a.ldx_q = ldx_q; a.Wp = Wp; a.h0 = h0; a.c0 = c0;
    a.H = H; a.C = C; a.N = N; a.Q_run = Q_run; a.d = lay.d; a.L = lay.L; a.R = lay.R;
    a.KG = lay.KG; a.nJB = lay.nJB; a.wp_bytes = (unsigned)(lay.floats * sizeof(float));
    a.ring = lay.ring; a.copy_bytes = (unsigned)(lay.copy_floats * sizeof(float));
    switch (lay.cell) {
        case ELM_CELL_ELMAN:
        case ELM_CELL_FC_MULTILAG:      // the Elman update on a ring of history slots
            return launch_cell<ELM_CELL_ELMAN>(ms, nch, a, N, lds_per_row, (size_t)lds_max, stream);
        case ELM_CELL_LSTM:  return launch_cell<ELM_CELL_LSTM>(ms, nch, a, N, lds_per_row, (size_t)lds_max, stream);
        case ELM_CELL_GRU:   return launch_cell<ELM_CELL_GRU>(ms, nch, a, N, lds_per_row, (size_t)lds_max, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace elm
