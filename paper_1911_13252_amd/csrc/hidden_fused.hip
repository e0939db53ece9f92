// Stages 1 and 2a in one kernel: every tile of H(Q) goes from LDS straight into the tall-skinny QR of
// [H | T] and is never stored (step 3 of the paper's Algorithm "S-R-ELM" uses H(Q) only through
// beta = H^+ T, and the R factor of [H | T] can absorb H a block of rows at a time).
//
// The grid is persistent: work-group b owns the R factor b of the TSQR's level 0 and takes the tiles
// b, b + gridDim.x, ...  After the last step of a tile the operand area of LDS is rewritten as the block
// [H(Q) | T | 0] and folded into R by the same code the TSQR kernel runs on blocks it loads from memory.
// Built for every stage-1 variant whose waves each own column blocks of all the tile's rows (layers
// wider than 64 units).  The variants that run one work-group per compute unit (LSTM wider than 128,
// Elman and GRU wider than 256 units) fold 64-row tiles (32 where two GRU operands fill the LDS); the
// narrower ones run two work-groups per compute unit, 32-row tiles, and their folds must fit the same
// 256 registers and half of the LDS.

#include "hidden_kernel.h"

namespace elm {
namespace {

using namespace hk;

template <int CELL, int MS, int NCH, int STAGE>
__global__ __launch_bounds__(kThreads, (MS == 1 && (NCH == 1 || (NCH == 2 && CELL != ELM_CELL_LSTM))) ? 2 : 1)
void hidden_fused_kernel(const HiddenArgs p) {
    extern __shared__ __align__(16) float lds[];
    float* Rw = p.Rout + (size_t)blockIdx.x * p.np * p.np;
    for (int idx = threadIdx.x; idx < p.np * p.np; idx += kThreads) Rw[idx] = 0.0f;
    __syncthreads();
    for (int64_t tile = blockIdx.x; tile < p.tiles; tile += gridDim.x)
        hidden_tile<CELL, MS, NCH, STAGE, 1, true>(p, tile, lds);
}

constexpr int kStage = 24;      // as in the plain kernel: 24 staged values per lane for the two-pass LSTM

struct Variant {
    void (*kern)(const HiddenArgs);
    int ms;
    int per_cu;            // work-groups per compute unit the variant is compiled for
    size_t stage_bytes;
};

// The stage-1 variant the plain launcher would pick for this layer when it has at least one tile per
// work-group slot; kern == nullptr where the waves split the rows (layers of at most 64 units), for the
// multi-lag cell and where the operand does not fit.
Variant pick_variant(const PackedLayout& lay, size_t lds_max) {
    Variant v{nullptr, 0, 1, 0};
    if (lay.ring != 1 || lay.nJB < 3) return v;
    const int nbuf = (lay.cell == ELM_CELL_GRU) ? 2 : 1;
    const size_t lds_per_row = (size_t)nbuf * lay.R * sizeof(float);
    if (lds_per_row * 32 > lds_max) return v;
    const int nch = (lay.nJB + 3) / 4;
    const bool lstm = lay.cell == ELM_CELL_LSTM;
    const bool two_waves = nch == 1 || (nch == 2 && !lstm);       // as in the plain launcher
    const int ms = (two_waves || lds_per_row * 64 > lds_max) ? 1 : 2;
    const size_t staged = (size_t)kStage * kThreads * sizeof(float);
    v.ms = ms;
    v.per_cu = two_waves ? 2 : 1;
    switch (lay.cell) {
        case ELM_CELL_LSTM:
            if (nch == 1) v.kern = hidden_fused_kernel<ELM_CELL_LSTM, 1, 1, 0>;
            else if (ms != 2) return v;
            else if (nch == 2) v.kern = hidden_fused_kernel<ELM_CELL_LSTM, 2, 2, 0>;
            else if (lds_per_row * 64 + staged > lds_max) return v;
            else {
                v.stage_bytes = staged;
                v.kern = (nch == 3) ? hidden_fused_kernel<ELM_CELL_LSTM, 2, 3, kStage>
                                    : hidden_fused_kernel<ELM_CELL_LSTM, 2, 4, kStage>;
            }
            return v;
        case ELM_CELL_ELMAN:
            if (nch == 1) v.kern = hidden_fused_kernel<ELM_CELL_ELMAN, 1, 1, 0>;
            else if (nch == 2) v.kern = hidden_fused_kernel<ELM_CELL_ELMAN, 1, 2, 0>;
            else if (ms != 2) return v;
            else v.kern = (nch == 3) ? hidden_fused_kernel<ELM_CELL_ELMAN, 2, 3, 0> : hidden_fused_kernel<ELM_CELL_ELMAN, 2, 4, 0>;
            return v;
        case ELM_CELL_GRU:
            if (nch == 1) v.kern = hidden_fused_kernel<ELM_CELL_GRU, 1, 1, 0>;
            else if (nch == 2) v.kern = hidden_fused_kernel<ELM_CELL_GRU, 1, 2, 0>;
            // two operand buffers: 64-row tiles fit only up to about 300 units (three column chunks)
            else if (ms == 2 && nch != 3) return v;
            else if (ms == 2) v.kern = hidden_fused_kernel<ELM_CELL_GRU, 2, 3, 0>;
            else v.kern = (nch == 3) ? hidden_fused_kernel<ELM_CELL_GRU, 1, 3, 0> : hidden_fused_kernel<ELM_CELL_GRU, 1, 4, 0>;
            return v;
        default: return v;
    }
}

struct Launch {
    Variant v;
    size_t lds;
};

hipError_t plan_launch(const PackedLayout& lay, int m, Launch* out, int* compute_units) {
    int dev = 0, lds_max = 0, cus = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    e = hipDeviceGetAttribute(&lds_max, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
    if (e != hipSuccess) return e;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    *compute_units = cus;
    out->v = pick_variant(lay, (size_t)lds_max);
    out->lds = 0;
    if (out->v.kern == nullptr) return hipSuccess;
    const int S = 32 * out->v.ms;
    const int np = (lay.L + m + 31) / 32 * 32;
    const int nbuf = (lay.cell == ELM_CELL_GRU) ? 2 : 1;
    const size_t hidden_lds = (size_t)nbuf * lay.R * sizeof(float) * S + out->v.stage_bytes;
    const size_t fold_lds = fold::lds_floats(np, S) * sizeof(float);
    out->lds = hidden_lds > fold_lds ? hidden_lds : fold_lds;
    if (out->lds > (size_t)lds_max / out->v.per_cu) out->v.kern = nullptr;
    return hipSuccess;
}

}  // namespace

int hidden_fused_groups(const PackedLayout& lay, int64_t N, int m, int* per_cu) {
    Launch l{};
    int cus = 0;
    if (plan_launch(lay, m, &l, &cus) != hipSuccess || l.v.kern == nullptr || cus < 1) return 0;
    if (per_cu != nullptr) *per_cu = l.v.per_cu;
    const int64_t tiles = (N + 32 * l.v.ms - 1) / (32 * l.v.ms);
    int64_t groups = (int64_t)l.v.per_cu * cus;
    if (groups > 1024) groups = 1024;
    return (int)(groups < tiles ? groups : tiles);
}

bool hidden_fused_available(const PackedLayout& lay, const SolvePlan& pl) {
    return hidden_fused_groups(lay, pl.N, pl.m) > 0;
}

hipError_t launch_hidden_fused(const PackedLayout& lay, const float* Wp, const float* X, int64_t ldx_n,
                               int64_t ldx_q, int64_t N, int Q, const float* T, const SolvePlan& pl, void* ws,
                               hipStream_t stream) {
    Launch l{};
    int cus = 0;
    hipError_t e = plan_launch(lay, pl.m, &l, &cus);
    if (e != hipSuccess) return e;
    if (l.v.kern == nullptr || pl.L != lay.L || pl.N != N || pl.groups[0] != hidden_fused_groups(lay, N, pl.m))
        return hipErrorInvalidValue;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(l.v.kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)l.lds);
    if (e != hipSuccess) return e;
    const int S = 32 * l.v.ms;
    HiddenArgs a{};
    a.X = X; a.ldx_n = ldx_n; a.ldx_q = ldx_q; a.Wp = Wp; a.h0 = nullptr; a.c0 = nullptr;
    a.H = nullptr; a.C = nullptr; a.N = N; a.Q_run = Q; a.d = lay.d; a.L = lay.L; a.R = lay.R;
    a.KG = lay.KG; a.nJB = lay.nJB; a.wp_bytes = (unsigned)(lay.floats * sizeof(float));
    a.ring = 1; a.copy_bytes = (unsigned)(lay.copy_floats * sizeof(float));
    a.T = T; a.m = pl.m; a.np = pl.np; a.ldb = pl.np + 1;
    a.Rout = reinterpret_cast<float*>(static_cast<char*>(ws) + pl.off_R[0]);
    a.tiles = (N + S - 1) / S;
    // one work-group per level-0 R factor of the plan; the combine levels then run as usual
    hipLaunchKernelGGL(l.v.kern, dim3(pl.groups[0]), dim3(kThreads), l.lds, stream, a);
    return hipGetLastError();
}

}  // namespace elm
