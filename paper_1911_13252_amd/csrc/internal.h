// Internal declarations shared by the translation units of libelmrnn (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

#include "elm_rnn.h"

namespace elm {

// Geometry of the packed weight operand [U; W; b] (K x G*L) as the hidden-matrix kernel reads it.
struct PackedLayout {
    int cell, d, L, G;
    int ring;     // history slots of L columns in the operand row (1 except for the fully connected multi-lag cell)
    int K;        // ring*L + d + 1 contraction rows: recurrent, input, bias
    int KG;       // k-groups of 8 rows (ceil(K / 8))
    int R;        // LDS row stride of the activation operand, 8*KG + 4 floats
    int nJB;      // hidden-unit blocks of 32 columns (ceil(L / 32))
    size_t copy_floats;   // one packed operand including the prefetch tail
    size_t floats;        // whole buffer: `ring` rotations of the operand
};

inline int gates_of(int cell) { return cell == ELM_CELL_LSTM ? 4 : cell == ELM_CELL_GRU ? 3 : 1; }
PackedLayout packed_layout(int cell, int d, int L, int ring = 1);

// Pack host W (d x GL), U (L x GL), b (GL) into the kernel's fragment order.
void pack_weights(const PackedLayout& lay, const float* W, const float* U, const float* b, float* out);
// Same for the fully connected multi-lag cell: A is [Q][L][L], lay.ring rotations are written.
void pack_weights_fc(const PackedLayout& lay, const float* W, const float* A, const float* b, float* out);
constexpr int kFcMaxK = 1272;      // contraction rows a 32-sample tile of the multi-lag cell can hold in LDS

// ---- the fully connected multi-lag cell when the history of a window does not fit LDS: a launch per step,
// the past states of a pass of rows kept in scratch memory that the caller's workspace provides
struct FcStepLayout {
    int Q, d, L;
    int ring;             // history slots per row (Q - 1, at least 1)
    int Lk;               // slot width: L rounded up to 8 columns
    int nJB;              // hidden-unit blocks of 32 columns
    int KGtot;            // k-groups of 8 rows in the stack [A_{Q-1}; ...; A_1; W; b]
    int KGpad;            // ... plus the zero groups the contraction may run or look into
    size_t floats;        // packed stack: nJB * KGpad * 256
    int64_t chunk_rows;   // most rows a pass takes (a multiple of 256, at most 65,536)
    int NU;               // 16-column units of the row-split kernel (layers of 65 to 96 units), else 0
    size_t floats16;      // the stack packed per unit: NU * KGpad * 128
};
// false: the shape is out of range (stack of 4 GiB or more, or a history row of 8 MiB or more)
bool fc_step_layout(int Q, int d, int L, FcStepLayout* out);
void pack_weights_fc_steps(const FcStepLayout& lay, const float* W, const float* A, const float* b, float* out);
void pack_weights_fc_rows(const FcStepLayout& lay, const float* W, const float* A, const float* b, float* out);
// Scratch of one call over N rows: the history of a pass ([slot][row][Lk]) followed by the carried / split
// sums.  bytes does not decrease when N grows, so the scratch for a chunk of rows also serves shorter ones.
struct FcScratch {
    int64_t pass_rows;    // min(N rounded up to 256, lay.chunk_rows)
    size_t hist_floats;   // pass_rows * ring * Lk
    size_t sums_floats;
    size_t off_sums;      // byte offset of the sums (256-byte aligned)
    size_t bytes;
};
FcScratch fc_scratch(const FcStepLayout& lay, int64_t N);
// scratch: fc_scratch(lay, N).bytes of device memory, contents destroyed
// Wp16: the per-unit packing (lay.floats16) where lay.NU > 0, else null
hipError_t launch_hidden_fc_steps(const FcStepLayout& lay, const float* Wp, const float* Wp16, void* scratch,
                                  const float* X, int64_t ldx_n, int64_t ldx_q, int64_t N, int Q_run, float* H,
                                  hipStream_t stream);

hipError_t launch_hidden(const PackedLayout& lay, const float* Wp, const float* X, int64_t ldx_n,
                         int64_t ldx_q, int64_t N, int Q_run, const float* h0, const float* c0,
                         float* H, float* C, hipStream_t stream);

// ---- layers of a few units on the vector ALU (a lane per sample); float32 contraction only
constexpr int kTinyMaxL = 12;
int tiny_padded_units(int cell, int L);                 // 0: no such kernel for this cell / width
size_t tiny_packed_floats(int cell, int d, int L);
void pack_weights_tiny(int cell, int d, int L, const float* W, const float* U, const float* b, float* out);
hipError_t launch_hidden_tiny(int cell, int d, int L, const float* Wp, const float* X, int64_t ldx_n, int64_t ldx_q,
                              int64_t N, int Q_run, const float* h0, const float* c0, float* H, float* C,
                              hipStream_t stream);

// Spectral radius of a row-major n x n float64 host matrix, computed on the current device; every launch
// and copy goes to `stream`, which is synchronised before the function returns.
hipError_t spectral_radius_device(const double* A, int n, double* rho_out, hipStream_t stream);
// compute units of the current device (256 when the query fails: the launch heuristics only need a scale)
int device_compute_units();

// ---- fast contraction mode (fp16 hi/lo split of the recurrent part, bf16 x 3 split of the input part)
struct SplitLayout {
    int cell, d, L, G;
    int KGh;        // recurrent groups of 16 rows (ceil(L / 16))
    int KGs;        // stream positions per column block: 2 for the input group + KGh
    int nJB;        // hidden-unit blocks of 32 columns
    int stride;     // LDS operand row stride in bytes
    int xoff;       // byte offset of the input group inside an operand row
    int log2_su;    // recurrent weights are scaled by 2^log2_su before the fp16 split
    float inv_scale;   // 1 / (2^13 * 2^log2_su): accumulator -> pre-activation
    size_t bytes;   // packed buffer length including the prefetch tail
    bool ok;        // false: this model cannot use the mode (d > 15, non-finite or out-of-range weights)
};
SplitLayout split_layout(int cell, int d, int L, const float* W, const float* U, const float* b);
void pack_weights_split(const SplitLayout& lay, const float* W, const float* U, const float* b, void* out);
hipError_t launch_hidden_split(const SplitLayout& lay, const void* Wp, const float* X, int64_t ldx_n,
                               int64_t ldx_q, int64_t N, int Q_run, const float* h0, const float* c0,
                               float* H, float* C, hipStream_t stream);

// The paper's own Elman cell (diagonal, multi-lag feedback).  Wt is W transposed [L][d], alpha is
// [L][lda] with lag k in column k-1, Q <= lda steps are run.
constexpr int kDiagMaxQ = 4096;
hipError_t launch_hidden_diag(const float* Wt, const float* alpha, const float* bias, int lda,
                              const float* X, int64_t ldx_n, int64_t ldx_q, int64_t N, int Q, int d, int L,
                              float* H, hipStream_t stream);

// ---- stage 2 -------------------------------------------------------------------------------
struct SolvePlan {
    int64_t N;
    int L, m, n, np;       // n = L + m columns, np = n rounded up to 32
    int block_rows;        // rows per folded block (64 or 128)
    int levels;            // number of fold launches (level 0 + combine levels)
    int groups[12];        // work-groups (= R factors produced) per level
    size_t off_R[2];       // ping-pong R-factor stacks (bytes from workspace base)
    size_t off_part;       // per-work-group partial sums of the residual pass (doubles)
    size_t off_small;      // beta64, gradient, scalars (doubles)
    size_t bytes;
};
// level0_groups > 0 fixes the number of level-0 R factors (at most 1024); 0 = chosen from N
SolvePlan make_solve_plan(int64_t N, int L, int m, int level0_groups = 0);

hipError_t launch_tsqr(const SolvePlan& plan, const float* H, const float* T, void* ws,
                       float** R_final, hipStream_t stream);
// The two halves of launch_tsqr, for callers that hand the rows over in chunks.
hipError_t launch_tsqr_level0(const SolvePlan& plan, const float* H, const float* T, int64_t rows, void* ws,
                              int keep, hipStream_t stream);
hipError_t launch_tsqr_combine(const SolvePlan& plan, void* ws, float** R_final, hipStream_t stream);
// Stage 1 and level 0 of the TSQR in one kernel (H is never stored), for the layers whose stage-1 variant
// runs one work-group per compute unit; the R factors land where launch_tsqr_level0 would put them.
// hidden_fused_groups: the persistent grid the fused kernel wants for N rows (work-groups per compute unit of
// its variant x compute units, at most one per tile), 0 where no fused variant exists; the plan passed to
// launch_hidden_fused must have been made with that many level-0 groups.  *per_cu receives the variant's
// work-groups per compute unit.
int hidden_fused_groups(const PackedLayout& lay, int64_t N, int m, int* per_cu = nullptr);
bool hidden_fused_available(const PackedLayout& lay, const SolvePlan& plan);
hipError_t launch_hidden_fused(const PackedLayout& lay, const float* Wp, const float* X, int64_t ldx_n,
                               int64_t ldx_q, int64_t N, int Q, const float* T, const SolvePlan& plan,
                               void* ws, hipStream_t stream);
hipError_t launch_backsolve(const SolvePlan& plan, const float* R, void* ws, hipStream_t stream);
hipError_t launch_residual_pass(const SolvePlan& plan, const float* H, const float* T, void* ws,
                                hipStream_t stream);
hipError_t launch_residual_chunk(const SolvePlan& plan, const float* H, const float* T, int64_t rows, void* ws,
                                 int accumulate, hipStream_t stream);
hipError_t launch_residual_finish(const SolvePlan& plan, void* ws, hipStream_t stream);
hipError_t launch_refine_update(const SolvePlan& plan, const float* R, void* ws, hipStream_t stream);
hipError_t launch_export_beta(const SolvePlan& plan, void* ws, float* beta32, double* beta64,
                              hipStream_t stream);
hipError_t launch_predict_gemv(const float* H, const double* beta64, int64_t N, int L, int m,
                               float* Y, hipStream_t stream);

// Stage 2 on `stream` with a plan the caller made; ws (device) holds plan.bytes.  Arguments as elm_rnn_solve;
// hidden_done (nullable) is an event recorded when stage 1 ended, from which the solve time is then measured.
int run_solve_with_plan(const SolvePlan& plan, const float* H, const float* T, int refine, float* beta_out,
                        double* beta64_out, elm_rnn_stats* stats, void* ws, hipStream_t stream,
                        double hidden_ms, hipEvent_t hidden_done);

// layout of the "small" double area of the solve workspace
struct SmallArea {
    static constexpr int BETA = 0;                 // L*m      current beta (float64)
    __host__ __device__ static size_t grad(int L, int m) { return (size_t)L * m; }            // L*m   H^T r
    __host__ __device__ static size_t scal(int L, int m) { return (size_t)2 * L * m; }        // 8 scalars:
    // [0] rss  [1] sum H^2  [2] ||g||^2  [3] rss from R22  [4] min|Rjj|  [5] max|Rjj|  [6] rank flag
    __host__ __device__ static size_t doubles(int L, int m) { return (size_t)2 * L * m + 8; }
};

void set_hip_error(hipError_t e, const char* where);
void set_error_text(const char* text);      // what elm_rnn_last_hip_error() then returns

}  // namespace elm

#define ELM_HIP_TRY(expr)                                   \
    do {                                                    \
        hipError_t e__ = (expr);                            \
        if (e__ != hipSuccess) {                            \
            elm::set_hip_error(e__, #expr);                 \
            return ELM_EHIP;                                \
        }                                                   \
    } while (0)
