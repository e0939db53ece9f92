/*
 * elm_rnn.h -- C ABI of the MI355X (gfx950) ELM-RNN fit library.
 *
 * Non-iterative training of a recurrent network (the paper's Algorithm
 * "S-R-ELM"): (1) input, recurrent and bias weights are drawn once from a seed
 * and frozen; (2) every training window is unrolled over Q steps through the
 * cell and its final hidden state becomes one row of H (N x L); (3) the output
 * weights are beta = H^+ T, computed here as the least-squares solution by a
 * Householder tall-skinny QR of [H | T] and a triangular back-solve (the
 * paper's section "Computing beta").
 *
 * General conventions
 *   - Every function returns 0 (ELM_OK) or a negative error code; nothing
 *     throws across this boundary.  elm_rnn_strerror() names a code and
 *     elm_rnn_last_hip_error() returns the text of the calling thread's last
 *     HIP failure (or the reason of its last ELM_EUNSUPPORTED, where one is given).
 *   - "device" pointers are HIP device memory on the current device, owned by
 *     the caller; the library never frees them and allocates no O(N) memory.
 *     "host" pointers are ordinary memory.  A model owns only its weight
 *     and beta buffers on the device (the packed lag matrices of the multi-lag
 *     cell are its largest: Q L^2 floats); every scratch buffer whose size
 *     grows with N comes from the caller's workspace, so calls on one model
 *     with different workspaces may overlap in time.
 *   - All device work of the functions that take hip_stream (a hipStream_t
 *     cast to void*, NULL = the default stream) is enqueued on that stream,
 *     the weight generation inside the two fit functions included.  Functions
 *     that return values to the host (stats) synchronise it before returning.
 *     The functions without a stream argument (model creation, weight and
 *     beta copies) use synchronous copies and, for Elman layers of 64 units
 *     or more with a spectral-radius target, kernels on the default stream,
 *     and return when their work is done.
 *   - Matrices are row-major float32 unless stated.  X[i, t, :] (sample i, step
 *     t, d contiguous channels) lives at X + i*ldx_n + t*ldx_q (strides in
 *     elements): materialised windows use ldx_n = Q*d, ldx_q = d; zero-copy
 *     sliding windows over a series use ldx_n = stride*d, ldx_q = d.  This is
 *     the paper's n x S x Q input with the step axis moved before the feature
 *     axis so that one step of one sample is contiguous.
 *   - Weight layout: W is d x kL, U is L x kL, b is kL with k gate blocks side
 *     by side: Elman k = 1; LSTM k = 4 in the order (i, f, o, g) = the paper's
 *     (in, lambda, o, candidate); GRU k = 3 in the order (z, r, n).  For
 *     ELM_CELL_ELMAN_DIAG k = 1 and U is the L x Q lag-weight matrix alpha; for
 *     ELM_CELL_FC_MULTILAG k = 1 and U is the Q x L x L stack of lag matrices.
 *   - Supported sizes: 1 <= L <= 512, 1 <= d <= 64, 1 <= m <= 16, N >= 1.
 */
#ifndef ELM_RNN_H
#define ELM_RNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ELM_CELL_ELMAN 0   /* h_t = tanh(x_t W + h_{t-1} U + b): dense lag-1 form of the paper's
                              "Fully Connected RNN" / "Elman" recurrences                        */
#define ELM_CELL_LSTM  1   /* the paper's section "LSTM" (no peepholes)                          */
#define ELM_CELL_GRU   2   /* the paper's section "GRU": f = (1-z) f_prev + z tanh(W x + U (r f_prev) + b) */

#define ELM_CELL_ELMAN_DIAG 3 /* the paper's section "Elman" as printed (Eq. hij_elman): neuron j feeds
                                back on itself only, from every earlier step of the window:
                                h_j(t) = tanh(x(t) W[:,j] + b_j + sum_{k=1}^{t-1} alpha[j][k-1] h_j(t-k));
                                its recurrent array "U" is alpha, L x Q (lag k in column k-1), Q <= 4096;
                                no initial state can be passed and Q_run <= Q                        */

#define ELM_CELL_FC_MULTILAG 4 /* the paper's section "Fully Connected RNN" (Eq. hij_fc): every neuron is fed
                                by every neuron's output of all earlier steps of the window:
                                h(t) = tanh(x(t) W + b + sum_{k=1}^{t-1} h(t-k) A_k);
                                its recurrent array "U" is A, Q x L x L (A[k-1][m][j]: neuron m, k steps
                                ago, into neuron j; the last block is never used); no initial state,
                                Q_run <= Q.  While the history of a window is short (max(Q-1,1)*L + d + 1
                                <= 1272, and <= 640 for L <= 64) it stays on chip for all steps; beyond
                                that every step is a launch of its own over a buffer of past states in
                                the caller's workspace (elm_rnn_hidden_workspace_bytes: below 2 GiB, room
                                for up to 65,536 rows, more rows are taken in passes).
                                ELM_EUNSUPPORTED if a window's history reaches 8 MiB or the packed lag
                                matrices 4 GiB                                                       */

/* How the dense cells carry the recurrent contraction h_{t-1} U of each step (the input part x_t W + b
 * and all point-wise work are float32-exact in both):
 *   ELM_CONTRACT_FP32    float32 matrix instructions (the default);
 *   ELM_CONTRACT_SPLIT16 every float32 operand value is split into an fp16 pair hi + lo (22 significant
 *                        bits) and the product is taken as hi*hi + hi*lo + lo*hi on fp16 matrix
 *                        instructions with float32 accumulation: float32-equivalent results (the
 *                        dropped term is 2^-22 relative) at several times the throughput.  Needs
 *                        d <= 15 and finite weights; |h0| must stay below 8 (states produced by the
 *                        cells lie in [-1, 1]). */
#define ELM_CONTRACT_FP32    0
#define ELM_CONTRACT_SPLIT16 1

#define ELM_OK            0
#define ELM_EINVAL       -1   /* null pointer, non-positive size, unknown cell, N < L for a solve */
#define ELM_EWORKSPACE   -2   /* workspace pointer null or smaller than the *_workspace_bytes()   */
#define ELM_ERANK        -3   /* H numerically rank deficient: min|R_jj| <= eps32 * max|R_jj|;
                                 beta is still written but must not be trusted                   */
#define ELM_EHIP         -4   /* a HIP call failed; see elm_rnn_last_hip_error()                  */
#define ELM_EUNSUPPORTED -5   /* size outside the supported range listed above                    */

typedef struct elm_rnn_model elm_rnn_model;   /* opaque; from *_create or fit, released by elm_rnn_free */

/* How step (1) of Algorithm "S-R-ELM" (the random assignment of the input, recurrent and bias
 * weights) draws its values.  A SplitMix64 stream seeded with `seed` yields u in [0,1) with 53 bits; each value is
 * (2u-1)*w_scale in double; draw order W (row-major), U (row-major), b; then
 *   spectral_radius > 0 (Elman only): U *= spectral_radius / max|eig(U)|
 *   zero_bias != 0: b = 0 (the draws are still consumed), else
 *   LSTM: forget_bias is added to the forget block of b;
 * finally everything is rounded to float32. */
typedef struct {
    double w_scale;
    double spectral_radius;
    double forget_bias;
    int    zero_bias;
    int    contraction;   /* ELM_CONTRACT_*: how models made from this init run the recurrence */
} elm_rnn_init;

/* Filled by elm_rnn_solve / elm_rnn_fit (host memory). */
typedef struct {
    double t_hidden_ms;   /* stage 1 (hidden-matrix build), device time; 0 from elm_rnn_solve     */
    double t_solve_ms;    /* stage 2 (TSQR + back-solve + refinement), device time                */
    double rmse;          /* sqrt(sum (H beta - T)^2 / (N m)) of the returned beta, from a float64
                             residual pass over H                                                 */
    double rmse_qr;       /* the same quantity read off the float32 R factor: ||R22||_F/sqrt(N m) */
    double ne_resid;      /* ||H^T (H beta - T)||_F / (||H||_F ||H beta - T||_F), float64          */
    double r_diag_min;    /* min and max |R_jj| over the L columns of H (condition indicator)      */
    double r_diag_max;
    int    refine_iters;  /* float64-residual refinement steps applied to beta                     */
} elm_rnn_stats;

/* ---- step (1): weights -------------------------------------------------------------------- */

/* Draw the weights for (cell, d, L) from `seed` on the host as described at elm_rnn_init, and
 * upload them.  Q is the default number of steps, m the number of outputs (beta is L x m, zero
 * until a fit stores it).  *model_out receives the new model. */
int elm_rnn_model_create(int cell, int Q, int d, int L, int m, uint64_t seed,
                         const elm_rnn_init* init, elm_rnn_model** model_out);

/* Same, but with caller-supplied float32 host weights W[d*kL], U[L*kL] (alpha[L*Q] for
 * ELM_CELL_ELMAN_DIAG, A[Q*L*L] for ELM_CELL_FC_MULTILAG), b[kL] (copied). */
int elm_rnn_model_create_from_weights(int cell, int Q, int d, int L, int m,
                                      const float* W, const float* U, const float* b,
                                      elm_rnn_model** model_out);

/* Switch an existing model between the contraction modes (ELM_CONTRACT_*).  Returns
 * ELM_EUNSUPPORTED, leaving the model unchanged, if it cannot run the requested mode. */
int elm_rnn_model_set_contraction(elm_rnn_model* model, int contraction);

/* Copy the model's weights to host arrays (any of W, U, b, beta64 may be NULL).  beta64 is the
 * L x m float64 output-weight matrix.  Synchronous. */
int elm_rnn_get_weights(const elm_rnn_model* model, float* W, float* U, float* b, double* beta64);

/* Store output weights (host, L x m float64) into the model, e.g. to predict with a loaded beta. */
int elm_rnn_set_beta(elm_rnn_model* model, const double* beta64);

void elm_rnn_free(elm_rnn_model* model);

/* ---- step (2): H(Q) ------------------------------------------------------------------------ */

/* Device scratch elm_rnn_hidden needs for N rows of a (cell, Q, d, L) model: 0 for every cell whose
 * per-step states stay on chip, i.e. all but ELM_CELL_FC_MULTILAG beyond its on-chip limit, where it is
 * the history of a pass of rows (min(N rounded up to 256, 65,536) x (Q-1) x L rounded up to 8 floats)
 * plus carried sums.  It never decreases when N grows.  0 also for unsupported sizes. */
size_t elm_rnn_hidden_workspace_bytes(int cell, int64_t N, int Q, int d, int L);

/* Unroll N windows through the model's cell for Q_run steps (1 <= Q_run; X must hold that many
 * steps) and write the final hidden state of sample i to H_out[i*L .. i*L+L) (device).  h0 / c0
 * (device, N x L, nullable = zero) give the state before the first step; c0 and c_out (nullable)
 * are used by the LSTM only.  Only H(Q) is produced: for the lag-1 cells the per-step states never
 * leave the chip (step 3 of Algorithm "S-R-ELM" uses H(Q) alone).  workspace (device, contents
 * destroyed) must hold elm_rnn_hidden_workspace_bytes() for the model's sizes and N, else
 * ELM_EWORKSPACE; it may be NULL where that is 0.  The model is only read: calls with different
 * workspaces and outputs may run concurrently on different streams. */
int elm_rnn_hidden(const elm_rnn_model* model, const float* X, int64_t ldx_n, int64_t ldx_q,
                   int64_t N, int Q_run, const float* h0, const float* c0,
                   float* H_out, float* c_out, void* workspace, size_t workspace_bytes,
                   void* hip_stream);

/* ---- step (3): beta = H^+ T ---------------------------------------------------------------- */

/* Device workspace elm_rnn_solve needs for an N x L system with m right-hand sides. */
size_t elm_rnn_solve_workspace_bytes(int64_t N, int L, int m);

/* Least squares min ||H beta - T||_F for device H (N x L) and T (N x m), N >= L.
 * Blocked Householder TSQR of [H | T] in float32 (the paper's H = QR, z = Q^T Y), back
 * substitution R beta = z, then `refine` steps of iterative refinement whose residual T - H beta
 * and gradient H^T r are accumulated in float64: refine = 0..4 steps, or -1 = two steps if
 * max|R_jj| > 30 min|R_jj| (the normal-equation residual of the unrefined solution is about
 * 1e-8 .. 6e-8 times that ratio) and none otherwise.  One more pass over H gives the statistics
 * of the returned beta.
 * beta_out (device, L x m float32) and beta64_out (device, L x m float64, nullable) receive
 * the result; stats (host, nullable) is filled after a stream synchronisation.
 * Returns ELM_ERANK (after writing outputs) if H is numerically rank deficient. */
int elm_rnn_solve(const float* H, const float* T, int64_t N, int L, int m, int refine,
                  float* beta_out, double* beta64_out, elm_rnn_stats* stats,
                  void* workspace, size_t workspace_bytes, void* hip_stream);

/* The same solve for callers that cannot allocate device memory or obtain a workspace: code running under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Everything elm_rnn_solve keeps
 * in its workspace (R factors, partial sums, the small float64 area) lives in a static device array of
 * ELM_RNN_STATIC_SCRATCH_BYTES that every GPU the library runs on holds from the load of the library until
 * the process ends; the call allocates nothing (no hipMalloc / hipFree, no library that does).  Arguments and
 * results as elm_rnn_solve.  Where the default number of level-0 R factors does not fit the array it is
 * halved until it does (same result up to float32 rounding, longer run time: cfg-sized examples are
 * 384 factors at L + m <= 160, 96 at 288, 48 at 544); ELM_EUNSUPPORTED, with the reason in
 * elm_rnn_last_hip_error(), if even one R factor plus the 1024 x (L m + 2) float64 partial sums do not fit
 * (e.g. L = 512 with m = 16).  All calls on one GPU share that GPU's array, which keeps the last call's
 * contents (nothing in it needs clearing between calls): calls that overlap in time on one GPU race and
 * must be serialised by the caller, e.g. by using one stream. */
#define ELM_RNN_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
size_t elm_rnn_solve_static_scratch_bytes(void);
int elm_rnn_solve_static(const float* H, const float* T, int64_t N, int L, int m, int refine,
                         float* beta_out, double* beta64_out, elm_rnn_stats* stats, void* hip_stream);

/* ---- the whole fit -------------------------------------------------------------------------- */

/* Workspace for elm_rnn_fit: the solve workspace, plus N*L floats when H_out is NULL, plus
 * elm_rnn_hidden_workspace_bytes(cell, N, Q, d, L).  0 for unsupported sizes. */
size_t elm_rnn_fit_workspace_bytes(int cell, int64_t N, int Q, int d, int L, int m, int h_in_workspace);

/* Algorithm "S-R-ELM" end to end: create the model from `seed`, build H(Q) from the device
 * windows X, solve for beta against the device targets T (N x m), keep beta in the model.
 * H_out (device, N x L) is nullable (then H lives in the workspace).  refine / beta_out /
 * beta64_out / stats as in elm_rnn_solve.  *model_out receives the model (also on ELM_ERANK). */
int elm_rnn_fit(int cell, const float* X, int64_t ldx_n, int64_t ldx_q, const float* T,
                int64_t N, int Q, int d, int L, int m, uint64_t seed, const elm_rnn_init* init,
                int refine, void* workspace, size_t workspace_bytes, void* hip_stream,
                float* H_out, float* beta_out, double* beta64_out,
                elm_rnn_stats* stats, elm_rnn_model** model_out);

/* ---- the whole fit without an N x L hidden matrix in memory ----------------------------------- */

/* Workspace for elm_rnn_fit_streamed: the solve workspace plus one chunk of H (chunk_rows x L floats;
 * chunk_rows <= 0 selects the default, about 128 MiB of H; other values are rounded up to a multiple of
 * 128 rows and capped at N) plus elm_rnn_hidden_workspace_bytes() for a chunk of rows. */
size_t elm_rnn_fit_streamed_workspace_bytes(int cell, int64_t N, int Q, int d, int L, int m,
                                            int64_t chunk_rows);

/* Algorithm "S-R-ELM" with steps (2) and (3) fused: only H(Q) enters step (3), and the R factor of
 * [H | T] can absorb H a block of rows at a time, so the N x L matrix never exists.  Two forms:
 *   in-kernel hand-off  the stage-1 kernel runs a persistent grid, one work-group per level-0 R factor
 *                       of the TSQR; every finished tile [H(Q) | T] is rewritten in LDS as the next row
 *                       block and folded into that R factor before the work-group starts its next tile.
 *                       Exists for float32-contraction models of the dense cells with more than 64
 *                       units; where stage 1 runs one work-group per compute unit (LSTM L > 128,
 *                       Elman / GRU L > 256) it costs nothing, where it runs two (32-row tiles) the
 *                       folds take four times the Householder steps of the chunked form (4 % slower at
 *                       L = 256), so the automatic mode uses it only for the former;
 *   chunked             H is produced one chunk of rows at a time into a buffer small enough to stay in
 *                       the memory-side cache and folded into the R factors by the TSQR's level 0 before
 *                       the next chunk overwrites it.  Any cell, any contraction.
 * chunk_rows = 0 picks the hand-off for the one-work-group-per-unit layers when N gives every work-group
 * of the grid a tile, else default chunks; chunk_rows > 0 asks for chunks of that many rows; chunk_rows = -1 asks for the
 * hand-off and returns ELM_EUNSUPPORTED where it does not exist.
 * Same arguments and results as elm_rnn_fit (there is no H_out), and the same beta up to float32
 * rounding in the factorisation, except:
 *   refine = 0      beta is the plain float32 TSQR solution; stats->rmse is read off the R factor
 *                   (= rmse_qr) and stats->ne_resid is NaN (no pass over H with the final beta exists);
 *   refine = 1..4   that many float64-residual refinement steps, each of which recomputes H chunk by
 *                   chunk (one more run of step (2)), plus one more run for the statistics;
 *   refine = -1     refine twice if max|R_jj| > 30 min|R_jj| (the unrefined normal-equation residual is
 *                   about 1e-8 .. 6e-8 times that ratio), else not at all.
 * stats->t_hidden_ms sums every run of step (2) (with the hand-off it includes level 0 of the TSQR);
 * stats->refine_iters reports the steps taken. */
int elm_rnn_fit_streamed(int cell, const float* X, int64_t ldx_n, int64_t ldx_q, const float* T,
                         int64_t N, int Q, int d, int L, int m, uint64_t seed, const elm_rnn_init* init,
                         int64_t chunk_rows, int refine, void* workspace, size_t workspace_bytes,
                         void* hip_stream, float* beta_out, double* beta64_out,
                         elm_rnn_stats* stats, elm_rnn_model** model_out);

/* Workspace with which elm_rnn_predict runs in one pass: N*L floats for H plus the model's
 * elm_rnn_hidden_workspace_bytes() for N rows. */
size_t elm_rnn_predict_workspace_bytes(const elm_rnn_model* model, int64_t N);

/* The paper's output equation y_hat = sum_i beta_i f_i(Q): build H(Q) for N new windows with
 * the model's weights and write Y_out = H beta (device, N x m float32).  A smaller workspace is
 * accepted as long as it holds elm_rnn_predict_workspace_bytes() for 256 rows (or for all N): H is then
 * produced and consumed in chunks of as many rows as fit, with the same result. */
int elm_rnn_predict(const elm_rnn_model* model, const float* X, int64_t ldx_n, int64_t ldx_q,
                    int64_t N, float* Y_out, void* workspace, size_t workspace_bytes,
                    void* hip_stream);

/* ---- diagnostics ---------------------------------------------------------------------------- */

/* Measured ceilings of the current device, for quoting kernel rates against what the chip sustains as well
 * as against its published peaks (the paper reports speed-ups only; this is measurement support, not
 * part of the method): TFLOP/s of a register-resident loop of float32 32x32x2 and of fp16 32x32x16 matrix
 * instructions (the two that step (2) is built on; 1,024 work-groups, four accumulators per wave), and
 * GB/s (read + written) of a streaming copy of half the workspace onto the other half.
 * valu_overlap_f32 / valu_overlap_f16 (nullable): how much of a vector-ALU loop is hidden behind a loop of
 * float32 / fp16 matrix instructions that another wave runs on the same SIMD (two waves per SIMD, each loop
 * timed alone and both together; 1 = the two overlap completely, 0 = one waits for the other): this decides
 * whether point-wise work can be hidden behind a contraction by giving it waves of its own.
 * workspace: device, at least elm_rnn_probe_workspace_bytes() (2 GiB), contents destroyed.  Synchronises the
 * stream. */
size_t elm_rnn_probe_workspace_bytes(void);
int elm_rnn_probe_ceilings(double* mfma_f32_tflops, double* mfma_f16_tflops, double* copy_gbs,
                           double* valu_overlap_f32, double* valu_overlap_f16,
                           void* workspace, size_t workspace_bytes, void* hip_stream);


const char* elm_rnn_strerror(int code);
const char* elm_rnn_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ELM_RNN_H */
