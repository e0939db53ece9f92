// C ABI of libelmrnn: argument checks, the seeded weight generator (step 1 of the paper's
// Algorithm "S-R-ELM"), model life-cycle and the orchestration of stage 1 and stage 2.

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "internal.h"

struct elm_rnn_model {
    int cell, Q, d, L, m, G;
    elm::PackedLayout lay;
    std::vector<float> W, U, b;   // host copies, float32
    float* dWp = nullptr;         // packed [W; b; U] on the device (dense cells; rotations for the multi-lag cell)
    float* dTiny = nullptr;       // dense cells of at most kTinyMaxL units: [b; W; U] rows padded for the vector-ALU kernel
    float* dDiag = nullptr;       // ELM_CELL_ELMAN_DIAG: W^T [L][d], alpha [L][Q], b [L] back to back
    elm::FcStepLayout fcs{};      // ELM_CELL_FC_MULTILAG beyond what LDS holds: one launch per step with
    float* dFcW = nullptr;        //   the packed stack [A_{Q-1}; ...; A_1; W; b] and
    float* dFcW16 = nullptr;      //   the same stack per 16-column unit (layers of 65 to 96 units);
                                  //   the past states of a pass of rows live in the caller's workspace
    int contraction = ELM_CONTRACT_FP32;
    elm::SplitLayout slay{};      // ELM_CONTRACT_SPLIT16: layout and packed split weights
    void* dWs = nullptr;
    double* dBeta = nullptr;      // L x m float64 on the device
};

namespace elm {

static thread_local char g_hip_error[512] = "";

void set_hip_error(hipError_t e, const char* where) {
    std::snprintf(g_hip_error, sizeof g_hip_error, "%s: %s", where, hipGetErrorString(e));
}

void set_error_text(const char* text) { std::snprintf(g_hip_error, sizeof g_hip_error, "%s", text); }

int device_compute_units() {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return 256;
    return cus;
}

namespace {

// SplitMix64 (Steele, Lea, Flood: "Fast splittable pseudorandom number generators").
struct SplitMix64 {
    uint64_t state;
    explicit SplitMix64(uint64_t seed) : state(seed) {}
    uint64_t next() {
        state += 0x9E3779B97F4A7C15ull;
        uint64_t z = state;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    double uniform() { return (double)(next() >> 11) * 0x1.0p-53; }
};

double frobenius(const std::vector<double>& a) {
    double s = 0.0;
    for (double v : a) s += v * v;
    return std::sqrt(s);
}

// C = B * B for row-major n x n matrices (host).
void square_into(const double* __restrict__ B, double* __restrict__ C, int n) {
    for (int i = 0; i < n; ++i) {
        double* crow = C + (size_t)i * n;
        for (int j = 0; j < n; ++j) crow[j] = 0.0;
        for (int k = 0; k < n; ++k) {
            const double bik = B[(size_t)i * n + k];
            const double* brow = B + (size_t)k * n;
            for (int j = 0; j < n; ++j) crow[j] += bik * brow[j];
        }
    }
}

// Spectral radius by Gelfand's formula rho = lim ||A^k||^(1/k) along k = 2^i with renormalised
// repeated squaring: A^(2^i) = exp(2^i s_i) B_i, ||B_i||_F = 1, s_{i+1} = s_i + 2^-(i+1) log||B_i^2||_F.
double spectral_radius(const std::vector<double>& A, int n) {
    std::vector<double> B(A), C((size_t)n * n);
    double nf = frobenius(B);
    if (nf == 0.0) return 0.0;
    for (double& v : B) v /= nf;
    double log_rho = std::log(nf), w = 1.0, prev = -1.0;
    int settled = 0;
    for (int it = 0; it < 48; ++it) {       // 2^-48 * |log ||B^2||| is below double rounding of log rho
        square_into(B.data(), C.data(), n);
        const double nc = frobenius(C);
        if (nc == 0.0) return 0.0;       // nilpotent
        w *= 0.5;
        // once ||B_i^2|| has stopped changing (B_i has converged to the dominant rank-one part)
        // the rest of the series is geometric: sum_{k>i} 2^-k log nc = 2^-i log nc
        settled = (std::fabs(nc - prev) <= 4e-16 * nc) ? settled + 1 : 0;
        if (settled >= 2) {
            log_rho += 2.0 * w * std::log(nc);
            break;
        }
        prev = nc;
        log_rho += w * std::log(nc);
        for (double& v : C) v /= nc;
        B.swap(C);
    }
    return std::exp(log_rho);
}

// history slots of the fully connected multi-lag cell: lags 1 .. Q-1 can occur inside a window
int fc_ring(int Q) { return Q > 1 ? Q - 1 : 1; }

// The multi-lag cell keeps the operand row [x | 1 | Q-1 slots of L] in LDS for all steps while a
// 32-sample tile of it fits; layers of at most two column blocks then leave waves idle (the tile cannot
// grow to the rows they would take), and past 640 columns the launch-per-step form is the faster one
// (measured at Q = 50, N = 700,000: L = 20 19.7 ms against 37.2 ms; L = 10 13.8 ms against 10.4 ms).
bool fc_in_lds(int Q, int d, int L) {
    const int64_t K = (int64_t)fc_ring(Q) * L + d + 1;
    return K <= kFcMaxK && (L > 64 || K <= 640);
}

int check_dims(int cell, int Q, int d, int L, int m) {
    if (cell != ELM_CELL_ELMAN && cell != ELM_CELL_LSTM && cell != ELM_CELL_GRU &&
        cell != ELM_CELL_ELMAN_DIAG && cell != ELM_CELL_FC_MULTILAG)
        return ELM_EINVAL;
    if (Q < 1 || d < 1 || L < 1 || m < 1) return ELM_EINVAL;
    if (L > 512 || d > 64 || m > 16) return ELM_EUNSUPPORTED;
    if (cell == ELM_CELL_ELMAN_DIAG && Q > kDiagMaxQ) return ELM_EUNSUPPORTED;
    if (cell == ELM_CELL_FC_MULTILAG && !fc_in_lds(Q, d, L) && !fc_step_layout(Q, d, L, nullptr))
        return ELM_EUNSUPPORTED;
    return ELM_OK;
}

// columns per row of the recurrent weight array: k*L for the dense lag-1 cells, Q lags for the
// diagonal cell, Q blocks of L for the fully connected multi-lag cell (stored [Q][L][L])
size_t recurrent_cols(int cell, int Q, int L) {
    if (cell == ELM_CELL_ELMAN_DIAG) return (size_t)Q;
    if (cell == ELM_CELL_FC_MULTILAG) return (size_t)Q * L;
    return (size_t)gates_of(cell) * L;
}

int build_model(int cell, int Q, int d, int L, int m, std::vector<float>&& W, std::vector<float>&& U,
                std::vector<float>&& b, elm_rnn_model** out) {
    elm_rnn_model* mdl = new (std::nothrow) elm_rnn_model();
    if (mdl == nullptr) return ELM_EINVAL;
    mdl->cell = cell; mdl->Q = Q; mdl->d = d; mdl->L = L; mdl->m = m; mdl->G = gates_of(cell);
    mdl->W = std::move(W); mdl->U = std::move(U); mdl->b = std::move(b);
    std::vector<float> packed;
    float** dst = &mdl->dWp;
    if (cell == ELM_CELL_ELMAN_DIAG) {
        mdl->lay = PackedLayout{};
        packed.resize((size_t)L * d + (size_t)L * Q + L);
        for (int j = 0; j < L; ++j)
            for (int s = 0; s < d; ++s) packed[(size_t)j * d + s] = mdl->W[(size_t)s * L + j];
        std::copy(mdl->U.begin(), mdl->U.end(), packed.begin() + (size_t)L * d);
        std::copy(mdl->b.begin(), mdl->b.end(), packed.begin() + (size_t)L * d + (size_t)L * Q);
        dst = &mdl->dDiag;
    } else if (cell == ELM_CELL_FC_MULTILAG && !fc_in_lds(Q, d, L)) {
        mdl->lay = PackedLayout{};
        if (!fc_step_layout(Q, d, L, &mdl->fcs)) {
            delete mdl;
            return ELM_EUNSUPPORTED;
        }
        packed.resize(mdl->fcs.floats);
        pack_weights_fc_steps(mdl->fcs, mdl->W.data(), mdl->U.data(), mdl->b.data(), packed.data());
        dst = &mdl->dFcW;
    } else if (cell == ELM_CELL_FC_MULTILAG) {
        mdl->lay = packed_layout(cell, d, L, fc_ring(Q));
        packed.resize(mdl->lay.floats);
        pack_weights_fc(mdl->lay, mdl->W.data(), mdl->U.data(), mdl->b.data(), packed.data());
    } else {
        mdl->lay = packed_layout(cell, d, L);
        packed.resize(mdl->lay.floats);
        pack_weights(mdl->lay, mdl->W.data(), mdl->U.data(), mdl->b.data(), packed.data());
    }
    hipError_t e = hipMalloc(dst, packed.size() * sizeof(float));
    if (e == hipSuccess && tiny_padded_units(cell, L) > 0) {
        std::vector<float> tiny(tiny_packed_floats(cell, d, L));
        pack_weights_tiny(cell, d, L, mdl->W.data(), mdl->U.data(), mdl->b.data(), tiny.data());
        e = hipMalloc(&mdl->dTiny, tiny.size() * sizeof(float));
        if (e == hipSuccess) e = hipMemcpy(mdl->dTiny, tiny.data(), tiny.size() * sizeof(float), hipMemcpyHostToDevice);
    }
    if (e == hipSuccess && dst == &mdl->dFcW && mdl->fcs.NU > 0) {
        std::vector<float> units(mdl->fcs.floats16);
        pack_weights_fc_rows(mdl->fcs, mdl->W.data(), mdl->U.data(), mdl->b.data(), units.data());
        e = hipMalloc(&mdl->dFcW16, units.size() * sizeof(float));
        if (e == hipSuccess)
            e = hipMemcpy(mdl->dFcW16, units.data(), units.size() * sizeof(float), hipMemcpyHostToDevice);
    }
    if (e == hipSuccess) e = hipMalloc(&mdl->dBeta, (size_t)L * m * sizeof(double));
    if (e == hipSuccess)
        e = hipMemcpy(*dst, packed.data(), packed.size() * sizeof(float), hipMemcpyHostToDevice);
    if (e == hipSuccess) {        // beta = 0 until a fit stores it; a synchronous copy, so that it is ordered
        const std::vector<double> zeros((size_t)L * m, 0.0);       // before work on any stream of the caller
        e = hipMemcpy(mdl->dBeta, zeros.data(), zeros.size() * sizeof(double), hipMemcpyHostToDevice);
    }
    if (e != hipSuccess) {
        set_hip_error(e, "model upload");
        elm_rnn_free(mdl);
        return ELM_EHIP;
    }
    *out = mdl;
    return ELM_OK;
}

// Build and upload the split-format weights of a model (once); ELM_EUNSUPPORTED if the model
// cannot use the mode.
int enable_split(elm_rnn_model* mdl) {
    if (mdl->dWs != nullptr) return ELM_OK;
    if (mdl->cell == ELM_CELL_ELMAN_DIAG || mdl->cell == ELM_CELL_FC_MULTILAG) return ELM_EUNSUPPORTED;
    mdl->slay = split_layout(mdl->cell, mdl->d, mdl->L, mdl->W.data(), mdl->U.data(), mdl->b.data());
    if (!mdl->slay.ok) return ELM_EUNSUPPORTED;
    std::vector<unsigned char> packed(mdl->slay.bytes);
    pack_weights_split(mdl->slay, mdl->W.data(), mdl->U.data(), mdl->b.data(), packed.data());
    ELM_HIP_TRY(hipMalloc(&mdl->dWs, packed.size()));
    ELM_HIP_TRY(hipMemcpy(mdl->dWs, packed.data(), packed.size(), hipMemcpyHostToDevice));
    return ELM_OK;
}

// device scratch stage 1 needs for N rows of this model (only the launch-per-step multi-lag cell has any)
size_t hidden_scratch_bytes(const elm_rnn_model* mdl, int64_t N) {
    return mdl->dFcW != nullptr ? fc_scratch(mdl->fcs, N).bytes : 0;
}

// the same before a model exists
size_t hidden_scratch_bytes(int cell, int64_t N, int Q, int d, int L) {
    FcStepLayout lay{};
    if (cell != ELM_CELL_FC_MULTILAG || N < 1 || fc_in_lds(Q, d, L) || !fc_step_layout(Q, d, L, &lay)) return 0;
    return fc_scratch(lay, N).bytes;
}

// stage 1 for any cell; scratch: hidden_scratch_bytes(mdl, N) of device memory (may be null when that is 0)
hipError_t run_hidden(const elm_rnn_model* mdl, const float* X, int64_t ldx_n, int64_t ldx_q, int64_t N,
                      int Q_run, const float* h0, const float* c0, float* H, float* C, void* scratch,
                      hipStream_t stream) {
    if (mdl->cell == ELM_CELL_ELMAN_DIAG) {
        const float* Wt = mdl->dDiag;
        const float* alpha = Wt + (size_t)mdl->L * mdl->d;
        const float* bias = alpha + (size_t)mdl->L * mdl->Q;
        return launch_hidden_diag(Wt, alpha, bias, mdl->Q, X, ldx_n, ldx_q, N, Q_run, mdl->d, mdl->L, H,
                                  stream);
    }
    if (mdl->dFcW != nullptr)
        return launch_hidden_fc_steps(mdl->fcs, mdl->dFcW, mdl->dFcW16, scratch, X, ldx_n, ldx_q, N, Q_run, H, stream);
    if (mdl->contraction == ELM_CONTRACT_FP32 && mdl->dTiny != nullptr)
        return launch_hidden_tiny(mdl->cell, mdl->d, mdl->L, mdl->dTiny, X, ldx_n, ldx_q, N, Q_run, h0, c0, H, C, stream);
    if (mdl->contraction == ELM_CONTRACT_SPLIT16 && mdl->dWs != nullptr)
        return launch_hidden_split(mdl->slay, mdl->dWs, X, ldx_n, ldx_q, N, Q_run, h0, c0, H, C, stream);
    return launch_hidden(mdl->lay, mdl->dWp, X, ldx_n, ldx_q, N, Q_run, h0, c0, H, C, stream);
}

struct EventPair {
    hipEvent_t a = nullptr, b = nullptr;
    hipError_t create() {
        hipError_t e = hipEventCreate(&a);
        if (e == hipSuccess) e = hipEventCreate(&b);
        return e;
    }
    ~EventPair() {
        if (a) (void)hipEventDestroy(a);
        if (b) (void)hipEventDestroy(b);
    }
};

// max|R_jj| / min|R_jj| above which refine = -1 refines beta: the normal-equation residual of the unrefined
// float32 solution grows like 1e-8 .. 6e-8 times this ratio
constexpr double kAutoRefineRatio = 30.0;

// stage 2 on the stream; fills stats (after a sync) when asked.  hidden_ms is copied through.
int run_solve(const float* H, const float* T, int64_t N, int L, int m, int refine, float* beta_out,
              double* beta64_out, elm_rnn_stats* stats, void* ws, size_t ws_bytes,
              hipStream_t stream, double hidden_ms, hipEvent_t hidden_done) {
    if (H == nullptr || T == nullptr || beta_out == nullptr) return ELM_EINVAL;
    if (N < 1 || L < 1 || m < 1 || N < L || refine < -1 || refine > 4) return ELM_EINVAL;
    if (L > 512 || m > 16) return ELM_EUNSUPPORTED;
    const SolvePlan plan = make_solve_plan(N, L, m);
    if (ws == nullptr || ws_bytes < plan.bytes) return ELM_EWORKSPACE;
    return run_solve_with_plan(plan, H, T, refine, beta_out, beta64_out, stats, ws, stream, hidden_ms, hidden_done);
}

}  // namespace

// Stage 2 with a plan the caller made (ws holds plan.bytes): TSQR, back-solve, refinement, statistics.
int run_solve_with_plan(const SolvePlan& plan, const float* H, const float* T, int refine, float* beta_out,
                        double* beta64_out, elm_rnn_stats* stats, void* ws, hipStream_t stream,
                        double hidden_ms, hipEvent_t hidden_done) {
    const int64_t N = plan.N;
    const int L = plan.L, m = plan.m;
    EventPair ev;
    ELM_HIP_TRY(ev.create());
    if (hidden_done == nullptr) ELM_HIP_TRY(hipEventRecord(ev.a, stream));

    float* R = nullptr;
    ELM_HIP_TRY(launch_tsqr(plan, H, T, ws, &R, stream));
    ELM_HIP_TRY(launch_backsolve(plan, R, ws, stream));
    double sc[8];
    const double* small = reinterpret_cast<const double*>(static_cast<const char*>(ws) + plan.off_small);
    if (refine < 0) {          // decide from the diagonal of R, which the back-solve has just recorded
        ELM_HIP_TRY(hipMemcpyAsync(sc, small + SmallArea::scal(L, m), sizeof sc, hipMemcpyDeviceToHost, stream));
        ELM_HIP_TRY(hipStreamSynchronize(stream));
        refine = (sc[6] == 0.0 && sc[5] > kAutoRefineRatio * sc[4]) ? 2 : 0;
    }
    for (int it = 0; it < refine; ++it) {
        ELM_HIP_TRY(launch_residual_pass(plan, H, T, ws, stream));
        ELM_HIP_TRY(launch_refine_update(plan, R, ws, stream));
    }
    ELM_HIP_TRY(launch_residual_pass(plan, H, T, ws, stream));     // statistics of the final beta
    ELM_HIP_TRY(launch_export_beta(plan, ws, beta_out, beta64_out, stream));
    ELM_HIP_TRY(hipEventRecord(ev.b, stream));

    // the rank flag is always read back: the return code depends on it
    ELM_HIP_TRY(hipMemcpyAsync(sc, small + SmallArea::scal(L, m), sizeof sc, hipMemcpyDeviceToHost, stream));
    ELM_HIP_TRY(hipStreamSynchronize(stream));
    if (stats != nullptr) {
        float ms = 0.0f;
        ELM_HIP_TRY(hipEventElapsedTime(&ms, hidden_done ? hidden_done : ev.a, ev.b));
        stats->t_hidden_ms = hidden_ms;
        stats->t_solve_ms = ms;
        const double nm = (double)N * m;
        stats->rmse = std::sqrt(sc[0] / nm);
        stats->rmse_qr = std::sqrt(sc[3] / nm);
        const double den = std::sqrt(sc[1]) * std::sqrt(sc[0]);
        stats->ne_resid = den > 0.0 ? std::sqrt(sc[2]) / den : 0.0;
        stats->r_diag_min = sc[4];
        stats->r_diag_max = sc[5];
        stats->refine_iters = refine;
    }
    return sc[6] != 0.0 ? ELM_ERANK : ELM_OK;
}

}  // namespace elm

using namespace elm;

extern "C" {

// step 1 of Algorithm "S-R-ELM"; device work (the spectral radius of a wide Elman matrix) goes to `stream`
static int create_model(int cell, int Q, int d, int L, int m, uint64_t seed, const elm_rnn_init* init,
                        hipStream_t stream, elm_rnn_model** model_out) {
    if (init == nullptr || model_out == nullptr) return ELM_EINVAL;
    int rc = check_dims(cell, Q, d, L, m);
    if (rc != ELM_OK) return rc;
    if (!(init->w_scale > 0.0) || init->spectral_radius < 0.0) return ELM_EINVAL;
    if (init->spectral_radius > 0.0 && cell != ELM_CELL_ELMAN) return ELM_EINVAL;
    if (init->contraction != ELM_CONTRACT_FP32 && init->contraction != ELM_CONTRACT_SPLIT16) return ELM_EINVAL;
    const int G = gates_of(cell), GL = G * L;
    SplitMix64 rng(seed);
    std::vector<double> W((size_t)d * GL), U((size_t)L * recurrent_cols(cell, Q, L)), b((size_t)GL);
    for (double& v : W) v = (2.0 * rng.uniform() - 1.0) * init->w_scale;
    for (double& v : U) v = (2.0 * rng.uniform() - 1.0) * init->w_scale;
    for (double& v : b) v = (2.0 * rng.uniform() - 1.0) * init->w_scale;
    if (init->spectral_radius > 0.0) {
        double rho = 0.0;
        if (L < 64) {
            rho = spectral_radius(U, L);        // microseconds on the host
        } else {
            ELM_HIP_TRY(spectral_radius_device(U.data(), L, &rho, stream));
        }
        if (!(rho > 0.0)) return ELM_EINVAL;
        const double f = init->spectral_radius / rho;
        for (double& v : U) v *= f;
    }
    if (init->zero_bias) {
        for (double& v : b) v = 0.0;
    } else if (cell == ELM_CELL_LSTM && init->forget_bias != 0.0) {
        for (int j = 0; j < L; ++j) b[(size_t)L + j] += init->forget_bias;
    }
    std::vector<float> Wf(W.begin(), W.end()), Uf(U.begin(), U.end()), bf(b.begin(), b.end());
    rc = build_model(cell, Q, d, L, m, std::move(Wf), std::move(Uf), std::move(bf), model_out);
    if (rc == ELM_OK && init->contraction != ELM_CONTRACT_FP32) {
        rc = elm_rnn_model_set_contraction(*model_out, init->contraction);
        if (rc != ELM_OK) {
            elm_rnn_free(*model_out);
            *model_out = nullptr;
        }
    }
    return rc;
}

int elm_rnn_model_create(int cell, int Q, int d, int L, int m, uint64_t seed,
                         const elm_rnn_init* init, elm_rnn_model** model_out) {
    return create_model(cell, Q, d, L, m, seed, init, nullptr, model_out);
}

int elm_rnn_model_create_from_weights(int cell, int Q, int d, int L, int m, const float* W,
                                      const float* U, const float* b, elm_rnn_model** model_out) {
    if (W == nullptr || U == nullptr || b == nullptr || model_out == nullptr) return ELM_EINVAL;
    int rc = check_dims(cell, Q, d, L, m);
    if (rc != ELM_OK) return rc;
    const size_t GL = (size_t)gates_of(cell) * L;
    std::vector<float> Wf(W, W + (size_t)d * GL), Uf(U, U + (size_t)L * recurrent_cols(cell, Q, L)),
        bf(b, b + GL);
    return build_model(cell, Q, d, L, m, std::move(Wf), std::move(Uf), std::move(bf), model_out);
}

int elm_rnn_get_weights(const elm_rnn_model* model, float* W, float* U, float* b, double* beta64) {
    if (model == nullptr) return ELM_EINVAL;
    if (W) std::memcpy(W, model->W.data(), model->W.size() * sizeof(float));
    if (U) std::memcpy(U, model->U.data(), model->U.size() * sizeof(float));
    if (b) std::memcpy(b, model->b.data(), model->b.size() * sizeof(float));
    if (beta64)
        ELM_HIP_TRY(hipMemcpy(beta64, model->dBeta, (size_t)model->L * model->m * sizeof(double),
                              hipMemcpyDeviceToHost));
    return ELM_OK;
}

int elm_rnn_model_set_contraction(elm_rnn_model* model, int contraction) {
    if (model == nullptr) return ELM_EINVAL;
    if (contraction == ELM_CONTRACT_FP32) {
        model->contraction = contraction;
        return ELM_OK;
    }
    if (contraction != ELM_CONTRACT_SPLIT16) return ELM_EINVAL;
    const int rc = enable_split(model);
    if (rc == ELM_OK) model->contraction = contraction;
    return rc;
}

int elm_rnn_set_beta(elm_rnn_model* model, const double* beta64) {
    if (model == nullptr || beta64 == nullptr) return ELM_EINVAL;
    ELM_HIP_TRY(hipMemcpy(model->dBeta, beta64, (size_t)model->L * model->m * sizeof(double),
                          hipMemcpyHostToDevice));
    return ELM_OK;
}

void elm_rnn_free(elm_rnn_model* model) {
    if (model == nullptr) return;
    if (model->dWp) (void)hipFree(model->dWp);
    if (model->dTiny) (void)hipFree(model->dTiny);
    if (model->dDiag) (void)hipFree(model->dDiag);
    if (model->dFcW) (void)hipFree(model->dFcW);
    if (model->dFcW16) (void)hipFree(model->dFcW16);
    if (model->dWs) (void)hipFree(model->dWs);
    if (model->dBeta) (void)hipFree(model->dBeta);
    delete model;
}

size_t elm_rnn_hidden_workspace_bytes(int cell, int64_t N, int Q, int d, int L) {
    if (check_dims(cell, Q, d, L, 1) != ELM_OK) return 0;
    return hidden_scratch_bytes(cell, N, Q, d, L);
}

int elm_rnn_hidden(const elm_rnn_model* model, const float* X, int64_t ldx_n, int64_t ldx_q,
                   int64_t N, int Q_run, const float* h0, const float* c0, float* H_out,
                   float* c_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (model == nullptr || X == nullptr || H_out == nullptr) return ELM_EINVAL;
    if (N < 1 || Q_run < 1 || ldx_n < 0 || ldx_q < 0) return ELM_EINVAL;
    const size_t need = hidden_scratch_bytes(model, N);
    if (need > 0 && (workspace == nullptr || workspace_bytes < need)) return ELM_EWORKSPACE;
    if ((model->cell == ELM_CELL_ELMAN_DIAG || model->cell == ELM_CELL_FC_MULTILAG) &&
        (h0 != nullptr || c0 != nullptr || c_out != nullptr || Q_run > model->Q))
        return ELM_EINVAL;
    ELM_HIP_TRY(run_hidden(model, X, ldx_n, ldx_q, N, Q_run, h0, c0, H_out, c_out, workspace,
                           static_cast<hipStream_t>(hip_stream)));
    return ELM_OK;
}

size_t elm_rnn_solve_workspace_bytes(int64_t N, int L, int m) {
    if (N < 1 || L < 1 || m < 1 || L > 512 || m > 16) return 0;
    return make_solve_plan(N, L, m).bytes;
}

int elm_rnn_solve(const float* H, const float* T, int64_t N, int L, int m, int refine,
                  float* beta_out, double* beta64_out, elm_rnn_stats* stats, void* workspace,
                  size_t workspace_bytes, void* hip_stream) {
    return run_solve(H, T, N, L, m, refine, beta_out, beta64_out, stats, workspace, workspace_bytes,
                     static_cast<hipStream_t>(hip_stream), 0.0, nullptr);
}

size_t elm_rnn_fit_workspace_bytes(int cell, int64_t N, int Q, int d, int L, int m, int h_in_workspace) {
    const size_t s = elm_rnn_solve_workspace_bytes(N, L, m);
    if (s == 0 || check_dims(cell, Q, d, L, m) != ELM_OK) return 0;
    return s + (h_in_workspace ? (((size_t)N * L * sizeof(float) + 255) & ~(size_t)255) : 0) +
           hidden_scratch_bytes(cell, N, Q, d, L);
}

int elm_rnn_fit(int cell, const float* X, int64_t ldx_n, int64_t ldx_q, const float* T, int64_t N,
                int Q, int d, int L, int m, uint64_t seed, const elm_rnn_init* init, int refine,
                void* workspace, size_t workspace_bytes, void* hip_stream, float* H_out, float* beta_out,
                double* beta64_out, elm_rnn_stats* stats, elm_rnn_model** model_out) {
    if (X == nullptr || T == nullptr || beta_out == nullptr || model_out == nullptr) return ELM_EINVAL;
    if (N < 1 || N < L || ldx_n < 0 || ldx_q < 0 || refine < -1 || refine > 4) return ELM_EINVAL;
    int rc = check_dims(cell, Q, d, L, m);
    if (rc != ELM_OK) return rc;
    const size_t need = elm_rnn_fit_workspace_bytes(cell, N, Q, d, L, m, H_out == nullptr);
    if (need == 0) return ELM_EUNSUPPORTED;
    if (workspace == nullptr || workspace_bytes < need) return ELM_EWORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    elm_rnn_model* mdl = nullptr;
    rc = create_model(cell, Q, d, L, m, seed, init, stream, &mdl);
    if (rc != ELM_OK) return rc;

    // workspace: [solve area][H when the caller gave no H_out][stage-1 scratch]
    const size_t solve_bytes = elm_rnn_solve_workspace_bytes(N, L, m);
    const size_t h_bytes = H_out ? 0 : (((size_t)N * L * sizeof(float) + 255) & ~(size_t)255);
    float* H = H_out ? H_out : reinterpret_cast<float*>(static_cast<char*>(workspace) + solve_bytes);
    void* scratch = static_cast<char*>(workspace) + solve_bytes + h_bytes;

    EventPair ev;
    hipError_t e = ev.create();
    if (e == hipSuccess) e = hipEventRecord(ev.a, stream);
    if (e == hipSuccess)
        e = run_hidden(mdl, X, ldx_n, ldx_q, N, Q, nullptr, nullptr, H, nullptr, scratch, stream);
    if (e == hipSuccess) e = hipEventRecord(ev.b, stream);
    if (e != hipSuccess) {
        set_hip_error(e, "hidden-matrix stage");
        elm_rnn_free(mdl);
        return ELM_EHIP;
    }
    // stage 2 is timed from the end of stage 1; the hidden time is read after the final sync
    elm_rnn_stats local{};
    rc = run_solve(H, T, N, L, m, refine, beta_out, beta64_out, &local, workspace, solve_bytes, stream, 0.0,
                   ev.b);
    if (rc != ELM_OK && rc != ELM_ERANK) {
        elm_rnn_free(mdl);
        return rc;
    }
    float hms = 0.0f;
    e = hipEventElapsedTime(&hms, ev.a, ev.b);
    if (e == hipSuccess) {
        const double* small = reinterpret_cast<const double*>(static_cast<const char*>(workspace) +
                                                              make_solve_plan(N, L, m).off_small);
        e = hipMemcpyAsync(mdl->dBeta, small + SmallArea::BETA, (size_t)L * m * sizeof(double),
                           hipMemcpyDeviceToDevice, stream);
    }
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) {
        set_hip_error(e, "fit epilogue");
        elm_rnn_free(mdl);
        return ELM_EHIP;
    }
    local.t_hidden_ms = hms;
    if (stats) *stats = local;
    *model_out = mdl;
    return rc;
}

// rows of H per chunk of the streamed fit
static int64_t streamed_chunk(int64_t N, int L, int64_t chunk_rows) {
    if (chunk_rows <= 0) {
        // about 128 MiB of H: the chunk stage 1 writes is still in the memory-side cache when level 0
        // of the TSQR reads it, and both kernels get a whole number of rounds of work-groups
        chunk_rows = (((int64_t)128 << 20) / (4 * (int64_t)L)) / 32768 * 32768;
        if (chunk_rows < 32768) chunk_rows = 32768;
    }
    chunk_rows = (chunk_rows + 127) / 128 * 128;       // whole row blocks of the TSQR
    return chunk_rows < N ? chunk_rows : N;
}

// level-0 R factors the in-kernel hand-off may ask for: two work-groups per compute unit for the layers of at
// most 256 units, one above; 256 compute units assumed when none is visible (sizes are asked for up front)
static int streamed_fused_groups_bound(int L) {
    const int64_t g = (int64_t)(L <= 256 ? 2 : 1) * device_compute_units();
    return (int)(g > 1024 ? 1024 : g);
}

// solve-plan part of the streamed fit's workspace: room for either form's R factors
static size_t streamed_plan_bytes(int64_t N, int L, int m) {
    const size_t a = make_solve_plan(N, L, m).bytes;
    const size_t b = make_solve_plan(N, L, m, streamed_fused_groups_bound(L)).bytes;
    return a > b ? a : b;
}

size_t elm_rnn_fit_streamed_workspace_bytes(int cell, int64_t N, int Q, int d, int L, int m, int64_t chunk_rows) {
    if (elm_rnn_solve_workspace_bytes(N, L, m) == 0 || check_dims(cell, Q, d, L, m) != ELM_OK) return 0;
    const int64_t chunk = streamed_chunk(N, L, chunk_rows);
    return streamed_plan_bytes(N, L, m) + (((size_t)chunk * L * sizeof(float) + 255) & ~(size_t)255) +
           hidden_scratch_bytes(cell, chunk, Q, d, L);
}

int elm_rnn_fit_streamed(int cell, const float* X, int64_t ldx_n, int64_t ldx_q, const float* T, int64_t N,
                         int Q, int d, int L, int m, uint64_t seed, const elm_rnn_init* init,
                         int64_t chunk_rows, int refine, void* workspace, size_t workspace_bytes,
                         void* hip_stream, float* beta_out, double* beta64_out, elm_rnn_stats* stats,
                         elm_rnn_model** model_out) {
    if (X == nullptr || T == nullptr || beta_out == nullptr || model_out == nullptr) return ELM_EINVAL;
    if (N < 1 || N < L || refine < -1 || refine > 4 || ldx_n < 0 || ldx_q < 0 || chunk_rows < -1) return ELM_EINVAL;
    int rc = check_dims(cell, Q, d, L, m);
    if (rc != ELM_OK) return rc;
    const size_t need = elm_rnn_fit_streamed_workspace_bytes(cell, N, Q, d, L, m, chunk_rows);
    if (need == 0) return ELM_EUNSUPPORTED;
    if (workspace == nullptr || workspace_bytes < need) return ELM_EWORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // workspace: [solve area][one chunk of H][stage-1 scratch for a chunk of rows]
    const int64_t chunk = streamed_chunk(N, L, chunk_rows);
    float* Hc = reinterpret_cast<float*>(static_cast<char*>(workspace) + streamed_plan_bytes(N, L, m));
    void* scratch = reinterpret_cast<char*>(Hc) + (((size_t)chunk * L * sizeof(float) + 255) & ~(size_t)255);

    elm_rnn_model* mdl = nullptr;
    rc = create_model(cell, Q, d, L, m, seed, init, stream, &mdl);
    if (rc != ELM_OK) return rc;

    // In-kernel hand-off (the tile goes from LDS into the fold) where stage 1 has such a variant: forced by
    // chunk_rows == -1; chosen by default for the variants that run one work-group per compute unit when
    // every work-group of the persistent grid gets a tile (the two-per-unit variants fold 32-row tiles,
    // four times the Householder steps of the chunked level 0: measured 4 % slower at cfg4, so they are
    // on request only).  The kernel brings its own number of level-0 R factors: the plan is made for it.
    int per_cu = 1;
    const int fused_groups = (mdl->contraction == ELM_CONTRACT_FP32 && mdl->dWp != nullptr &&
                              (mdl->cell == ELM_CELL_ELMAN || mdl->cell == ELM_CELL_LSTM || mdl->cell == ELM_CELL_GRU))
                                 ? hidden_fused_groups(mdl->lay, N, m, &per_cu) : 0;
    if (chunk_rows == -1 && (fused_groups == 0 || fused_groups > streamed_fused_groups_bound(L))) {
        elm_rnn_free(mdl);
        return ELM_EUNSUPPORTED;
    }
    const bool fuse = fused_groups > 0 && fused_groups <= streamed_fused_groups_bound(L) &&
                      (chunk_rows == -1 || (chunk_rows == 0 && per_cu == 1 && fused_groups >= device_compute_units()));
    const SolvePlan plan = fuse ? make_solve_plan(N, L, m, fused_groups) : make_solve_plan(N, L, m);
    const double* small = reinterpret_cast<const double*>(static_cast<const char*>(workspace) + plan.off_small);

    // one event pair around every stage-1 launch: their sum is the stage-1 time, the rest of the
    // span is stage 2.  The pairs are summed (after a stream synchronisation) and reused every 64 chunks,
    // so that a fit in many small chunks does not pile up events.
    struct Events {
        std::vector<hipEvent_t> ev;
        size_t used = 0;
        double sum_ms = 0.0;
        ~Events() { for (hipEvent_t e : ev) (void)hipEventDestroy(e); }
        hipError_t mark(hipStream_t s) {
            if (used == ev.size()) {
                hipEvent_t e = nullptr;
                hipError_t rc = hipEventCreate(&e);
                if (rc != hipSuccess) return rc;
                ev.push_back(e);
            }
            return hipEventRecord(ev[used++], s);
        }
        // adds the elapsed time of the recorded pairs to sum_ms; the events can then be recorded again
        hipError_t collect(hipStream_t s) {
            hipError_t rc = hipStreamSynchronize(s);
            for (size_t i = 0; rc == hipSuccess && i + 1 < used; i += 2) {
                float ms = 0.0f;
                rc = hipEventElapsedTime(&ms, ev[i], ev[i + 1]);
                sum_ms += ms;
            }
            used = 0;
            return rc;
        }
    } span, s1;

    // one sweep over the rows: stage 1 on a chunk, then `consume` on that chunk
    auto sweep = [&](auto&& consume) -> hipError_t {
        for (int64_t r0 = 0; r0 < N; r0 += chunk) {
            const int64_t rows = (N - r0 < chunk) ? N - r0 : chunk;
            hipError_t e = (s1.used >= 128) ? s1.collect(stream) : hipSuccess;
            if (e == hipSuccess) e = s1.mark(stream);
            if (e == hipSuccess)
                e = run_hidden(mdl, X + r0 * ldx_n, ldx_n, ldx_q, rows, Q, nullptr, nullptr, Hc, nullptr, scratch, stream);
            if (e == hipSuccess) e = s1.mark(stream);
            if (e == hipSuccess) e = consume(T + r0 * m, rows, r0 > 0);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    };
    auto fail = [&](hipError_t e, const char* where) {
        set_hip_error(e, where);
        elm_rnn_free(mdl);
        return ELM_EHIP;
    };

    hipError_t e = span.mark(stream);
    if (e == hipSuccess && fuse) {
        e = s1.mark(stream);
        if (e == hipSuccess)
            e = launch_hidden_fused(mdl->lay, mdl->dWp, X, ldx_n, ldx_q, N, Q, T, plan, workspace, stream);
        if (e == hipSuccess) e = s1.mark(stream);
    } else if (e == hipSuccess) {
        e = sweep([&](const float* Tc, int64_t rows, bool later) {
            return launch_tsqr_level0(plan, Hc, Tc, rows, workspace, later ? 1 : 0, stream);
        });
    }
    float* R = nullptr;
    if (e == hipSuccess) e = launch_tsqr_combine(plan, workspace, &R, stream);
    if (e == hipSuccess) e = launch_backsolve(plan, R, workspace, stream);
    if (e != hipSuccess) return fail(e, "streamed fit: factorisation");

    double sc[8];
    int updates = refine;
    if (refine < 0) {
        e = hipMemcpyAsync(sc, small + SmallArea::scal(L, m), sizeof sc, hipMemcpyDeviceToHost, stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);
        if (e != hipSuccess) return fail(e, "streamed fit: condition read-back");
        updates = (sc[6] == 0.0 && sc[5] > kAutoRefineRatio * sc[4]) ? 2 : 0;
    }
    // every refinement step, and the statistics of the final beta, need H again: it is recomputed
    for (int it = 0; updates > 0 && it <= updates; ++it) {
        e = sweep([&](const float* Tc, int64_t rows, bool later) {
            return launch_residual_chunk(plan, Hc, Tc, rows, workspace, later ? 1 : 0, stream);
        });
        if (e == hipSuccess) e = launch_residual_finish(plan, workspace, stream);
        if (e == hipSuccess && it < updates) e = launch_refine_update(plan, R, workspace, stream);
        if (e != hipSuccess) return fail(e, "streamed fit: refinement");
    }
    e = launch_export_beta(plan, workspace, beta_out, beta64_out, stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(mdl->dBeta, small + SmallArea::BETA, (size_t)L * m * sizeof(double),
                           hipMemcpyDeviceToDevice, stream);
    if (e == hipSuccess) e = span.mark(stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(sc, small + SmallArea::scal(L, m), sizeof sc, hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return fail(e, "streamed fit: epilogue");

    if (stats != nullptr) {
        float total = 0.0f;
        e = hipEventElapsedTime(&total, span.ev[0], span.ev[1]);
        if (e == hipSuccess) e = s1.collect(stream);
        if (e != hipSuccess) return fail(e, "streamed fit: timing");
        const double hidden = s1.sum_ms;
        const double nm = (double)N * m;
        stats->t_hidden_ms = hidden;
        stats->t_solve_ms = total - hidden;
        stats->rmse_qr = std::sqrt(sc[3] / nm);
        if (updates > 0) {
            stats->rmse = std::sqrt(sc[0] / nm);
            const double den = std::sqrt(sc[1]) * std::sqrt(sc[0]);
            stats->ne_resid = den > 0.0 ? std::sqrt(sc[2]) / den : 0.0;
        } else {           // no pass over H with the final beta was made
            stats->rmse = stats->rmse_qr;
            stats->ne_resid = std::nan("");
        }
        stats->r_diag_min = sc[4];
        stats->r_diag_max = sc[5];
        stats->refine_iters = updates;
    }
    *model_out = mdl;
    return sc[6] != 0.0 ? ELM_ERANK : ELM_OK;
}

// H for `rows` rows followed by the stage-1 scratch for as many
static size_t predict_bytes(const elm_rnn_model* model, int64_t rows) {
    return (((size_t)rows * model->L * sizeof(float) + 255) & ~(size_t)255) + hidden_scratch_bytes(model, rows);
}

size_t elm_rnn_predict_workspace_bytes(const elm_rnn_model* model, int64_t N) {
    if (model == nullptr || N < 1) return 0;
    return predict_bytes(model, N);
}

int elm_rnn_predict(const elm_rnn_model* model, const float* X, int64_t ldx_n, int64_t ldx_q,
                    int64_t N, float* Y_out, void* workspace, size_t workspace_bytes,
                    void* hip_stream) {
    if (model == nullptr || X == nullptr || Y_out == nullptr || N < 1 || ldx_n < 0 || ldx_q < 0) return ELM_EINVAL;
    if (workspace == nullptr) return ELM_EWORKSPACE;
    // H is produced and consumed in chunks of as many rows as the workspace holds (whole groups of 256);
    // predict_bytes() never decreases with the rows, so the largest chunk that fits is found by bisection
    int64_t chunk = N;
    if (predict_bytes(model, N) > workspace_bytes) {
        int64_t lo = 0, hi = (N + 255) / 256;               // in units of 256 rows: lo fits (or is 0), hi does not
        while (hi - lo > 1) {
            const int64_t mid = lo + (hi - lo) / 2;
            if (predict_bytes(model, mid * 256) <= workspace_bytes) lo = mid; else hi = mid;
        }
        chunk = lo * 256;
    }
    if (chunk < 1) return ELM_EWORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    float* H = static_cast<float*>(workspace);
    void* scratch = static_cast<char*>(workspace) + (((size_t)chunk * model->L * sizeof(float) + 255) & ~(size_t)255);
    for (int64_t r0 = 0; r0 < N; r0 += chunk) {
        const int64_t rows = (N - r0 < chunk) ? N - r0 : chunk;
        ELM_HIP_TRY(run_hidden(model, X + r0 * ldx_n, ldx_n, ldx_q, rows, model->Q, nullptr, nullptr, H, nullptr,
                               scratch, stream));
        ELM_HIP_TRY(launch_predict_gemv(H, model->dBeta, rows, model->L, model->m, Y_out + r0 * model->m, stream));
    }
    return ELM_OK;
}

const char* elm_rnn_strerror(int code) {
    switch (code) {
        case ELM_OK: return "ok";
        case ELM_EINVAL: return "invalid argument";
        case ELM_EWORKSPACE: return "workspace missing or too small";
        case ELM_ERANK: return "hidden matrix is numerically rank deficient";
        case ELM_EHIP: return "HIP runtime error";
        case ELM_EUNSUPPORTED: return "size outside the supported range";
        default: return "unknown error code";
    }
}

const char* elm_rnn_last_hip_error(void) { return g_hip_error; }

}  // extern "C"
