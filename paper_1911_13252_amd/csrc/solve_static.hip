// elm_rnn_solve for callers that must not allocate: the TSQR's R factors, the partial sums of the residual
// passes and the small float64 area live in a file-scope device array instead of a caller workspace.

#include <mutex>

#include "internal.h"

namespace {

constexpr size_t kScratchBytes = ELM_RNN_STATIC_SCRATCH_BYTES;

// One copy per GPU, at its own address, held until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress: kernels and copies get the per-device pointer looked up below.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices] = {};      // device address of `scratch` on each device, once looked up

// The current device's copy of the array (looked up once per device, with that device current).
hipError_t scratch_address(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(g_lock);
    if (g_scratch_ptr[dev] == nullptr) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (ptr == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

// The default plan if it fits the array, else the same tree with the level-0 work-groups halved until it
// does (fewer, longer Householder chains: slower, same result up to float32 rounding); false if even one
// R factor, the partial sums and the small area do not fit.
bool plan_within_scratch(int64_t N, int L, int m, elm::SolvePlan* out) {
    elm::SolvePlan pl = elm::make_solve_plan(N, L, m);
    int groups = pl.groups[0];
    while (pl.bytes > kScratchBytes && groups > 1) {
        groups = (groups + 1) / 2;
        pl = elm::make_solve_plan(N, L, m, groups);
    }
    if (pl.bytes > kScratchBytes) return false;
    *out = pl;
    return true;
}

}  // namespace

extern "C" size_t elm_rnn_solve_static_scratch_bytes(void) { return kScratchBytes; }

extern "C" int elm_rnn_solve_static(const float* H, const float* T, int64_t N, int L, int m, int refine,
                                    float* beta_out, double* beta64_out, elm_rnn_stats* stats,
                                    void* hip_stream) {
    if (H == nullptr || T == nullptr || beta_out == nullptr) return ELM_EINVAL;
    if (N < 1 || L < 1 || m < 1 || N < L || refine < -1 || refine > 4) return ELM_EINVAL;
    if (L > 512 || m > 16) return ELM_EUNSUPPORTED;
    elm::SolvePlan plan{};
    if (!plan_within_scratch(N, L, m, &plan)) {
        elm::set_error_text("elm_rnn_solve_static: L x m too large for the static scratch array (one R factor, "
                            "1024 x (L m + 2) float64 partial sums and the small area must fit "
                            "ELM_RNN_STATIC_SCRATCH_BYTES); use elm_rnn_solve with a workspace");
        return ELM_EUNSUPPORTED;
    }
    void* ws = nullptr;
    ELM_HIP_TRY(scratch_address(&ws));
    // Nothing in the array has to start at zero: level 0 of the TSQR clears every R factor it folds into
    // (the combine levels copy theirs), every partial record that is summed has been written by the pass
    // before it, and the small area is written by the back-solve before anything reads it.  What the last
    // call left there is overwritten or never read.
    return elm::run_solve_with_plan(plan, H, T, refine, beta_out, beta64_out, stats, ws,
                                    static_cast<hipStream_t>(hip_stream), 0.0, nullptr);
}
