// Measured ceilings of the device the library runs on, for quoting kernel rates against what the chip
// sustains as well as against its published peaks: a register-resident matrix-instruction loop (float32
// 32x32x2 and fp16 32x32x16, the two instructions stage 1 is built on) and a streaming copy.
// Diagnostics only: nothing on the fit path calls this.

#include <vector>

#include "internal.h"

namespace elm {
namespace {

typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// Every wave issues back-to-back matrix instructions on four independent accumulators; the operands are
// loaded once (small random values), nothing touches memory inside the loop.
template <int MODE>   // 0: float32 32x32x2, 1: fp16 32x32x16
__global__ __launch_bounds__(256) void mfma_loop_kernel(const float* __restrict__ in, float* __restrict__ out,
                                                        int iters) {
    const float f0 = in[threadIdx.x], f1 = in[threadIdx.x + 256], f2 = in[threadIdx.x + 512], f3 = in[threadIdx.x + 768];
    halfx8 a0, a1, b0, b1;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a0[i] = (_Float16)(f0 * (i + 1));
        a1[i] = (_Float16)(f1 * (i + 1));
        b0[i] = (_Float16)(f2 * (i + 1));
        b1[i] = (_Float16)(f3 * (i + 1));
    }
    floatx16 acc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[q][i] = 0.0f;
    for (int it = 0; it < iters; ++it) {
        if (MODE == 0) {
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(f0, f2, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(f0, f3, acc[1], 0, 0, 0);
            acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(f1, f2, acc[2], 0, 0, 0);
            acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(f1, f3, acc[3], 0, 0, 0);
        } else {
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, b0, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, b1, acc[1], 0, 0, 0);
            acc[2] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, b0, acc[2], 0, 0, 0);
            acc[3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, b1, acc[3], 0, 0, 0);
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[q][i];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

constexpr int kWgs = 1024;      // four work-groups of four waves per compute unit

// Do vector-ALU work and matrix instructions of two waves on one SIMD run at the same time?  Eight waves per
// work-group, two per SIMD: waves 0-3 run `valu_iters` rounds of sixteen independent multiply-adds, waves
// 4-7 `mfma_iters` dependent matrix instructions (MODE as above).  Timed alone (the other count zero) and
// together: together = max of the two means they overlap, together = sum means they exclude each other.
template <int MODE>
__global__ __launch_bounds__(512) void coexec_kernel(const float* __restrict__ in, float* __restrict__ out,
                                                     int valu_iters, int mfma_iters) {
    const int wave = threadIdx.x >> 6;
    float x[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = in[(threadIdx.x + 64 * i) & 1023];
    floatx16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
    if (wave < 4) {
        for (int it = 0; it < valu_iters; ++it) {
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = fmaf(x[i], 1.0001f, 0.5f);
        }
    } else if (MODE == 0) {
        for (int it = 0; it < mfma_iters; ++it) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(x[0], x[1], acc, 0, 0, 0);
    } else {
        halfx8 a, b;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a[i] = (_Float16)x[i];
            b[i] = (_Float16)x[i + 8];
        }
        for (int it = 0; it < mfma_iters; ++it) acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc, 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += x[i] + acc[i];
    out[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

}  // namespace
}  // namespace elm

using namespace elm;

extern "C" size_t elm_rnn_probe_workspace_bytes(void) { return (size_t)2 << 30; }

extern "C" int elm_rnn_probe_ceilings(double* mfma_f32_tflops, double* mfma_f16_tflops, double* copy_gbs,
                                      double* valu_overlap_f32, double* valu_overlap_f16,
                                      void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (mfma_f32_tflops == nullptr || mfma_f16_tflops == nullptr || copy_gbs == nullptr) return ELM_EINVAL;
    if (workspace == nullptr || workspace_bytes < elm_rnn_probe_workspace_bytes()) return ELM_EWORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    float* in = static_cast<float*>(workspace);                 // 1024 operand seeds
    float* out = in + 1024;                                     // kWgs * 256 results
    std::vector<float> seeds(1024);
    uint64_t state = 0x1911013252ull;
    for (float& v : seeds) {
        state = state * 6364136223846793005ull + 1442695040888963407ull;
        v = ((float)((state >> 40) & 0xffff) / 65536.0f - 0.5f) * 0.01f;
    }
    ELM_HIP_TRY(hipMemcpyAsync(in, seeds.data(), seeds.size() * sizeof(float), hipMemcpyHostToDevice, stream));
    hipEvent_t a = nullptr, b = nullptr;
    ELM_HIP_TRY(hipEventCreate(&a));
    {
        const hipError_t eb = hipEventCreate(&b);
        if (eb != hipSuccess) {
            (void)hipEventDestroy(a);
            set_hip_error(eb, "hipEventCreate");
            return ELM_EHIP;
        }
    }
    auto timed = [&](auto&& launch, float* ms) -> hipError_t {
        launch();                                               // warm-up
        hipError_t e = hipEventRecord(a, stream);
        if (e == hipSuccess) launch();
        if (e == hipSuccess) e = hipGetLastError();
        if (e == hipSuccess) e = hipEventRecord(b, stream);
        if (e == hipSuccess) e = hipEventSynchronize(b);
        if (e == hipSuccess) e = hipEventElapsedTime(ms, a, b);
        return e;
    };
    int rc = ELM_OK;
    float ms = 0.0f;
    const int it32 = 100000, it16 = 200000;
    hipError_t e = timed([&] { hipLaunchKernelGGL(mfma_loop_kernel<0>, dim3(kWgs), dim3(256), 0, stream, in, out, it32); }, &ms);
    if (e == hipSuccess) {
        *mfma_f32_tflops = 32.0 * 32 * 2 * 2 * 4.0 * it32 * 4 * kWgs / (ms * 1e-3) / 1e12;
        e = timed([&] { hipLaunchKernelGGL(mfma_loop_kernel<1>, dim3(kWgs), dim3(256), 0, stream, in, out, it16); }, &ms);
    }
    if (e == hipSuccess) {
        *mfma_f16_tflops = 32.0 * 32 * 16 * 2 * 4.0 * it16 * 4 * kWgs / (ms * 1e-3) / 1e12;
        const size_t half = workspace_bytes / 2 / sizeof(float4);
        const float4* src = static_cast<const float4*>(workspace);
        float4* dst = static_cast<float4*>(workspace) + half;
        e = timed([&] { hipLaunchKernelGGL(copy_kernel, dim3(8192), dim3(256), 0, stream, src, dst, half); }, &ms);
        if (e == hipSuccess) *copy_gbs = 2.0 * half * sizeof(float4) / (ms * 1e-3) / 1e9;
    }
    // overlap of vector work with the matrix instructions of another wave of the same SIMD: the share of the
    // shorter of the two loops that is hidden when both run together (1 = they overlap, 0 = one waits)
    for (int mode = 0; mode < 2 && e == hipSuccess; ++mode) {
        double* dst = mode == 0 ? valu_overlap_f32 : valu_overlap_f16;
        if (dst == nullptr) continue;
        const int vi = 20000, mi = mode == 0 ? 30000 : 60000;      // about 2e6 cycles each
        float t[3] = {0.0f, 0.0f, 0.0f};
        const int counts[3][2] = {{vi, 0}, {0, mi}, {vi, mi}};
        for (int c = 0; c < 3 && e == hipSuccess; ++c) {
            e = timed([&] {
                if (mode == 0)
                    hipLaunchKernelGGL(coexec_kernel<0>, dim3(256), dim3(512), 0, stream, in, out, counts[c][0], counts[c][1]);
                else
                    hipLaunchKernelGGL(coexec_kernel<1>, dim3(256), dim3(512), 0, stream, in, out, counts[c][0], counts[c][1]);
            }, &t[c]);
        }
        if (e == hipSuccess) {
            const double shorter = t[0] < t[1] ? t[0] : t[1];
            double ov = (t[0] + t[1] - t[2]) / shorter;
            *dst = ov < 0.0 ? 0.0 : ov > 1.0 ? 1.0 : ov;
        }
    }
    if (e != hipSuccess) {
        set_hip_error(e, "ceilings probe");
        rc = ELM_EHIP;
    }
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    return rc;
}
