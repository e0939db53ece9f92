// Spectral radius of the Elman recurrent matrix (step 1 of the paper's Algorithm "S-R-ELM" with the
// benchmark's "recurrent scaled to spectral radius 0.9") on the device, in float64.
//
// Gelfand's formula rho = lim ||A^k||^(1/k) along k = 2^i with renormalised repeated squaring:
// A^(2^i) = exp(2^i s_i) B_i with ||B_i||_F = 1 and s_{i+1} = s_i + 2^-(i+1) log ||B_i^2||_F.
// The device keeps the un-normalised squares M_{i+1} = (M_i / ||M_i||)^2 and their Frobenius norms;
// the host turns the norm sequence into rho.  All sums run in a fixed order (deterministic).

#include <cmath>
#include <vector>

#include "internal.h"

namespace elm {
namespace {

constexpr int TS = 32;

// out = (M / norm_prev)^2, partial[block] = sum of squares of the block's entries of out
__global__ __launch_bounds__(256) void square_kernel(const double* __restrict__ M, double* __restrict__ out,
                                                     int n, const double* __restrict__ norm_prev,
                                                     double* __restrict__ partial) {
    __shared__ double As[TS][TS + 1], Bs[TS][TS + 1];
    __shared__ double red[256];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;      // a thread owns a 2 x 2 patch
    const int row0 = blockIdx.y * TS, col0 = blockIdx.x * TS;
    double acc[2][2] = {{0.0, 0.0}, {0.0, 0.0}};
    for (int k0 = 0; k0 < n; k0 += TS) {
        for (int e = tid; e < TS * TS; e += 256) {
            const int r = e / TS, c = e - r * TS;
            As[r][c] = (row0 + r < n && k0 + c < n) ? M[(size_t)(row0 + r) * n + k0 + c] : 0.0;
            Bs[r][c] = (k0 + r < n && col0 + c < n) ? M[(size_t)(k0 + r) * n + col0 + c] : 0.0;
        }
        __syncthreads();
#pragma unroll 8
        for (int k = 0; k < TS; ++k) {
            const double a0 = As[2 * ty][k], a1 = As[2 * ty + 1][k];
            const double b0 = Bs[k][2 * tx], b1 = Bs[k][2 * tx + 1];
            acc[0][0] = fma(a0, b0, acc[0][0]);
            acc[0][1] = fma(a0, b1, acc[0][1]);
            acc[1][0] = fma(a1, b0, acc[1][0]);
            acc[1][1] = fma(a1, b1, acc[1][1]);
        }
        __syncthreads();
    }
    const double nrm = norm_prev[0];
    const double sc = 1.0 / (nrm * nrm);
    double ss = 0.0;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int r = row0 + 2 * ty + i, c = col0 + 2 * tx + j;
            if (r < n && c < n) {
                const double v = acc[i][j] * sc;
                out[(size_t)r * n + c] = v;
                ss += v * v;
            }
        }
    red[tid] = ss;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (tid < s) red[tid] += red[tid + s];
        __syncthreads();
    }
    if (tid == 0) partial[blockIdx.y * gridDim.x + blockIdx.x] = red[0];
}

__global__ void norm_kernel(const double* __restrict__ partial, int nblocks, double* __restrict__ norm_out) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        double s = 0.0;
        for (int i = 0; i < nblocks; ++i) s += partial[i];
        norm_out[0] = sqrt(s);
    }
}

struct DeviceBuffers {
    double* m[2] = {nullptr, nullptr};
    double* partial = nullptr;
    double* norms = nullptr;
    ~DeviceBuffers() {
        for (double* q : {m[0], m[1], partial, norms})
            if (q != nullptr) (void)hipFree(q);
    }
};

}  // namespace

hipError_t spectral_radius_device(const double* A, int n, double* rho_out) {
    constexpr int kMaxSquarings = 48;    // 2^-48 |log ||B^2||| is below double rounding of log rho
    constexpr int kBatch = 8;            // squarings enqueued between two looks at the norms
    double nf = 0.0;
    for (size_t i = 0; i < (size_t)n * n; ++i) nf += A[i] * A[i];
    nf = std::sqrt(nf);
    if (nf == 0.0) {
        *rho_out = 0.0;
        return hipSuccess;
    }
    const int tiles = (n + TS - 1) / TS, nblocks = tiles * tiles;
    DeviceBuffers d;
    hipError_t e = hipMalloc(&d.m[0], (size_t)n * n * sizeof(double));
    if (e == hipSuccess) e = hipMalloc(&d.m[1], (size_t)n * n * sizeof(double));
    if (e == hipSuccess) e = hipMalloc(&d.partial, (size_t)nblocks * sizeof(double));
    if (e == hipSuccess) e = hipMalloc(&d.norms, (kMaxSquarings + 1) * sizeof(double));
    if (e == hipSuccess) e = hipMemcpy(d.m[0], A, (size_t)n * n * sizeof(double), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(d.norms, &nf, sizeof(double), hipMemcpyHostToDevice);
    if (e != hipSuccess) return e;

    double norms[kMaxSquarings + 1];
    double log_rho = std::log(nf), w = 1.0, prev = -1.0;
    int settled = 0;
    for (int base = 0; base < kMaxSquarings; base += kBatch) {
        for (int it = base; it < base + kBatch; ++it) {
            hipLaunchKernelGGL(square_kernel, dim3(tiles, tiles), dim3(256), 0, nullptr, d.m[it & 1],
                               d.m[(it + 1) & 1], n, d.norms + it, d.partial);
            hipLaunchKernelGGL(norm_kernel, dim3(1), dim3(64), 0, nullptr, d.partial, nblocks, d.norms + it + 1);
        }
        e = hipGetLastError();
        if (e == hipSuccess)
            e = hipMemcpy(norms + base + 1, d.norms + base + 1, kBatch * sizeof(double), hipMemcpyDeviceToHost);
        if (e != hipSuccess) return e;
        for (int it = base; it < base + kBatch; ++it) {
            const double nc = norms[it + 1];
            if (nc == 0.0) {                 // nilpotent
                *rho_out = 0.0;
                return hipSuccess;
            }
            if (!std::isfinite(nc)) return hipErrorUnknown;
            w *= 0.5;
            // once ||B_i^2|| has stopped changing (B_i has converged to the dominant rank-one part)
            // the rest of the series is geometric: sum_{k>i} 2^-k log nc = 2^-i log nc
            settled = (std::fabs(nc - prev) <= 4e-16 * nc) ? settled + 1 : 0;
            if (settled >= 2) {
                *rho_out = std::exp(log_rho + 2.0 * w * std::log(nc));
                return hipSuccess;
            }
            prev = nc;
            log_rho += w * std::log(nc);
        }
    }
    *rho_out = std::exp(log_rho);
    return hipSuccess;
}

}  // namespace elm
