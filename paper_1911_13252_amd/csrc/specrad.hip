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
constexpr int KC = 128;     // contraction indices staged in LDS at a time

// out = (M / ||M||_F)^2 with ||M||_F^2 = the sum of partial_prev[0 .. nprev) (summed in index order by
// every work-group, so all of them scale by the same value); partial[block] = sum of squares of the
// block's entries of out; work-group (0, 0) also stores ||M||_F in norm_slot[0].
__global__ __launch_bounds__(256) void square_kernel(const double* __restrict__ M, double* __restrict__ out,
                                                     int n, const double* __restrict__ partial_prev, int nprev,
                                                     double* __restrict__ partial, double* __restrict__ norm_slot) {
    // the row panel and the column panel of this tile, KC contraction indices at a time (all of them for
    // n <= 128: one round of loads and one barrier per squaring, which is what a chain of 48 dependent
    // 100 x 100 squarings is made of)
    __shared__ double As[TS][KC + 1], Bs[KC][TS + 1];
    __shared__ double red[256];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;      // a thread owns a 2 x 2 patch
    const int row0 = blockIdx.y * TS, col0 = blockIdx.x * TS;
    double acc[2][2] = {{0.0, 0.0}, {0.0, 0.0}};
    for (int k0 = 0; k0 < n; k0 += KC) {
        const int kc = min(KC, n - k0);
        for (int e = tid; e < TS * KC; e += 256) {
            const int r = e / KC, c = e - r * KC;                   // As: row r, contraction index c
            As[r][c] = (row0 + r < n && c < kc) ? M[(size_t)(row0 + r) * n + k0 + c] : 0.0;
            const int kr = e / TS, cc = e - kr * TS;                // Bs: contraction index kr, column cc
            Bs[kr][cc] = (kr < kc && col0 + cc < n) ? M[(size_t)(k0 + kr) * n + col0 + cc] : 0.0;
        }
        __syncthreads();
#pragma unroll 8
        for (int k = 0; k < kc; ++k) {
            const double a0 = As[2 * ty][k], a1 = As[2 * ty + 1][k];
            const double b0 = Bs[k][2 * tx], b1 = Bs[k][2 * tx + 1];
            acc[0][0] = fma(a0, b0, acc[0][0]);
            acc[0][1] = fma(a0, b1, acc[0][1]);
            acc[1][0] = fma(a1, b0, acc[1][0]);
            acc[1][1] = fma(a1, b1, acc[1][1]);
        }
        __syncthreads();
    }
    double s2 = 0.0;
    for (int i = 0; i < nprev; ++i) s2 += partial_prev[i];
    const double nrm = sqrt(s2);
    if (tid == 0 && blockIdx.x == 0 && blockIdx.y == 0) norm_slot[0] = nrm;
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

// one allocation: both matrices, two sets of per-work-group partial sums (used in turn), the norms
struct DeviceBuffers {
    double* base = nullptr;
    double* m[2] = {nullptr, nullptr};
    double* partial = nullptr;
    double* norms = nullptr;
    hipError_t allocate(size_t nn, size_t nblocks, size_t nnorms) {
        hipError_t e = hipMalloc(&base, (2 * nn + 2 * nblocks + nnorms) * sizeof(double));
        if (e != hipSuccess) return e;
        m[0] = base;
        m[1] = base + nn;
        partial = m[1] + nn;
        norms = partial + 2 * nblocks;
        return hipSuccess;
    }
    ~DeviceBuffers() {
        if (base != nullptr) (void)hipFree(base);
    }
};

}  // namespace

hipError_t spectral_radius_device(const double* A, int n, double* rho_out) {
    constexpr int kMaxSquarings = 48;    // 2^-48 |log ||B^2||| is below double rounding of log rho
    constexpr int kBatch = 8;            // squarings enqueued between two looks at the norms
    double nf2 = 0.0;
    for (size_t i = 0; i < (size_t)n * n; ++i) nf2 += A[i] * A[i];
    const double nf = std::sqrt(nf2);
    if (nf == 0.0) {
        *rho_out = 0.0;
        return hipSuccess;
    }
    const int tiles = (n + TS - 1) / TS, nblocks = tiles * tiles;
    DeviceBuffers d;
    hipError_t e = d.allocate((size_t)n * n, (size_t)nblocks, kMaxSquarings + 1);
    if (e == hipSuccess) e = hipMemcpy(d.m[0], A, (size_t)n * n * sizeof(double), hipMemcpyHostToDevice);
    // the first squaring reads ||A||_F^2 as a single partial sum
    if (e == hipSuccess) e = hipMemcpy(d.partial + nblocks, &nf2, sizeof(double), hipMemcpyHostToDevice);
    if (e != hipSuccess) return e;

    double norms[kMaxSquarings + 1];
    double log_rho = std::log(nf), w = 1.0, prev = -1.0;
    int settled = 0;
    for (int base = 0; base < kMaxSquarings; base += kBatch) {
        // squaring `it` writes its partial sums to set it & 1 and reads those of squaring it - 1 from the
        // other set (the very first one reads the single entry ||A||_F^2 placed there by the host); it
        // stores the norm of its input, so one norm kernel per batch supplies the last output's norm
        for (int it = base; it < base + kBatch; ++it) {
            hipLaunchKernelGGL(square_kernel, dim3(tiles, tiles), dim3(256), 0, nullptr, d.m[it & 1],
                               d.m[(it + 1) & 1], n, d.partial + ((it + 1) & 1) * nblocks, it == 0 ? 1 : nblocks,
                               d.partial + (it & 1) * nblocks, d.norms + it);
        }
        hipLaunchKernelGGL(norm_kernel, dim3(1), dim3(64), 0, nullptr, d.partial + ((base + kBatch - 1) & 1) * nblocks,
                           nblocks, d.norms + base + kBatch);
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
