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

constexpr int TS = 32;      // a work-group owns a 32 x 32 tile of the square, a wave a 16 x 16 quarter of it

typedef double doublex4 __attribute__((ext_vector_type(4)));

// out = (M / ||M||_F)^2 with ||M||_F^2 = the sum of partial_prev[0 .. nprev) (summed in index order by
// every work-group, so all of them scale by the same value); partial[block] = sum of squares of the
// block's entries of out; work-group (0, 0) also stores ||M||_F in norm_slot[0].
// The product runs on the float64 matrix instruction (16 x 16 x 4): lane (r = lane % 16, q = lane / 16)
// supplies M[row0 + r][4s + q] and M[4s + q][col0 + r] for k-step s; its result register v is row 4v + q,
// column r of the 16 x 16 tile (the float64 form interleaves the rows, unlike the float32 one).  Operands come straight from L2 (a 100 x 100 matrix is 80 KB), eight k-steps of
// loads in flight: a squaring of the chain of 48 is then little more than a launch and one round of loads.
__global__ __launch_bounds__(256) void square_kernel(const double* __restrict__ M, double* __restrict__ out,
                                                     int n, const double* __restrict__ partial_prev, int nprev,
                                                     double* __restrict__ partial, double* __restrict__ norm_slot) {
    __shared__ double red[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, q = lane >> 4;
    const int row0 = blockIdx.y * TS + (wave >> 1) * 16, col0 = blockIdx.x * TS + (wave & 1) * 16;
    const bool row_ok = row0 + r < n, col_ok = col0 + r < n;
    const double* arow = M + (size_t)(row0 + r) * n;        // read only where row_ok
    const double* bcol = M + col0 + r;                      // read only where col_ok
    doublex4 acc = {0.0, 0.0, 0.0, 0.0};
    constexpr int U = 8;                                    // k-steps per batch of loads
    const int steps = (n + 3) / 4;
    double a[U], b[U];
    auto fetch = [&](int s0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = 4 * (s0 + u) + q;
            a[u] = (row_ok && k < n) ? arow[k] : 0.0;
            b[u] = (col_ok && k < n) ? bcol[(size_t)k * n] : 0.0;
        }
    };
    for (int s0 = 0; s0 < steps; s0 += U) {
        fetch(s0);
#pragma unroll
        for (int u = 0; u < U; ++u) acc = __builtin_amdgcn_mfma_f64_16x16x4f64(a[u], b[u], acc, 0, 0, 0);
    }
    double s2 = 0.0;
    for (int i = 0; i < nprev; ++i) s2 += partial_prev[i];
    const double nrm = sqrt(s2);
    if (tid == 0 && blockIdx.x == 0 && blockIdx.y == 0) norm_slot[0] = nrm;
    const double sc = 1.0 / (nrm * nrm);
    double ss = 0.0;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int rr = row0 + 4 * v + q, cc = col0 + r;
        if (rr < n && cc < n) {
            const double val = acc[v] * sc;
            out[(size_t)rr * n + cc] = val;
            ss += val * val;
        }
    }
    // fixed-order sums: lanes of a wave by halving distances, then the four waves in index order
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) ss += __shfl_down(ss, d, 64);
    if (lane == 0) red[wave] = ss;
    __syncthreads();
    if (tid == 0) partial[blockIdx.y * gridDim.x + blockIdx.x] = ((red[0] + red[1]) + red[2]) + red[3];
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

hipError_t spectral_radius_device(const double* A, int n, double* rho_out, hipStream_t stream) {
    constexpr int kMaxSquarings = 48;    // 2^-48 |log ||B^2||| is below double rounding of log rho
    constexpr int kBatch = 16;           // squarings enqueued between two looks at the norms
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
    // every copy and launch below is on the caller's stream; the host buffers of the uploads stay alive until
    // the first read-back has synchronised that stream
    if (e == hipSuccess)
        e = hipMemcpyAsync(d.m[0], A, (size_t)n * n * sizeof(double), hipMemcpyHostToDevice, stream);
    // the first squaring reads ||A||_F^2 as a single partial sum
    if (e == hipSuccess)
        e = hipMemcpyAsync(d.partial + nblocks, &nf2, sizeof(double), hipMemcpyHostToDevice, stream);
    if (e != hipSuccess) {
        (void)hipStreamSynchronize(stream);       // nothing may still read A or nf2 after the return
        return e;
    }

    double norms[kMaxSquarings + 1];
    double log_rho = std::log(nf), w = 1.0, prev = -1.0;
    int settled = 0;
    for (int base = 0; base < kMaxSquarings; base += kBatch) {
        // squaring `it` writes its partial sums to set it & 1 and reads those of squaring it - 1 from the
        // other set (the very first one reads the single entry ||A||_F^2 placed there by the host); it
        // stores the norm of its input, so one norm kernel per batch supplies the last output's norm
        for (int it = base; it < base + kBatch; ++it) {
            hipLaunchKernelGGL(square_kernel, dim3(tiles, tiles), dim3(256), 0, stream, d.m[it & 1],
                               d.m[(it + 1) & 1], n, d.partial + ((it + 1) & 1) * nblocks, it == 0 ? 1 : nblocks,
                               d.partial + (it & 1) * nblocks, d.norms + it);
        }
        hipLaunchKernelGGL(norm_kernel, dim3(1), dim3(64), 0, stream, d.partial + ((base + kBatch - 1) & 1) * nblocks,
                           nblocks, d.norms + base + kBatch);
        e = hipGetLastError();
        if (e == hipSuccess)
            e = hipMemcpyAsync(norms + base + 1, d.norms + base + 1, kBatch * sizeof(double), hipMemcpyDeviceToHost,
                               stream);
        const hipError_t es = hipStreamSynchronize(stream);     // also on failure: the buffers are freed on return
        if (e == hipSuccess) e = es;
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
