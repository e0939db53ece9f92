// Stage 2b: from the R factor of [H | T] to beta (the paper's section "Computing beta": the triangular
// back-solve R11 beta = R12, i.e. R beta = z with z = Q^T Y), plus float64-residual iterative
// refinement of beta and the prediction product Y = H beta (the paper's output equation
// y_hat = sum_i beta_i f_i).
//
// R = [R11 R12; 0 R22] (np x np float32, upper triangular).  beta0 = R11^{-1} R12 in float64
// arithmetic.  A refinement step streams H once:  r = T - H beta and g = H^T r accumulated in
// float64, then  beta += (R11^T R11)^{-1} g  by one forward and one backward triangular solve.

#include "internal.h"

namespace elm {
namespace {

constexpr int kThreads = 256;
constexpr int kTileRows = 32;

// ---- triangular solves on one work-group: blocks of 32, diagonal block by one wave in registers
// y (LDS, doubles, length >= 32*ceil(L/32)) is overwritten by the solution of R11 x = y.
// lane k's value in every lane (k is a constant after unrolling: two scalar broadcasts instead of a trip
// through the LDS crossbar, on the critical path of every elimination step)
__device__ __forceinline__ double lane_value(double v, int k) {
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), k);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), k);
    return __hiloint2double(hi, lo);
}

__device__ void solve_upper(const float* __restrict__ R, int np, int L, double* y) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int nb = (L + 31) / 32;
    for (int kb = nb - 1; kb >= 0; --kb) {
        const int c0 = kb * 32;
        if (tid < 64) {
            const int i = lane & 31, row = c0 + i;
            double drow[32];
#pragma unroll
            for (int l = 0; l < 32; ++l) {
                const int col = c0 + l;
                double v = (l == i) ? 1.0 : 0.0;
                if (row < L && col < L) v = (double)R[(size_t)row * np + col];
                drow[l] = v;
            }
            double yi = (row < L) ? y[row] : 0.0;
            double diag = 1.0;                 // this lane's diagonal entry; its reciprocal is taken off the chain
#pragma unroll
            for (int l = 0; l < 32; ++l)
                if (l == i) diag = drow[l];
            const double dinv = 1.0 / diag;
#pragma unroll
            for (int k = 31; k >= 0; --k) {
                const double xk = lane_value(yi, k) * lane_value(dinv, k);
                if (i == k) yi = xk;
                else if (i < k) yi -= drow[k] * xk;
            }
            if (lane < 32 && row < L) y[row] = yi;
        }
        __syncthreads();
        for (int i = tid; i < c0; i += kThreads) {
            double acc = 0.0;
            const float* rr = R + (size_t)i * np + c0;
            for (int l = 0; l < 32; ++l)
                if (c0 + l < L) acc += (double)rr[l] * y[c0 + l];
            y[i] -= acc;
        }
        __syncthreads();
    }
}

// y is overwritten by the solution of R11^T x = y.
__device__ void solve_upper_transposed(const float* __restrict__ R, int np, int L, double* y) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int nb = (L + 31) / 32;
    for (int kb = 0; kb < nb; ++kb) {
        const int c0 = kb * 32;
        if (tid < 64) {
            const int i = lane & 31, col = c0 + i;
            double dcol[32];      // dcol[l] = R[c0+l][c0+i]
#pragma unroll
            for (int l = 0; l < 32; ++l) {
                const int row = c0 + l;
                double v = (l == i) ? 1.0 : 0.0;
                if (row < L && col < L) v = (double)R[(size_t)row * np + col];
                dcol[l] = v;
            }
            double yi = (col < L) ? y[col] : 0.0;
            double diag = 1.0;
#pragma unroll
            for (int l = 0; l < 32; ++l)
                if (l == i) diag = dcol[l];
            const double dinv = 1.0 / diag;
#pragma unroll
            for (int k = 0; k < 32; ++k) {
                const double xk = lane_value(yi, k) * lane_value(dinv, k);
                if (i == k) yi = xk;
                else if (i > k) yi -= dcol[k] * xk;
            }
            if (lane < 32 && col < L) y[col] = yi;
        }
        __syncthreads();
        for (int jj = c0 + 32 + tid; jj < L; jj += kThreads) {
            double acc = 0.0;
            for (int l = 0; l < 32; ++l)
                if (c0 + l < L) acc += (double)R[(size_t)(c0 + l) * np + jj] * y[c0 + l];
            y[jj] -= acc;
        }
        __syncthreads();
    }
}

// beta0 = R11^{-1} R12, diagnostics of R.
__global__ __launch_bounds__(kThreads) void backsolve_kernel(const float* __restrict__ R, int np, int L,
                                                             int m, double* small) {
    __shared__ double y[544];
    __shared__ double sred[kThreads];
    __shared__ double smin[kThreads], smax[kThreads];
    const int tid = threadIdx.x;
    double* beta = small + SmallArea::BETA;
    double* scal = small + SmallArea::scal(L, m);

    // residual mass left in the T columns below row L, and the diagonal range of R11
    double rs = 0.0, dmin = 1e300, dmax = 0.0;
    for (int idx = tid; idx < m * m; idx += kThreads) {
        const int i = idx / m, jx = idx - i * m;
        if (jx >= i) {
            const double v = (double)R[(size_t)(L + i) * np + L + jx];
            rs += v * v;
        }
    }
    for (int k = tid; k < L; k += kThreads) {
        const double v = fabs((double)R[(size_t)k * np + k]);
        dmin = fmin(dmin, v);
        dmax = fmax(dmax, v);
    }
    sred[tid] = rs; smin[tid] = dmin; smax[tid] = dmax;
    __syncthreads();
    for (int s = kThreads / 2; s > 0; s >>= 1) {
        if (tid < s) {
            sred[tid] += sred[tid + s];
            smin[tid] = fmin(smin[tid], smin[tid + s]);
            smax[tid] = fmax(smax[tid], smax[tid + s]);
        }
        __syncthreads();
    }
    const bool deficient = !(smin[0] > 1.1920928955078125e-07 * smax[0]);
    if (tid == 0) {
        scal[3] = sred[0];
        scal[4] = smin[0];
        scal[5] = smax[0];
        scal[6] = deficient ? 1.0 : 0.0;
    }
    for (int c = 0; c < m; ++c) {
        for (int i = tid; i < 544; i += kThreads) y[i] = (i < L) ? (double)R[(size_t)i * np + L + c] : 0.0;
        __syncthreads();
        if (!deficient) solve_upper(R, np, L, y);
        for (int i = tid; i < L; i += kThreads) beta[(size_t)i * m + c] = deficient ? 0.0 : y[i];
        __syncthreads();
    }
}

// beta += (R11^T R11)^{-1} g
__global__ __launch_bounds__(kThreads) void refine_kernel(const float* __restrict__ R, int np, int L,
                                                          int m, double* small) {
    __shared__ double y[544];
    const int tid = threadIdx.x;
    double* beta = small + SmallArea::BETA;
    const double* grad = small + SmallArea::grad(L, m);
    const double* scal = small + SmallArea::scal(L, m);
    if (scal[6] != 0.0) return;       // rank deficient: leave beta alone
    for (int c = 0; c < m; ++c) {
        for (int i = tid; i < 544; i += kThreads) y[i] = (i < L) ? grad[(size_t)i * m + c] : 0.0;
        __syncthreads();
        solve_upper_transposed(R, np, L, y);
        solve_upper(R, np, L, y);
        for (int i = tid; i < L; i += kThreads) beta[(size_t)i * m + c] += y[i];
        __syncthreads();
    }
}

// One streaming pass over H.  MODE 0: per-work-group partial sums of g = H^T (T - H beta),
// ||T - H beta||^2 and ||H||^2.  MODE 1: Y = H beta.
template <int M, int MODE>
__global__ __launch_bounds__(kThreads) void stream_kernel(const float* __restrict__ H,
                                                          const float* __restrict__ T, int64_t N, int L,
                                                          int m, const double* __restrict__ beta,
                                                          double* __restrict__ part, float* __restrict__ Y) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int ldh = L + 1;
    double* bs = reinterpret_cast<double*>(smem);                        // [L][M]
    double* rs = bs + (size_t)L * M;                                     // [32][M]
    float* Hs = reinterpret_cast<float*>(rs + kTileRows * M);            // [32][ldh]
    __shared__ double sred[kThreads];

    const int tid = threadIdx.x;
    for (int idx = tid; idx < L * M; idx += kThreads) {
        const int jx = idx / M, c = idx - jx * M;
        bs[idx] = (c < m) ? beta[(size_t)jx * m + c] : 0.0;
    }
    double gacc[2][M];
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int c = 0; c < M; ++c) gacc[q][c] = 0.0;
    double rss = 0.0, h2 = 0.0;

    const int64_t ntiles = (N + kTileRows - 1) / kTileRows;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t r0 = tile * kTileRows;
        __syncthreads();                       // previous tile fully consumed (and bs written)
        for (int idx = tid; idx < kTileRows * L; idx += kThreads) {
            const int r = idx / L, c = idx - r * L;
            const int64_t row = r0 + r;
            const float v = (row < N) ? H[row * L + c] : 0.0f;
            Hs[r * ldh + c] = v;
            if (MODE == 0) h2 += (double)v * (double)v;
        }
        __syncthreads();
        {   // 8 lanes per row: partial dot products, then a shuffle reduction over the 8
            const int r = tid >> 3, sub = tid & 7;
            double acc[M];
#pragma unroll
            for (int c = 0; c < M; ++c) acc[c] = 0.0;
            for (int jx = sub; jx < L; jx += 8) {
                const double hv = (double)Hs[r * ldh + jx];
#pragma unroll
                for (int c = 0; c < M; ++c) acc[c] = fma(hv, bs[jx * M + c], acc[c]);
            }
#pragma unroll
            for (int c = 0; c < M; ++c) {
                acc[c] += __shfl_xor(acc[c], 1);
                acc[c] += __shfl_xor(acc[c], 2);
                acc[c] += __shfl_xor(acc[c], 4);
            }
            const int64_t row = r0 + r;
            if (sub == 0) {
#pragma unroll
                for (int c = 0; c < M; ++c) {
                    if (MODE == 0) {
                        double res = 0.0;
                        if (row < N && c < m) res = (double)T[row * m + c] - acc[c];
                        rs[r * M + c] = res;
                        rss += res * res;
                    } else if (row < N && c < m) {
                        Y[row * m + c] = (float)acc[c];
                    }
                }
            }
        }
        if (MODE == 0) {
            __syncthreads();
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int jx = tid + q * kThreads;
                if (jx < L) {
                    for (int r = 0; r < kTileRows; ++r) {
                        const double hv = (double)Hs[r * ldh + jx];
#pragma unroll
                        for (int c = 0; c < M; ++c) gacc[q][c] = fma(hv, rs[r * M + c], gacc[q][c]);
                    }
                }
            }
        }
    }
    if (MODE == 0) {
        double* mypart = part + (size_t)blockIdx.x * ((size_t)L * m + 2);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int jx = tid + q * kThreads;
            if (jx < L)
#pragma unroll
                for (int c = 0; c < M; ++c)
                    if (c < m) mypart[(size_t)jx * m + c] = gacc[q][c];
        }
        __syncthreads();
        sred[tid] = rss;
        __syncthreads();
        for (int s = kThreads / 2; s > 0; s >>= 1) {
            if (tid < s) sred[tid] += sred[tid + s];
            __syncthreads();
        }
        if (tid == 0) mypart[(size_t)L * m] = sred[0];
        __syncthreads();
        sred[tid] = h2;
        __syncthreads();
        for (int s = kThreads / 2; s > 0; s >>= 1) {
            if (tid < s) sred[tid] += sred[tid + s];
            __syncthreads();
        }
        if (tid == 0) mypart[(size_t)L * m + 1] = sred[0];
    }
}

// Same contract as stream_kernel for m <= 4 and L <= 512, organised for HBM rate: one wavefront
// owns a row at a time (lane l holds columns l, l+64, ...), beta and the gradient accumulators
// live in registers, the row dot products are reduced with wavefront shuffles, and there is no
// work-group barrier inside the row loop.
template <int M, int MODE, int EPL>
__global__ __launch_bounds__(kThreads) void stream_rows_kernel(const float* __restrict__ H,
                                                               const float* __restrict__ T, int64_t N, int L,
                                                               int m, const double* __restrict__ beta,
                                                               double* __restrict__ part,
                                                               float* __restrict__ Y) {
    // EPL = columns per lane (L <= 64 * EPL)
    __shared__ double wsum[EPL * 64 * M + 2];     // in-group sum of the 4 waves' results
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    double bt[EPL][M], gacc[EPL][M];
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        const int jx = e * 64 + lane;
#pragma unroll
        for (int c = 0; c < M; ++c) {
            bt[e][c] = (jx < L && c < m) ? beta[(size_t)jx * m + c] : 0.0;
            gacc[e][c] = 0.0;
        }
    }
    double rss = 0.0, h2 = 0.0;
    const int64_t wave_id = (int64_t)blockIdx.x * 4 + wave;
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    // the next row of this wave is requested before the current one is reduced
    float hn[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        const int jx = e * 64 + lane;
        hn[e] = (wave_id < N && jx < L) ? H[wave_id * L + jx] : 0.0f;
    }
    for (int64_t row = wave_id; row < N; row += nwaves) {
        float hv[EPL];
#pragma unroll
        for (int e = 0; e < EPL; ++e) hv[e] = hn[e];
        const int64_t nxt = row + nwaves;
        if (nxt < N) {
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                const int jx = e * 64 + lane;
                hn[e] = (jx < L) ? H[nxt * L + jx] : 0.0f;
            }
        }
        double dot[M];
#pragma unroll
        for (int c = 0; c < M; ++c) dot[c] = 0.0;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            const double h = (double)hv[e];
            if (MODE == 0) h2 = fma(h, h, h2);
#pragma unroll
            for (int c = 0; c < M; ++c) dot[c] = fma(h, bt[e][c], dot[c]);
        }
#pragma unroll
        for (int c = 0; c < M; ++c) {
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) dot[c] += __shfl_xor(dot[c], off);
        }
        if (MODE == 0) {
            double res[M];
#pragma unroll
            for (int c = 0; c < M; ++c) {
                res[c] = (c < m) ? (double)T[row * m + c] - dot[c] : 0.0;
                if (lane == 0) rss = fma(res[c], res[c], rss);
            }
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                const double h = (double)hv[e];
#pragma unroll
                for (int c = 0; c < M; ++c) gacc[e][c] = fma(h, res[c], gacc[e][c]);
            }
        } else if (lane < m) {
            double v = dot[0];
#pragma unroll
            for (int c = 1; c < M; ++c) v = (lane == c) ? dot[c] : v;
            Y[row * m + lane] = (float)v;
        }
    }
    if (MODE == 0) {
        // fixed-order sum over the 4 waves (wave 0 first), then one partial record per work-group
        for (int off = 32; off > 0; off >>= 1) h2 += __shfl_xor(h2, off);
        for (int w = 0; w < 4; ++w) {
            if (wave == w) {
#pragma unroll
                for (int e = 0; e < EPL; ++e)
#pragma unroll
                    for (int c = 0; c < M; ++c) {
                        const int idx = (e * 64 + lane) * M + c;
                        wsum[idx] = (w == 0) ? gacc[e][c] : wsum[idx] + gacc[e][c];
                    }
                if (lane == 0) {
                    wsum[EPL * 64 * M] = (w == 0) ? rss : wsum[EPL * 64 * M] + rss;
                    wsum[EPL * 64 * M + 1] = (w == 0) ? h2 : wsum[EPL * 64 * M + 1] + h2;
                }
            }
            __syncthreads();
        }
        double* mypart = part + (size_t)blockIdx.x * ((size_t)L * m + 2);
        for (int idx = tid; idx < L * m; idx += kThreads) {
            const int jx = idx / m, c = idx - jx * m;
            mypart[idx] = wsum[jx * M + c];
        }
        if (tid < 2) mypart[(size_t)L * m + tid] = wsum[EPL * 64 * M + tid];
    }
}

// Same contract for narrow layers (L <= LG, m <= 4): a wave handles 64 / LG rows at a time, LG lanes
// per row and one column per lane, so a 10-column matrix keeps 40 of 64 lanes busy instead of 10 and a
// row's dot products need log2(LG) exchange steps instead of six.  Rows are contiguous in memory, so a
// wave's loads stay coalesced.  Partial sums are added in a fixed order, as in stream_rows_kernel.
template <int M, int MODE, int LG>
__global__ __launch_bounds__(kThreads) void stream_narrow_kernel(const float* __restrict__ H,
                                                                 const float* __restrict__ T, int64_t N, int L,
                                                                 int m, const double* __restrict__ beta,
                                                                 double* __restrict__ part,
                                                                 float* __restrict__ Y) {
    constexpr int RPW = 64 / LG;                   // rows a wave covers with one load
    constexpr int UNR = 4;                         // independent loads / reductions in flight per lane
    __shared__ double wsum[LG * M + 2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = lane % LG, slot = lane / LG;     // column of this lane, row slot inside a group of RPW rows
    double bt[M], gacc[M];
#pragma unroll
    for (int c = 0; c < M; ++c) {
        bt[c] = (j < L && c < m) ? beta[(size_t)j * m + c] : 0.0;
        gacc[c] = 0.0;
    }
    double rss = 0.0, h2 = 0.0;
    // a wave takes UNR * RPW consecutive rows per pass: lane (slot, j) the rows base + u * RPW + slot
    const int64_t first = ((int64_t)blockIdx.x * 4 + wave) * (UNR * RPW);
    const int64_t stride = (int64_t)gridDim.x * 4 * (UNR * RPW);
    float hn[UNR];                                 // the next pass is requested one pass ahead
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
        const int64_t row = first + u * RPW + slot;
        hn[u] = (row < N && j < L) ? H[row * L + j] : 0.0f;
    }
    for (int64_t base = first; base < N; base += stride) {
        float hv[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            hv[u] = hn[u];
            const int64_t nxt = base + stride + u * RPW + slot;
            hn[u] = (nxt < N && j < L) ? H[nxt * L + j] : 0.0f;
        }
        double dot[UNR][M];
#pragma unroll
        for (int u = 0; u < UNR; ++u)
#pragma unroll
            for (int c = 0; c < M; ++c) dot[u][c] = (double)hv[u] * bt[c];
#pragma unroll
        for (int off = LG / 2; off > 0; off >>= 1)
#pragma unroll
            for (int u = 0; u < UNR; ++u)
#pragma unroll
                for (int c = 0; c < M; ++c) dot[u][c] += __shfl_xor(dot[u][c], off);
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int64_t row = base + u * RPW + slot;
            const double h = (double)hv[u];
            if (MODE == 0) {
                h2 = fma(h, h, h2);
                if (row < N) {
#pragma unroll
                    for (int c = 0; c < M; ++c) {
                        const double res = (c < m) ? (double)T[row * m + c] - dot[u][c] : 0.0;
                        if (j == 0) rss = fma(res, res, rss);
                        gacc[c] = fma(h, res, gacc[c]);
                    }
                }
            } else if (row < N && j < m) {
                double v = dot[u][0];
#pragma unroll
                for (int c = 1; c < M; ++c) v = (j == c) ? dot[u][c] : v;
                Y[row * m + j] = (float)v;
            }
        }
    }
    if (MODE == 0) {
        // the row slots of a wave first (lanes LG, 2 LG, ... apart), then the 4 waves in order
#pragma unroll
        for (int off = LG; off < 64; off <<= 1) {
#pragma unroll
            for (int c = 0; c < M; ++c) gacc[c] += __shfl_xor(gacc[c], off);
            rss += __shfl_xor(rss, off);
        }
        for (int off = 32; off > 0; off >>= 1) h2 += __shfl_xor(h2, off);
        for (int w = 0; w < 4; ++w) {
            if (wave == w && lane < LG) {
#pragma unroll
                for (int c = 0; c < M; ++c) {
                    const int idx = lane * M + c;
                    wsum[idx] = (w == 0) ? gacc[c] : wsum[idx] + gacc[c];
                }
                if (lane == 0) {
                    wsum[LG * M] = (w == 0) ? rss : wsum[LG * M] + rss;
                    wsum[LG * M + 1] = (w == 0) ? h2 : wsum[LG * M + 1] + h2;
                }
            }
            __syncthreads();
        }
        double* mypart = part + (size_t)blockIdx.x * ((size_t)L * m + 2);
        for (int idx = tid; idx < L * m; idx += kThreads) {
            const int jx = idx / m, c = idx - jx * m;
            mypart[idx] = wsum[jx * M + c];
        }
        if (tid < 2) mypart[(size_t)L * m + tid] = wsum[LG * M + tid];
    }
}

// Sum the per-work-group partials in a fixed order.  Thread (o, q) of a work-group adds the
// partials w = q, q+8, ... of output o; the 8 sub-sums are then added in order.
__global__ __launch_bounds__(kThreads) void reduce_partials_kernel(const double* __restrict__ part,
                                                                   int nparts, int L, int m,
                                                                   double* small, int accumulate) {
    __shared__ double sub[8][32];
    const int tid = threadIdx.x, ol = tid & 31, q = tid >> 5;
    const int nout = L * m + 2;
    const int o = blockIdx.x * 32 + ol;
    double s = 0.0;
    if (o < nout) {
        // partials w = q, q + 8, ... in that order; eight loads are in flight at a time
        for (int w0 = q; w0 < nparts; w0 += 64) {
            double v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int w = w0 + 8 * u;
                v[u] = (w < nparts) ? part[(size_t)w * nout + o] : 0.0;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
    }
    sub[q][ol] = s;
    __syncthreads();
    if (q == 0 && o < nout) {
        double t = 0.0;
#pragma unroll
        for (int r = 0; r < 8; ++r) t += sub[r][ol];
        // [0] rss, [1] sum H^2 behind the gradient; a later chunk of rows adds to the earlier ones
        double* dst = (o < L * m) ? small + SmallArea::grad(L, m) + o : small + SmallArea::scal(L, m) + (o - L * m);
        *dst = accumulate ? *dst + t : t;
    }
}

// scal[2] = ||g||_F^2
__global__ __launch_bounds__(kThreads) void grad_norm_kernel(int L, int m, double* small) {
    __shared__ double sred[kThreads];
    const int tid = threadIdx.x;
    const double* grad = small + SmallArea::grad(L, m);
    double g2 = 0.0;
    for (int o = tid; o < L * m; o += kThreads) g2 = fma(grad[o], grad[o], g2);
    sred[tid] = g2;
    __syncthreads();
    for (int st = kThreads / 2; st > 0; st >>= 1) {
        if (tid < st) sred[tid] += sred[tid + st];
        __syncthreads();
    }
    if (tid == 0) small[SmallArea::scal(L, m) + 2] = sred[0];
}

__global__ void export_beta_kernel(const double* __restrict__ beta, int count, float* b32, double* b64) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) {
        b32[i] = (float)beta[i];
        if (b64 != nullptr) b64[i] = beta[i];
    }
}

size_t stream_lds_bytes(int L, int M) {
    return ((size_t)L * M + kTileRows * M) * sizeof(double) + (size_t)kTileRows * (L + 1) * sizeof(float);
}

int stream_grid(int64_t N) {
    const int64_t ntiles = (N + kTileRows - 1) / kTileRows;
    return (int)(ntiles < 1024 ? ntiles : 1024);      // <= 1024 partial records in the workspace
}

template <int MODE>
hipError_t launch_stream(const float* H, const float* T, int64_t N, int L, int m, const double* beta,
                         double* part, float* Y, hipStream_t stream) {
    const int grid = stream_grid(N);
    int M = 1;
    while (M < m) M *= 2;
    if (M <= 4 && L <= 32) {        // narrow layers: several rows per wave
#define ELM_NARROW_LAUNCH(MM, GG)                                                                          \
    hipLaunchKernelGGL((stream_narrow_kernel<MM, MODE, GG>), dim3(grid), dim3(kThreads), 0, stream, H, T, N, L, \
                       m, beta, part, Y)
#define ELM_NARROW_CASE(MM)                                 \
    if (L <= 8) ELM_NARROW_LAUNCH(MM, 8);                   \
    else if (L <= 16) ELM_NARROW_LAUNCH(MM, 16);            \
    else ELM_NARROW_LAUNCH(MM, 32)
        switch (M) {
            case 1: ELM_NARROW_CASE(1); break;
            case 2: ELM_NARROW_CASE(2); break;
            default: ELM_NARROW_CASE(4); break;
        }
#undef ELM_NARROW_CASE
#undef ELM_NARROW_LAUNCH
        return hipGetLastError();
    }
    if (M <= 4 && L <= 512) {       // register-resident variant, columns per lane sized to L
#define ELM_ROWS_LAUNCH(MM, EE)                                                                        \
    hipLaunchKernelGGL((stream_rows_kernel<MM, MODE, EE>), dim3(grid), dim3(kThreads), 0, stream, H, T, N, L, \
                       m, beta, part, Y)
#define ELM_ROWS_CASE(MM)                                   \
    if (L <= 128) ELM_ROWS_LAUNCH(MM, 2);                   \
    else if (L <= 256) ELM_ROWS_LAUNCH(MM, 4);              \
    else ELM_ROWS_LAUNCH(MM, 8)
        switch (M) {
            case 1: ELM_ROWS_CASE(1); break;
            case 2: ELM_ROWS_CASE(2); break;
            default: ELM_ROWS_CASE(4); break;
        }
#undef ELM_ROWS_CASE
#undef ELM_ROWS_LAUNCH
        return hipGetLastError();
    }
    const size_t lds = stream_lds_bytes(L, M);
#define ELM_STREAM_CASE(MM)                                                                         \
    case MM: {                                                                                      \
        auto kern = stream_kernel<MM, MODE>;                                                        \
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                     \
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);   \
        if (e != hipSuccess) return e;                                                              \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, stream, H, T, N, L, m, beta, part, Y); \
        return hipGetLastError();                                                                   \
    }
    switch (M) {
        ELM_STREAM_CASE(8)
        ELM_STREAM_CASE(16)
        default: return hipErrorInvalidValue;
    }
#undef ELM_STREAM_CASE
}

}  // namespace

hipError_t launch_backsolve(const SolvePlan& pl, const float* R, void* ws, hipStream_t stream) {
    double* small = reinterpret_cast<double*>(static_cast<char*>(ws) + pl.off_small);
    hipLaunchKernelGGL(backsolve_kernel, dim3(1), dim3(kThreads), 0, stream, R, pl.np, pl.L, pl.m, small);
    return hipGetLastError();
}

// Residual statistics of `rows` rows (a chunk of the N rows, or all of them): r = T - H beta, H^T r,
// sum r^2, sum H^2 in float64; accumulate != 0 adds to what earlier chunks left in the workspace.
hipError_t launch_residual_chunk(const SolvePlan& pl, const float* H, const float* T, int64_t rows, void* ws,
                                 int accumulate, hipStream_t stream) {
    char* base = static_cast<char*>(ws);
    double* small = reinterpret_cast<double*>(base + pl.off_small);
    double* part = reinterpret_cast<double*>(base + pl.off_part);
    hipError_t e = launch_stream<0>(H, T, rows, pl.L, pl.m, small + SmallArea::BETA, part, nullptr, stream);
    if (e != hipSuccess) return e;
    const int nout = pl.L * pl.m + 2;
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((nout + 31) / 32), dim3(kThreads), 0, stream, part,
                       stream_grid(rows), pl.L, pl.m, small, accumulate);
    return hipGetLastError();
}

// After the last chunk: the gradient norm.
hipError_t launch_residual_finish(const SolvePlan& pl, void* ws, hipStream_t stream) {
    double* small = reinterpret_cast<double*>(static_cast<char*>(ws) + pl.off_small);
    hipLaunchKernelGGL(grad_norm_kernel, dim3(1), dim3(kThreads), 0, stream, pl.L, pl.m, small);
    return hipGetLastError();
}

hipError_t launch_residual_pass(const SolvePlan& pl, const float* H, const float* T, void* ws,
                                hipStream_t stream) {
    hipError_t e = launch_residual_chunk(pl, H, T, pl.N, ws, 0, stream);
    if (e != hipSuccess) return e;
    return launch_residual_finish(pl, ws, stream);
}

hipError_t launch_refine_update(const SolvePlan& pl, const float* R, void* ws, hipStream_t stream) {
    double* small = reinterpret_cast<double*>(static_cast<char*>(ws) + pl.off_small);
    hipLaunchKernelGGL(refine_kernel, dim3(1), dim3(kThreads), 0, stream, R, pl.np, pl.L, pl.m, small);
    return hipGetLastError();
}

hipError_t launch_export_beta(const SolvePlan& pl, void* ws, float* beta32, double* beta64,
                              hipStream_t stream) {
    const double* small = reinterpret_cast<const double*>(static_cast<char*>(ws) + pl.off_small);
    const int count = pl.L * pl.m;
    hipLaunchKernelGGL(export_beta_kernel, dim3((count + 255) / 256), dim3(256), 0, stream,
                       small + SmallArea::BETA, count, beta32, beta64);
    return hipGetLastError();
}

hipError_t launch_predict_gemv(const float* H, const double* beta64, int64_t N, int L, int m, float* Y,
                               hipStream_t stream) {
    return launch_stream<1>(H, nullptr, N, L, m, beta64, nullptr, Y, stream);
}

}  // namespace elm
