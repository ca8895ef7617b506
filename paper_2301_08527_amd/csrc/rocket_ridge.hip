// ROCKET transform library for MI355X (gfx950): ridge regressor on the pooled features
// (paper section 3 part (3), section 3.3).  See include/rocket.h for the contract.
//
// Model: minimise ||y - X w - b||^2 + alpha ||w||^2 with an unpenalised intercept.  With
// n examples and p >> n features the fit works in the n x n dual system
//     a = (Xc Xc^T + alpha I)^-1 yc,   w = Xc^T a,   b = mean(y) - mean(X) . w
// (Xc, yc centred).  Everything is fp64 on fp32 features.  Kernels, in launch order:
//   rr_col_means     column means of X and the mean target
//   rr_gram          G = Xc Xc^T + alpha I, 32x32 output tiles, operands staged through
//                    LDS in fp64 with the mean subtracted on the way in
//   rr_cholesky_solve  one workgroup: in-place Cholesky of G and the two triangular solves
//   rr_coefficients  w = Xc^T a
//   rr_intercept     b = mean(y) - mean(X) . w
//   rr_predict       yhat = X w + b, one workgroup per row
#include <hip/hip_runtime.h>

#include <cmath>
#include <string>

#include "rocket_internal.hpp"

namespace {

constexpr int kTile = 32;        // Gram output tile and depth of one staged slab
constexpr int kSolveThreads = 1024;
constexpr int kMaxExamples = 4096;   // the dual system is factored by one workgroup with a column in LDS

// means[j] = mean_i X[i][j] for j < p; means[p] = mean_i y[i]
__global__ __launch_bounds__(256) void rr_col_means(const float *__restrict__ X, const float *__restrict__ y, int n,
                                                    int p, double *__restrict__ means)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j > p) return;
    double s = 0.0;
    if (j < p) {
        for (int i = 0; i < n; ++i) s += static_cast<double>(X[static_cast<size_t>(i) * p + j]);
    } else {
        for (int i = 0; i < n; ++i) s += static_cast<double>(y[i]);
    }
    means[j] = s / static_cast<double>(n);
}

// One workgroup (16 x 16 threads, 2 x 2 outputs each) per 32 x 32 tile of the upper
// triangle of G; the mirror tile is written as well.
__global__ __launch_bounds__(256) void rr_gram(const float *__restrict__ X, const double *__restrict__ means, int n,
                                               int p, double alpha, double *__restrict__ G)
{
    const int ti = blockIdx.y, tj = blockIdx.x;
    if (tj < ti) return;
    __shared__ double sa[kTile][kTile + 1];   // rows ti*32.., slab of 32 features
    __shared__ double sb[kTile][kTile + 1];   // rows tj*32..
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    double acc[2][2] = {{0.0, 0.0}, {0.0, 0.0}};
    for (int j0 = 0; j0 < p; j0 += kTile) {
        // stage: thread t loads elements (row = t / 32 + 8*q, col = t % 32) of both slabs
        for (int q = 0; q < 4; ++q) {
            const int rr = (threadIdx.x >> 5) + 8 * q, cc = threadIdx.x & 31;
            const int j = j0 + cc;
            const int ra = ti * kTile + rr, rb = tj * kTile + rr;
            const double mu = j < p ? means[j] : 0.0;
            sa[rr][cc] = (ra < n && j < p) ? static_cast<double>(X[static_cast<size_t>(ra) * p + j]) - mu : 0.0;
            sb[rr][cc] = (rb < n && j < p) ? static_cast<double>(X[static_cast<size_t>(rb) * p + j]) - mu : 0.0;
        }
        __syncthreads();
#pragma unroll 8
        for (int c = 0; c < kTile; ++c) {
            const double a0 = sa[ty][c], a1 = sa[ty + 16][c];
            const double b0 = sb[tx][c], b1 = sb[tx + 16][c];
            acc[0][0] = fma(a0, b0, acc[0][0]);
            acc[0][1] = fma(a0, b1, acc[0][1]);
            acc[1][0] = fma(a1, b0, acc[1][0]);
            acc[1][1] = fma(a1, b1, acc[1][1]);
        }
        __syncthreads();
    }
    for (int u = 0; u < 2; ++u)
        for (int v = 0; v < 2; ++v) {
            const int i = ti * kTile + ty + 16 * u, j = tj * kTile + tx + 16 * v;
            if (i < n && j < n) {
                const double g = acc[u][v] + (i == j ? alpha : 0.0);
                G[static_cast<size_t>(i) * n + j] = g;
                G[static_cast<size_t>(j) * n + i] = g;
            }
        }
}

// Single workgroup of 32 x 32 threads.  G (n x n, symmetric positive definite, n <=
// kMaxExamples) is overwritten by its lower Cholesky factor (right-looking, the current
// column is kept in LDS); rhs[i] = y[i] - mean(y) is overwritten by the dual coefficients.
__global__ __launch_bounds__(kSolveThreads) void rr_cholesky_solve(double *__restrict__ G, int n,
                                                                  const float *__restrict__ y,
                                                                  const double *__restrict__ means, int p,
                                                                  double *__restrict__ rhs)
{
    const int t = threadIdx.x, tx = t & 31, ty = t >> 5;
    __shared__ double s_col[kMaxExamples];
    __shared__ double s_diag;
    for (int i = t; i < n; i += kSolveThreads) rhs[i] = static_cast<double>(y[i]) - means[p];
    __syncthreads();
    for (int k = 0; k < n; ++k) {
        if (t == 0) {
            s_diag = sqrt(G[static_cast<size_t>(k) * n + k]);
            G[static_cast<size_t>(k) * n + k] = s_diag;
        }
        __syncthreads();
        const double inv = 1.0 / s_diag;
        for (int i = k + 1 + t; i < n; i += kSolveThreads) {
            const double l = G[static_cast<size_t>(i) * n + k] * inv;
            G[static_cast<size_t>(i) * n + k] = l;
            s_col[i] = l;
        }
        __syncthreads();
        // trailing update of the lower triangle: G[i][j] -= L[i][k] * L[j][k], k < j <= i < n
        for (int i = k + 1 + ty; i < n; i += 32) {
            const double lik = s_col[i];
            for (int j = k + 1 + tx; j <= i; j += 32) G[static_cast<size_t>(i) * n + j] -= lik * s_col[j];
        }
        __syncthreads();
    }
    // forward substitution L z = rhs (column oriented), then back substitution L^T a = z
    for (int k = 0; k < n; ++k) {
        if (t == 0) rhs[k] /= G[static_cast<size_t>(k) * n + k];
        __syncthreads();
        const double zk = rhs[k];
        for (int i = k + 1 + t; i < n; i += kSolveThreads) rhs[i] -= G[static_cast<size_t>(i) * n + k] * zk;
        __syncthreads();
    }
    for (int k = n - 1; k >= 0; --k) {
        if (t == 0) rhs[k] /= G[static_cast<size_t>(k) * n + k];
        __syncthreads();
        const double ak = rhs[k];
        for (int i = t; i < k; i += kSolveThreads) rhs[i] -= G[static_cast<size_t>(k) * n + i] * ak;
        __syncthreads();
    }
}

// w[j] = sum_i a[i] * (X[i][j] - mean_j)
__global__ __launch_bounds__(256) void rr_coefficients(const float *__restrict__ X, const double *__restrict__ means,
                                                       const double *__restrict__ a, int n, int p,
                                                       double *__restrict__ w)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= p) return;
    const double mu = means[j];
    double s = 0.0;
    for (int i = 0; i < n; ++i) s = fma(a[i], static_cast<double>(X[static_cast<size_t>(i) * p + j]) - mu, s);
    w[j] = s;
}

__device__ __forceinline__ double rr_block_sum(double v)
{
    __shared__ double part[256 / 64];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
    __syncthreads();
    double s = 0.0;
    for (int w = 0; w < 256 / 64; ++w) s += part[w];
    __syncthreads();
    return s;
}

// b = mean(y) - sum_j mean_j * w[j]   (one workgroup)
__global__ __launch_bounds__(256) void rr_intercept(const double *__restrict__ means, const double *__restrict__ w, int p,
                                                    double *__restrict__ b)
{
    double s = 0.0;
    for (int j = threadIdx.x; j < p; j += 256) s = fma(means[j], w[j], s);
    s = rr_block_sum(s);
    if (threadIdx.x == 0) b[0] = means[p] - s;
}

// pred[i] = b + sum_j X[i][j] * w[j]   (one workgroup per row)
__global__ __launch_bounds__(256) void rr_predict(const float *__restrict__ X, int p, const double *__restrict__ w,
                                                  const double *__restrict__ b, double *__restrict__ pred)
{
    const float *row = X + static_cast<size_t>(blockIdx.x) * p;
    double s = 0.0;
    for (int j = threadIdx.x; j < p; j += 256) s = fma(static_cast<double>(row[j]), w[j], s);
    s = rr_block_sum(s);
    if (threadIdx.x == 0) pred[blockIdx.x] = s + b[0];
}

inline size_t up256(size_t v) { return (v + 255) / 256 * 256; }

}  // namespace

#define RR_HIP(call)                                                                   \
    do {                                                                               \
        hipError_t e_ = (call);                                                        \
        if (e_ != hipSuccess)                                                          \
            return rk_fail(ROCKET_EHIP, std::string(#call) + ": " + hipGetErrorString(e_)); \
    } while (0)

extern "C" size_t rocket_ridge_workspace_bytes(int32_t n, int32_t p)
{
    if (n < 1 || p < 1) return 0;
    // means (p+1), Gram (n*n), dual coefficients (n)
    return up256(static_cast<size_t>(p + 1) * 8) + up256(static_cast<size_t>(n) * n * 8) + up256(static_cast<size_t>(n) * 8);
}

extern "C" int rocket_ridge_fit(const float *features_dev, const float *targets_dev, int32_t n, int32_t p, double alpha,
                                double *coef_dev, double *intercept_dev, void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!features_dev || !targets_dev || !coef_dev || !intercept_dev)
        return rk_fail(ROCKET_EINVAL, "rocket_ridge_fit: NULL pointer");
    if (n < 1 || p < 1) return rk_fail(ROCKET_EINVAL, "rocket_ridge_fit: n and p must be >= 1");
    if (n > kMaxExamples) return rk_fail(ROCKET_EINVAL, "rocket_ridge_fit: at most 4096 examples (the dual system is solved by one workgroup)");
    if (!(alpha > 0.0) || !std::isfinite(alpha)) return rk_fail(ROCKET_EINVAL, "rocket_ridge_fit: alpha must be positive and finite");
    const size_t need = rocket_ridge_workspace_bytes(n, p);
    if (!ws || ws_bytes < need)
        return rk_fail(ROCKET_EWORKSPACE, "rocket_ridge_fit: workspace of " + std::to_string(need) + " bytes required");
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return rk_fail(ROCKET_EWORKSPACE, "rocket_ridge_fit: workspace must be 256-byte aligned");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    char *base = static_cast<char *>(ws);
    double *means = reinterpret_cast<double *>(base);
    double *G = reinterpret_cast<double *>(base + up256(static_cast<size_t>(p + 1) * 8));
    double *dual = reinterpret_cast<double *>(reinterpret_cast<char *>(G) + up256(static_cast<size_t>(n) * n * 8));

    hipLaunchKernelGGL(rr_col_means, dim3((p + 1 + 255) / 256), dim3(256), 0, stream, features_dev, targets_dev, n, p, means);
    const int tiles = (n + kTile - 1) / kTile;
    hipLaunchKernelGGL(rr_gram, dim3(tiles, tiles), dim3(256), 0, stream, features_dev, means, n, p, alpha, G);
    hipLaunchKernelGGL(rr_cholesky_solve, dim3(1), dim3(kSolveThreads), 0, stream, G, n, targets_dev, means, p, dual);
    hipLaunchKernelGGL(rr_coefficients, dim3((p + 255) / 256), dim3(256), 0, stream, features_dev, means, dual, n, p, coef_dev);
    hipLaunchKernelGGL(rr_intercept, dim3(1), dim3(256), 0, stream, means, coef_dev, p, intercept_dev);
    RR_HIP(hipGetLastError());
    return ROCKET_OK;
}

extern "C" int rocket_ridge_predict(const float *features_dev, int32_t m, int32_t p, const double *coef_dev,
                                    const double *intercept_dev, double *pred_dev, void *hip_stream)
{
    if (!features_dev || !coef_dev || !intercept_dev || !pred_dev)
        return rk_fail(ROCKET_EINVAL, "rocket_ridge_predict: NULL pointer");
    if (m < 1 || p < 1) return rk_fail(ROCKET_EINVAL, "rocket_ridge_predict: m and p must be >= 1");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipLaunchKernelGGL(rr_predict, dim3(m), dim3(256), 0, stream, features_dev, p, coef_dev, intercept_dev, pred_dev);
    RR_HIP(hipGetLastError());
    return ROCKET_OK;
}
