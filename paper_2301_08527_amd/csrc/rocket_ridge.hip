// ROCKET transform library for MI355X (gfx950): ridge regressor on the pooled features
// (paper section 3 part (3), section 3.3).  See include/rocket.h for the contract.
//
// Model: minimise ||y - X w - b||^2 + alpha ||w||^2 with an unpenalised intercept.  With
// n examples and p >> n features the fit works in the n x n dual system
//     a = (Xc Xc^T + alpha I)^-1 yc,   w = Xc^T a,   b = mean(y) - mean(X) . w
// (Xc, yc centred).  Everything is fp64 on fp32 features, and every sum has a fixed order
// (no atomics), so a fit is reproducible bit for bit.  Kernels, in launch order:
//   rr_col_sums, rr_means       column means of X and the mean target (rows split over the grid)
//   rr_gram                     partial 64 x 64 tiles of Xc Xc^T on the fp64 matrix cores
//                               (v_mfma_f64_16x16x4f64), one wavefront per (tile pair, slice of
//                               the p features); operands go from global memory straight into
//                               the MFMA operand registers, centred on the way
//   rr_gram_finish              sums the slices, adds alpha on the diagonal, writes the lower
//                               triangle of the (n+1) x (n+1) system whose last row is yc
//   per 32 columns: rr_panel    Cholesky of the 32 x 32 diagonal block inside one wavefront's
//                               registers, then the rows below it solved against that block
//                   rr_trailing the rank-32 update of what is left, 32 x 32 tiles on the MFMA
//                               units.  The row of yc takes part like any other row, so when
//                               the factorisation ends it holds L^-1 yc (forward substitution
//                               costs nothing extra).
//   rr_back_substitute          L^T a = L^-1 yc, panel by panel, one workgroup
//   rr_coef_partial, rr_coef_finish, rr_intercept     w = Xc^T a and b
//   rr_predict                  yhat = X w + b, one workgroup per row
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <string>

#include "rocket_internal.hpp"

namespace {

typedef double d4 __attribute__((ext_vector_type(4)));
typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));   // rows of X start at any multiple of 4 bytes

constexpr int kGramTile = 64;       // rows of one Gram tile (4 x 4 MFMA tiles per wavefront)
constexpr int kNB = 32;             // panel width of the factorisation
constexpr int kMaxExamples = 32768; // (n+1)^2 doubles of workspace: 8.6 GB at this size
constexpr int kGramWaves = 2048;    // wavefronts the Gram kernel aims for (256 CUs x 4 SIMDs x 2)
constexpr int kMaxRowSplits = 16;

// D = A B + C on one wavefront: lane l supplies A[l % 16][l / 16] and B[l / 16][l % 16] and holds
// D[4 v + l / 16][l % 16] in element v of the result.
__device__ __forceinline__ d4 rr_mfma(double a, double b, d4 c) { return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0); }

__device__ __forceinline__ double rr_lane(double v, int lane)   // v of a given lane, to all lanes (lane: wave-uniform)
{
    const long long bits = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_readlane(static_cast<int>(bits), lane);
    const int hi = __builtin_amdgcn_readlane(static_cast<int>(bits >> 32), lane);
    return __longlong_as_double((static_cast<long long>(hi) << 32) | static_cast<unsigned int>(lo));
}

// part[r][j] = sum of X[i][j] over the rows i of slice r, j < p; column p is the target vector
__global__ __launch_bounds__(256) void rr_col_sums(const float *__restrict__ X, const float *__restrict__ y, int n,
                                                   int p, int rows_per, double *__restrict__ part)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j > p) return;
    const int i0 = blockIdx.y * rows_per, i1 = min(n, i0 + rows_per);
    double s = 0.0;
    if (j < p) {
        for (int i = i0; i < i1; ++i) s += static_cast<double>(X[static_cast<size_t>(i) * p + j]);
    } else {
        for (int i = i0; i < i1; ++i) s += static_cast<double>(y[i]);
    }
    part[static_cast<size_t>(blockIdx.y) * (p + 1) + j] = s;
}

// means[j] = mean_i X[i][j] for j < p; means[p] = mean_i y[i]
__global__ __launch_bounds__(256) void rr_means(const double *__restrict__ part, int splits, int n, int p,
                                                double *__restrict__ means)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j > p) return;
    double s = 0.0;
    for (int r = 0; r < splits; ++r) s += part[static_cast<size_t>(r) * (p + 1) + j];
    means[j] = s / static_cast<double>(n);
}

// One wavefront per (pair of 64-row tiles ti <= tj, slice of the features).  Work items are dealt
// so that one XCD (workgroup ids go round the eight of them) takes all tile pairs of a slice one
// after the other: the slab of X for that slice then stays in that XCD's L2.  The order of the
// features inside a step of 16 is permuted (lane q = l / 16 takes features 4q..4q+3 as one
// 16-byte load); a sum does not care, and both operands use the same permutation.
__global__ __launch_bounds__(64) void rr_gram(const float *__restrict__ X, const double *__restrict__ means, int n,
                                              int p, int tiles, int pairs, int chunk, int splits,
                                              double *__restrict__ part)
{
    const int total = pairs * splits, per = (total + 7) / 8;
    const int w = (blockIdx.x % 8) * per + blockIdx.x / 8;
    if (blockIdx.x / 8 >= per || w >= total) return;
    const int split = w / pairs, pair = w % pairs;
    int ti = 0, rem = pair;
    while (rem >= tiles - ti) { rem -= tiles - ti; ++ti; }
    const int tj = ti + rem;
    const bool diag = ti == tj;
    const int l = threadIdx.x, r = l & 15, q = l >> 4;
    const int kbeg = split * chunk, kend = min(p, kbeg + chunk);

    const float *pa[4], *pb[4];   // rows past n repeat row n - 1: their results are never stored
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        pa[a] = X + static_cast<size_t>(min(ti * kGramTile + 16 * a + r, n - 1)) * p;
        pb[a] = X + static_cast<size_t>(min(tj * kGramTile + 16 * a + r, n - 1)) * p;
    }
    d4 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = d4{0.0, 0.0, 0.0, 0.0};

    for (int k0 = kbeg; k0 < kend; k0 += 16) {
        const int k = k0 + 4 * q;
        f4u xa[4], xb[4];
        d4 mu;
        if (k0 + 16 <= kend) {
#pragma unroll
            for (int a = 0; a < 4; ++a) xa[a] = *reinterpret_cast<const f4u *>(pa[a] + k);
            if (!diag) {
#pragma unroll
                for (int a = 0; a < 4; ++a) xb[a] = *reinterpret_cast<const f4u *>(pb[a] + k);
            }
            mu = *reinterpret_cast<const d4 *>(means + k);
        } else {   // ragged end of the features: absent ones enter as 0 - 0
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool ok = k + e < kend;
                mu[e] = ok ? means[k + e] : 0.0;
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    xa[a][e] = ok ? pa[a][k + e] : 0.0f;
                    xb[a][e] = ok ? pb[a][k + e] : 0.0f;
                }
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            double am[4], bm[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) am[a] = static_cast<double>(xa[a][e]) - mu[e];
#pragma unroll
            for (int a = 0; a < 4; ++a) bm[a] = diag ? am[a] : static_cast<double>(xb[a][e]) - mu[e];
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[a][b] = rr_mfma(am[a], bm[b], acc[a][b]);
        }
    }
    double *dst = part + (static_cast<size_t>(pair) * splits + split) * (kGramTile * kGramTile);
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) dst[(16 * a + 4 * v + q) * kGramTile + 16 * b + r] = acc[a][b][v];
}

// M (n+1 rows, leading dimension ld): the lower triangle of Xc Xc^T + alpha I in rows 0..n-1,
// yc in row n.  grid.x = tile pairs + 1 (the last one writes row n), grid.y = 16 slabs of a tile.
__global__ __launch_bounds__(256) void rr_gram_finish(const double *__restrict__ part, int tiles, int pairs, int splits,
                                                      int n, int ld, double alpha, const float *__restrict__ y,
                                                      const double *__restrict__ means, int p, double *__restrict__ M)
{
    if (static_cast<int>(blockIdx.x) == pairs) {
        for (int j = blockIdx.y * 256 + threadIdx.x; j < n; j += 16 * 256)
            M[static_cast<size_t>(n) * ld + j] = static_cast<double>(y[j]) - means[p];
        return;
    }
    int ti = 0, rem = blockIdx.x;
    while (rem >= tiles - ti) { rem -= tiles - ti; ++ti; }
    const int tj = ti + rem;
    const int e = blockIdx.y * 256 + threadIdx.x;
    const double *src = part + static_cast<size_t>(blockIdx.x) * splits * (kGramTile * kGramTile) + e;
    double s = 0.0;
    for (int c = 0; c < splits; ++c) s += src[static_cast<size_t>(c) * (kGramTile * kGramTile)];
    const int gi = ti * kGramTile + e / kGramTile, gj = tj * kGramTile + e % kGramTile;
    if (gi < n && gj < n && gj >= gi) M[static_cast<size_t>(gj) * ld + gi] = s + (gi == gj ? alpha : 0.0);
}

// One wavefront per 64 rows below the diagonal block at (k0, k0) of width nb <= 32.  Every
// wavefront factors the block itself (lane r keeps row r in registers, values of other rows come
// through readlane), then solves its rows x L11^T = A21 with one row per lane.  The rows are
// written back in place and, packed 32 to a row, to P for the trailing update.  Workgroup 0
// writes the factored block to D (32 x 32, its own array: the other workgroups are still reading
// the unfactored block in M).  A block narrower than 32 is padded with the identity.
__global__ __launch_bounds__(64) void rr_panel(double *__restrict__ M, int ld, int nrows, int k0, int nb,
                                               double *__restrict__ P, double *__restrict__ D)
{
    const int l = threadIdx.x;
    double row[kNB];
    {
        const int rr = min(l, nb - 1);
        const double *src = M + static_cast<size_t>(k0 + rr) * ld + k0;
#pragma unroll
        for (int c = 0; c < kNB; ++c) {
            double v = (c == l) ? 1.0 : 0.0;
            if (l < nb && c <= l) v = src[c];
            row[c] = v;
        }
    }
#pragma unroll
    for (int k = 0; k < kNB; ++k) {
        const double d = sqrt(rr_lane(row[k], k));
        const double lrk = (l == k) ? d : row[k] / d;    // meaningful in lanes k..31
        row[k] = lrk;
#pragma unroll
        for (int j = k + 1; j < kNB; ++j) row[j] = fma(-lrk, rr_lane(lrk, j), row[j]);   // meaningful where j <= lane
    }
    if (blockIdx.x == 0 && l < kNB) {
        double *dst = D + static_cast<size_t>(k0 / kNB) * (kNB * kNB) + l * kNB;
#pragma unroll
        for (int c = 0; c < kNB; ++c) dst[c] = c <= l ? row[c] : 0.0;
    }
    const int first = k0 + nb;
    const int i = first + blockIdx.x * 64 + l;
    const bool live = i < nrows;
    double x[kNB];
    {
        const double *src = M + static_cast<size_t>(live ? i : nrows - 1) * ld + k0;
#pragma unroll
        for (int c = 0; c < kNB; ++c) x[c] = c < nb ? src[c] : 0.0;
    }
#pragma unroll
    for (int j = 0; j < kNB; ++j) {
#pragma unroll
        for (int m = 0; m < j; ++m) x[j] = fma(-x[m], rr_lane(row[m], j), x[j]);
        x[j] = x[j] / rr_lane(row[j], j);
    }
    if (live) {
        double *dst = M + static_cast<size_t>(i) * ld + k0;
        double *pk = P + static_cast<size_t>(i - first) * kNB;
#pragma unroll
        for (int c = 0; c < kNB; ++c) {
            if (c < nb) dst[c] = x[c];
            pk[c] = x[c];
        }
    }
}

// C -= P P^T on the lower triangle of what lies below and right of the panel: one wavefront per
// 32 x 32 tile (ti >= tj), 2 x 2 MFMA tiles, the 32 columns of P in 8 steps (lane q = l / 16
// takes columns 8q..8q+7 of its row; same permutation on both sides).  rows = rows of P (the row
// of yc included), cols = columns still to be factored (rows - 1: yc has no column).
__global__ __launch_bounds__(64) void rr_trailing(double *__restrict__ M, int ld, int first, int rows, int cols,
                                                  const double *__restrict__ P)
{
    const int ti = blockIdx.y, tj = blockIdx.x;
    if (tj > ti) return;
    const int l = threadIdx.x, r = l & 15, q = l >> 4;
    double av[2][8], bv[2][8];
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        const double *sa = P + static_cast<size_t>(min(ti * 32 + 16 * a + r, rows - 1)) * kNB + 8 * q;
        const double *sb = P + static_cast<size_t>(min(tj * 32 + 16 * a + r, rows - 1)) * kNB + 8 * q;
#pragma unroll
        for (int e = 0; e < 8; ++e) { av[a][e] = sa[e]; bv[a][e] = sb[e]; }
    }
    d4 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = d4{0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int e = 0; e < 8; ++e)
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b) acc[a][b] = rr_mfma(av[a][e], bv[b][e], acc[a][b]);
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int gi = ti * 32 + 16 * a + 4 * v + q, gj = tj * 32 + 16 * b + r;
                if (gi < rows && gj < cols && gj <= gi) M[static_cast<size_t>(first + gi) * ld + first + gj] -= acc[a][b][v];
            }
}

// One workgroup of 32 x 32 threads.  Row n of M holds z = L^-1 yc, D the factored diagonal
// blocks; solves L^T a = z from the last panel to the first: a_panel = L11^-T (z_panel - L21^T a_below).
__global__ __launch_bounds__(1024) void rr_back_substitute(const double *__restrict__ M, int ld, int n,
                                                           const double *__restrict__ D, double *a)
{
    __shared__ double red[32][kNB + 1];
    __shared__ double sl[kNB][kNB + 1];
    const int t = threadIdx.x, c = t & 31, g = t >> 5;
    for (int k0 = (n - 1) / kNB * kNB; k0 >= 0; k0 -= kNB) {
        const int nb = min(kNB, n - k0);
        double s = 0.0;
        if (c < nb)
            for (int i = k0 + nb + g; i < n; i += 32) s = fma(M[static_cast<size_t>(i) * ld + k0 + c], a[i], s);
        red[g][c] = s;
        sl[g][c] = D[static_cast<size_t>(k0 / kNB) * (kNB * kNB) + g * kNB + c];
        __syncthreads();
        if (t < 32) {
            double v = c < nb ? M[static_cast<size_t>(n) * ld + k0 + c] : 0.0;
            for (int gg = 0; gg < 32; ++gg) v -= red[gg][c];
            for (int m = kNB - 1; m >= 0; --m) {
                const double xm = __shfl(v, m, 32) / sl[m][m];
                if (c == m) v = xm;
                else if (c < m) v = fma(-sl[m][c], xm, v);
            }
            if (c < nb) a[k0 + c] = v;
        }
        __syncthreads();
    }
}

// wpart[r][j] = sum over the rows i of slice r of a[i] * (X[i][j] - mean_j)
__global__ __launch_bounds__(256) void rr_coef_partial(const float *__restrict__ X, const double *__restrict__ means,
                                                       const double *__restrict__ a, int n, int p, int rows_per,
                                                       double *__restrict__ wpart)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= p) return;
    const int i0 = blockIdx.y * rows_per, i1 = min(n, i0 + rows_per);
    const double mu = means[j];
    double s = 0.0;
    for (int i = i0; i < i1; ++i) s = fma(a[i], static_cast<double>(X[static_cast<size_t>(i) * p + j]) - mu, s);
    wpart[static_cast<size_t>(blockIdx.y) * p + j] = s;
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

// w[j] = sum_r wpart[r][j]; bpart[block] = sum over the block's j of mean_j * w[j]
__global__ __launch_bounds__(256) void rr_coef_finish(const double *__restrict__ wpart, int splits, int p,
                                                      const double *__restrict__ means, double *__restrict__ w,
                                                      double *__restrict__ bpart)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    double s = 0.0;
    if (j < p) {
        for (int r = 0; r < splits; ++r) s += wpart[static_cast<size_t>(r) * p + j];
        w[j] = s;
        s *= means[j];
    }
    s = rr_block_sum(s);
    if (threadIdx.x == 0) bpart[blockIdx.x] = s;
}

// b = mean(y) - sum_j mean_j * w[j]   (one workgroup over the block sums)
__global__ __launch_bounds__(256) void rr_intercept(const double *__restrict__ means, const double *__restrict__ bpart,
                                                    int blocks, int p, double *__restrict__ b)
{
    double s = 0.0;
    for (int j = threadIdx.x; j < blocks; j += 256) s += bpart[j];
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

namespace {

// Where the pieces of the workspace lie and how the work is cut, for n examples and p features.
struct RidgePlan {
    int ld;            // leading dimension of the (n+1)-row system
    int tiles, pairs;  // 64-row tiles of the Gram matrix and pairs ti <= tj of them
    int chunk, splits; // features per slice (a multiple of 16) and slices
    int row_splits, rows_per;
    size_t off_means, off_M, off_dual, off_P, off_D, off_scratch, bytes;
};

RidgePlan ridge_plan(int n, int p)
{
    RidgePlan q;
    q.ld = (n + 1 + 3) / 4 * 4;
    q.tiles = (n + kGramTile - 1) / kGramTile;
    q.pairs = q.tiles * (q.tiles + 1) / 2;
    const int want = std::max(1, std::min(64, kGramWaves / q.pairs));
    q.chunk = std::max(64, ((p + want - 1) / want + 15) / 16 * 16);
    q.splits = (p + q.chunk - 1) / q.chunk;
    q.row_splits = std::max(1, std::min(kMaxRowSplits, n / 32));
    q.rows_per = (n + q.row_splits - 1) / q.row_splits;
    q.row_splits = (n + q.rows_per - 1) / q.rows_per;
    const size_t coef_blocks = (static_cast<size_t>(p) + 255) / 256;
    const size_t scratch = std::max({static_cast<size_t>(q.row_splits) * (p + 1),
                                     static_cast<size_t>(q.pairs) * q.splits * kGramTile * kGramTile,
                                     static_cast<size_t>(q.row_splits) * p + coef_blocks});
    size_t at = 0;
    q.off_means = at;   at += up256(static_cast<size_t>(p + 1) * 8);
    q.off_M = at;       at += up256(static_cast<size_t>(n + 1) * q.ld * 8);
    q.off_dual = at;    at += up256(static_cast<size_t>(n) * 8);
    q.off_P = at;       at += up256(static_cast<size_t>(n + 1) * kNB * 8);
    q.off_D = at;       at += up256(static_cast<size_t>((n + kNB - 1) / kNB) * kNB * kNB * 8);
    q.off_scratch = at; at += up256(scratch * 8);
    q.bytes = at;
    return q;
}

}  // namespace

extern "C" size_t rocket_ridge_workspace_bytes(int32_t n, int32_t p)
{
    if (n < 1 || p < 1 || n > kMaxExamples) return 0;
    return ridge_plan(n, p).bytes;
}

extern "C" int rocket_ridge_fit(const float *features_dev, const float *targets_dev, int32_t n, int32_t p, double alpha,
                                double *coef_dev, double *intercept_dev, void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!features_dev || !targets_dev || !coef_dev || !intercept_dev)
        return rk_fail(ROCKET_EINVAL, "rocket_ridge_fit: NULL pointer");
    if (n < 1 || p < 1) return rk_fail(ROCKET_EINVAL, "rocket_ridge_fit: n and p must be >= 1");
    if (n > kMaxExamples) return rk_fail(ROCKET_EINVAL, "rocket_ridge_fit: at most 32768 examples (the dual system is stored densely)");
    if (!(alpha > 0.0) || !std::isfinite(alpha)) return rk_fail(ROCKET_EINVAL, "rocket_ridge_fit: alpha must be positive and finite");
    const RidgePlan q = ridge_plan(n, p);
    if (!ws || ws_bytes < q.bytes)
        return rk_fail(ROCKET_EWORKSPACE, "rocket_ridge_fit: workspace of " + std::to_string(q.bytes) + " bytes required");
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return rk_fail(ROCKET_EWORKSPACE, "rocket_ridge_fit: workspace must be 256-byte aligned");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    char *base = static_cast<char *>(ws);
    double *means = reinterpret_cast<double *>(base + q.off_means);
    double *M = reinterpret_cast<double *>(base + q.off_M);
    double *dual = reinterpret_cast<double *>(base + q.off_dual);
    double *P = reinterpret_cast<double *>(base + q.off_P);
    double *D = reinterpret_cast<double *>(base + q.off_D);
    double *scratch = reinterpret_cast<double *>(base + q.off_scratch);

    hipLaunchKernelGGL(rr_col_sums, dim3((p + 1 + 255) / 256, q.row_splits), dim3(256), 0, stream, features_dev,
                       targets_dev, n, p, q.rows_per, scratch);
    hipLaunchKernelGGL(rr_means, dim3((p + 1 + 255) / 256), dim3(256), 0, stream, scratch, q.row_splits, n, p, means);
    const int items = q.pairs * q.splits;
    hipLaunchKernelGGL(rr_gram, dim3((items + 7) / 8 * 8), dim3(64), 0, stream, features_dev, means, n, p, q.tiles,
                       q.pairs, q.chunk, q.splits, scratch);
    hipLaunchKernelGGL(rr_gram_finish, dim3(q.pairs + 1, 16), dim3(256), 0, stream, scratch, q.tiles, q.pairs, q.splits,
                       n, q.ld, alpha, targets_dev, means, p, M);
    const int nrows = n + 1;
    for (int k0 = 0; k0 < n; k0 += kNB) {
        const int nb = std::min(kNB, n - k0);
        const int first = k0 + nb, rows = nrows - first;   // rows >= 1: the row of yc is always below
        hipLaunchKernelGGL(rr_panel, dim3((rows + 63) / 64), dim3(64), 0, stream, M, q.ld, nrows, k0, nb, P, D);
        if (rows > 1) {
            const int t = (rows + 31) / 32;
            hipLaunchKernelGGL(rr_trailing, dim3(t, t), dim3(64), 0, stream, M, q.ld, first, rows, rows - 1, P);
        }
    }
    hipLaunchKernelGGL(rr_back_substitute, dim3(1), dim3(1024), 0, stream, M, q.ld, n, D, dual);
    const int coef_blocks = (p + 255) / 256;
    double *wpart = scratch, *bpart = scratch + static_cast<size_t>(q.row_splits) * p;
    hipLaunchKernelGGL(rr_coef_partial, dim3(coef_blocks, q.row_splits), dim3(256), 0, stream, features_dev, means, dual,
                       n, p, q.rows_per, wpart);
    hipLaunchKernelGGL(rr_coef_finish, dim3(coef_blocks), dim3(256), 0, stream, wpart, q.row_splits, p, means, coef_dev,
                       bpart);
    hipLaunchKernelGGL(rr_intercept, dim3(1), dim3(256), 0, stream, means, bpart, coef_blocks, p, intercept_dev);
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
