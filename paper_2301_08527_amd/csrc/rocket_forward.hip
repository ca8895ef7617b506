// ROCKET transform for MI355X (gfx950): forward kernels (zero-padding copy, conv + pooling for
// series longer than 8,192 samples, combination of the partial results) and their launchers.
// See include/rocket.h for the contract of the entry points.
//
// Work decomposition of the forward pass (paper section 3, parts (1)-(2)):
//   The n outputs of a kernel with dilation d are viewed as a grid of rows of d consecutive
//   positions: t = m*d + r.  A kernel's rows are cut into jobs (time tiles of at least 16,384
//   positions); one workgroup (256 lanes) owns one (series, job) pair and writes the job's
//   partial max / positive count / sigmoid sum, which rk_finalize combines per kernel in a fixed
//   order.  Jobs are sorted by the window of the series they read, so that workgroups running
//   together share one stretch of one series in L2.
//   A lane owns a vertical strip of R rows in one column r, i.e. outputs t0, t0+d, ...,
//   t0+(R-1)d.  Those R outputs read the R+len-1 inputs x[t0-p+i*d]; each input is loaded once
//   and feeds up to len fused multiply-adds from registers.  Neighbouring lanes own neighbouring
//   columns, so every load instruction of a wavefront reads consecutive floats.  Three paths,
//   uniform per workgroup: bands of 32, 16, 8, 4, 2 and 1 rows plus the partial last row, so every
//   strip is fully valid and the pooling needs no masks (register path); tiles staged through
//   LDS for dilations below 16; one strip over all rows for large dilations with few rows.
//   Weights are wavefront-uniform (scalar registers); max / PPV count / softPPV sum stay in
//   registers and are closed with wavefront shuffles.
//   The batch is first copied into a zero-padded workspace so that no dilated read leaves the
//   zeros around its row and "same" padding needs no bounds checks.
#include "rocket_forward_impl.hpp"

// Copies nrows rows of L floats into rows of row_len floats: `lead` zeros, the samples, zeros
// to the end; row number nrows (one past the last) is written as zeros only.  One thread
// writes four consecutive floats.
__global__ __launch_bounds__(256) void rk_pad_rows(const float *__restrict__ x, float *__restrict__ xpad,
                                                   int L, int lead, int row_len, int nrows)
{
    const int col = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (col >= row_len) return;
    for (int row = blockIdx.y; row <= nrows; row += gridDim.y) {
        const float *src = x + static_cast<size_t>(row) * L;
        const int len = row < nrows ? L : 0;
        float4 v;
        const int s = col - lead;
        v.x = (s >= 0 && s < len) ? src[s] : 0.f;
        v.y = (s + 1 >= 0 && s + 1 < len) ? src[s + 1] : 0.f;
        v.z = (s + 2 >= 0 && s + 2 < len) ? src[s + 2] : 0.f;
        v.w = (s + 3 >= 0 && s + 3 < len) ? src[s + 3] : 0.f;
        *reinterpret_cast<float4 *>(xpad + static_cast<size_t>(row) * row_len + col) = v;
    }
}

// ------------------------------------------------------------------ launchers

int rk_launch_pad(const rocket_kernels *h, const float *x, int32_t B, float *xpad, void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    const int nrows = B * h->C;
    dim3 grid(static_cast<unsigned>((h->row_len / 4 + 255) / 256), static_cast<unsigned>(nrows < 32768 ? nrows + 1 : 32768));
    hipLaunchKernelGGL(rk_pad_rows, grid, dim3(256), 0, stream, x, xpad, h->L, h->lead,
                       static_cast<int>(h->row_len), nrows);
    return hipGetLastError() == hipSuccess ? ROCKET_OK : ROCKET_EHIP;
}

int rk_launch_forward(const rocket_kernels *h, const float *xpad, int32_t B, uint32_t mask, float nl, float ns,
                      float *partials, void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    const int J = static_cast<int>(h->jobs.size());
    const int spread = rk_spread(h, B);
    hipLaunchKernelGGL(rk_forward<kThreads>, dim3(static_cast<unsigned>(rk_grid_groups(B, J, spread))), dim3(kThreads), 0, stream, xpad,
                       static_cast<int>(h->row_len), h->lead, h->L, h->C, J, h->d_rec, h->d_jobs, h->d_channels,
                       h->d_weights, mask, nl, ns, partials, B, spread);
    return hipGetLastError() == hipSuccess ? ROCKET_OK : ROCKET_EHIP;
}

// One thread per (series, kernel): combines the kernel's job partials in job order and
// writes the feature planes out[b*F*K + f*K + k] (max + bias, count / n, sum / n).
__global__ __launch_bounds__(256) void rk_finalize(const float *__restrict__ partials, int B, int K, int J,
                                                   const RkKernelRec *__restrict__ recs,
                                                   const int32_t *__restrict__ kjob_off,
                                                   const int32_t *__restrict__ kjob_idx, uint32_t mask,
                                                   float *__restrict__ out)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= B * K) return;
    const int b = i / K, kid = i - b * K;
    const size_t plane = static_cast<size_t>(B) * J;
    const size_t base = static_cast<size_t>(b) * J;
    float m = -INFINITY, sm = 0.f;
    int cn = 0;
    for (int q = kjob_off[kid]; q < kjob_off[kid + 1]; ++q) {
        const size_t slot = base + kjob_idx[q];
        m = fmaxf(m, partials[slot]);
        cn += reinterpret_cast<const int *>(partials)[plane + slot];
        sm += partials[2 * plane + slot];
    }
    const RkKernelRec rec = recs[kid];
    const int F = __builtin_popcount(mask);
    float *o = out + static_cast<size_t>(b) * F * K + kid;
    int f = 0;
    if (mask & ROCKET_F_MAX) { o[static_cast<size_t>(f) * K] = m + rec.bias; ++f; }
    if (mask & ROCKET_F_PPV) { o[static_cast<size_t>(f) * K] = static_cast<float>(static_cast<double>(cn) / static_cast<double>(rec.nout)); ++f; }
    if (mask & ROCKET_F_SOFTPPV) { o[static_cast<size_t>(f) * K] = sm / static_cast<float>(rec.nout); ++f; }
}

int rk_launch_finalize(const rocket_kernels *h, const float *partials, int32_t B, uint32_t mask, float *out,
                       void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    const int total = B * h->K;
    hipLaunchKernelGGL(rk_finalize, dim3((total + 255) / 256), dim3(256), 0, stream, partials, B, h->K,
                       static_cast<int>(h->jobs.size()), h->d_rec, h->d_kjob_off, h->d_kjob_idx, mask, out);
    return hipGetLastError() == hipSuccess ? ROCKET_OK : ROCKET_EHIP;
}
