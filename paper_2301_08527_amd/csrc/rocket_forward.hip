// ROCKET transform for MI355X (gfx950): forward kernels (zero-padding copy, conv +
// pooling) and their launchers.  See include/rocket.h for the contract of the entry points.
//
// Work decomposition of the forward pass (paper section 3, parts (1)-(2)):
//   one workgroup (256 lanes) owns one (series b, kernel k) pair and produces
//   its pooled features, so no cross-workgroup combine is needed.
//   The n outputs of a kernel with dilation d are viewed as a grid of rows of d
//   consecutive positions: t = m*d + r.  A lane owns a vertical strip of R rows
//   in one column r, i.e. outputs t0, t0+d, ..., t0+(R-1)d.  Those R outputs
//   read the R+len-1 inputs x[t0-p+i*d]; each input is loaded once and feeds up
//   to len fused multiply-adds from registers.  Neighbouring lanes own
//   neighbouring columns, so every load instruction of a wavefront reads
//   consecutive floats.  The row range is cut into bands of 16, 8, 4, 2 and 1
//   rows (binary decomposition of the row count) plus the partial last row, so
//   every strip is fully valid and the pooling needs no masks.
//   Weights are wavefront-uniform (scalar registers); max / PPV count / softPPV
//   sum stay in registers and are closed with wavefront shuffles.
//   The batch is first copied into a zero-padded workspace so that no dilated
//   read leaves its row and "same" padding needs no bounds checks.
#include "rocket_forward_impl.hpp"

// Copies B*C rows of L floats into rows of row_len floats: `lead` zeros, the
// samples, zeros to the end.  One thread writes four consecutive floats.
__global__ __launch_bounds__(256) void rk_pad_rows(const float *__restrict__ x, float *__restrict__ xpad,
                                                   int L, int lead, int row_len, int nrows)
{
    const int col = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (col >= row_len) return;
    for (int row = blockIdx.y; row < nrows; row += gridDim.y) {
        const float *src = x + static_cast<size_t>(row) * L;
        float4 v;
        const int s = col - lead;
        v.x = (s >= 0 && s < L) ? src[s] : 0.f;
        v.y = (s + 1 >= 0 && s + 1 < L) ? src[s + 1] : 0.f;
        v.z = (s + 2 >= 0 && s + 2 < L) ? src[s + 2] : 0.f;
        v.w = (s + 3 >= 0 && s + 3 < L) ? src[s + 3] : 0.f;
        *reinterpret_cast<float4 *>(xpad + static_cast<size_t>(row) * row_len + col) = v;
    }
}

// ------------------------------------------------------------------ launchers

int rk_launch_pad(const rocket_kernels *h, const float *x, int32_t B, float *xpad, void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    const int nrows = B * h->C;
    dim3 grid(static_cast<unsigned>((h->row_len / 4 + 255) / 256), static_cast<unsigned>(nrows < 32768 ? nrows : 32768));
    hipLaunchKernelGGL(rk_pad_rows, grid, dim3(256), 0, stream, x, xpad, h->L, h->lead,
                       static_cast<int>(h->row_len), nrows);
    return hipGetLastError() == hipSuccess ? ROCKET_OK : ROCKET_EHIP;
}

int rk_launch_forward(const rocket_kernels *h, const float *xpad, int32_t B, uint32_t mask, float nl, float ns,
                      float *out, void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    hipLaunchKernelGGL(rk_forward<kThreads>, dim3(static_cast<unsigned>(B) * h->K), dim3(kThreads), 0, stream, xpad,
                       static_cast<int>(h->row_len), h->lead, h->L, h->C, h->K, h->d_rec, h->d_order, h->d_channels,
                       h->d_weights, mask, nl, ns, out);
    return hipGetLastError() == hipSuccess ? ROCKET_OK : ROCKET_EHIP;
}
