// ROCKET transform for MI355X (gfx950): fused input prologue for raw 8-bit samples.
//
// The paper's examples are integer light intensities, 20 sensor channels per example, and
// every channel is z-normalised before the transform (sections 4.1 and 4.3).  Instead of
// materialising a normalised fp32 copy of the batch, the zero-padding copy that the transform
// makes anyway reads the bytes and writes (x - mean) / std: the batch is read as 1 byte per
// sample instead of 4, and no extra pass over it is needed beyond the row statistics.
//
//   rk_row_stats_u8 : one workgroup per (series, channel) row; exact 64-bit integer sums of
//                     x and x^2, then mean and population standard deviation in fp64
//   rk_pad_rows_u8  : the padding copy with the normalisation folded in; fp64 subtract and
//                     divide, rounded once to fp32.  A row with zero variance becomes zeros.
#include <hip/hip_runtime.h>

#include "rocket_internal.hpp"

namespace {

__device__ __forceinline__ unsigned long long rk_wave_sum_u64(unsigned long long v)
{
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

}  // namespace

__global__ __launch_bounds__(256) void rk_row_stats_u8(const uint8_t *__restrict__ x, int L, int nrows,
                                                       double2 *__restrict__ stats)
{
    __shared__ unsigned long long part[2][4];
    for (int row = blockIdx.x; row < nrows; row += gridDim.x) {
        const uint8_t *src = x + static_cast<size_t>(row) * L;
        unsigned long long s = 0, s2 = 0;
        for (int i = threadIdx.x; i < L; i += 256) {
            const unsigned v = src[i];
            s += v;
            s2 += v * v;
        }
        s = rk_wave_sum_u64(s);
        s2 = rk_wave_sum_u64(s2);
        const int wave = threadIdx.x >> 6;
        if ((threadIdx.x & 63) == 0) {
            part[0][wave] = s;
            part[1][wave] = s2;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            const unsigned long long ts = part[0][0] + part[0][1] + part[0][2] + part[0][3];
            const unsigned long long ts2 = part[1][0] + part[1][1] + part[1][2] + part[1][3];
            const double mean = static_cast<double>(ts) / L;
            const double var = (static_cast<double>(ts2) - static_cast<double>(ts) * mean) / L;
            // ts2 == ts*mean exactly when all samples are equal; guard tiny negative rounding too
            stats[row] = make_double2(mean, var > 0.0 ? sqrt(var) : 0.0);
        }
        __syncthreads();
    }
}

// Rows of row_len floats: `lead` zeros, the L normalised samples, zeros to the end; row number
// nrows (one past the last) is written as zeros only.
__global__ __launch_bounds__(256) void rk_pad_rows_u8(const uint8_t *__restrict__ x,
                                                      const double2 *__restrict__ stats,
                                                      float *__restrict__ xpad, int L, int lead, int row_len,
                                                      int nrows)
{
    const int col = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (col >= row_len) return;
    for (int row = blockIdx.y; row <= nrows; row += gridDim.y) {
        const uint8_t *src = x + static_cast<size_t>(row) * L;
        const double2 ms = row < nrows ? stats[row] : make_double2(0.0, 0.0);
        const bool live = ms.y > 0.0;
        const double sd = live ? ms.y : 1.0;
        float v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int s = col + q - lead;
            float z = 0.f;
            if (live && s >= 0 && s < L) z = static_cast<float>((static_cast<double>(src[s]) - ms.x) / sd);
            v[q] = z;
        }
        *reinterpret_cast<float4 *>(xpad + static_cast<size_t>(row) * row_len + col) = make_float4(v[0], v[1], v[2], v[3]);
    }
}

int rk_launch_pad_u8(const rocket_kernels *h, const uint8_t *x, int32_t B, float *xpad, void *stats_ptr,
                     void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    double2 *stats = static_cast<double2 *>(stats_ptr);
    const int nrows = B * h->C;
    hipLaunchKernelGGL(rk_row_stats_u8, dim3(static_cast<unsigned>(nrows < 65536 ? nrows : 65536)), dim3(256), 0,
                       stream, x, h->L, nrows, stats);
    if (hipGetLastError() != hipSuccess) return ROCKET_EHIP;
    dim3 grid(static_cast<unsigned>((h->row_len / 4 + 255) / 256), static_cast<unsigned>(nrows < 32768 ? nrows + 1 : 32768));
    hipLaunchKernelGGL(rk_pad_rows_u8, grid, dim3(256), 0, stream, x, stats, xpad, h->L, h->lead,
                       static_cast<int>(h->row_len), nrows);
    return hipGetLastError() == hipSuccess ? ROCKET_OK : ROCKET_EHIP;
}
