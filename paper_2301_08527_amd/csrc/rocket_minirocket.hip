// ROCKET transform for MI355X (gfx950): fitting the biases of MINIROCKET-style kernels to data.
//
// The paper's related-work section says of MINIROCKET that its biases are sampled from the input data.  Here
// kernel k's bias is minus an order statistic of its own bias-free output on one training example (which
// example and which rank are drawn on the host, sampler.cpp).  Two kernels per chunk of kernels:
//   rk_mr_outputs : the bias-free conv output of every kernel of the chunk on its example, to a buffer
//   rk_mr_select  : one workgroup per kernel finds the value of the drawn rank by a radix selection over
//                   the order-preserving integer image of the floats (four passes of 8 bits, LDS histograms;
//                   exact: it returns an element of the row, whatever the ties) and writes its negative into
//                   the kernel's device record.
// The features themselves come from rocket_transform's PPV plane (the two weight values -1 and 2 are exact in
// fp32, so its multiply-adds give what additions would) or from the group kernel in
// rocket_minirocket_forward.hip, which shares the tap sums between the 84 kernels of a group.
#include <hip/hip_runtime.h>

#include "rocket_internal.hpp"

namespace {

constexpr int kTile = 4096;     // outputs per workgroup of rk_mr_outputs

__global__ __launch_bounds__(256) void rk_mr_outputs(const float *__restrict__ xpad, int row_len, int lead, int C,
                                                     const RkKernelRec *__restrict__ recs,
                                                     const int32_t *__restrict__ channels,
                                                     const float *__restrict__ weights,
                                                     const int32_t *__restrict__ example, int k0, long long stride,
                                                     float *__restrict__ ybuf)
{
    const int kid = k0 + static_cast<int>(blockIdx.x);
    const RkKernelRec rec = recs[kid];
    const int t_begin = static_cast<int>(blockIdx.y) * kTile;
    if (t_begin >= rec.nout) return;
    const int t_end = min(rec.nout, t_begin + kTile);
    const float *series = xpad + static_cast<size_t>(example[kid]) * C * row_len + (lead - rec.pad);
    float *y = ybuf + static_cast<size_t>(blockIdx.x) * stride;
    for (int t = t_begin + static_cast<int>(threadIdx.x); t < t_end; t += 256) {
        float acc = 0.f;
        for (int c = 0; c < rec.nch; ++c) {
            const float *row = series + static_cast<size_t>(channels[rec.ch_off + c]) * row_len + t;
            const float *w = weights + rec.w_off + c * rec.len;
            for (int j = 0; j < rec.len; ++j) acc = fmaf(w[j], row[static_cast<size_t>(j) * rec.dil], acc);
        }
        y[t] = acc;
    }
}

// float bits -> unsigned key with the same order as the floats
__device__ __forceinline__ unsigned rk_ordered_key(float v)
{
    const unsigned b = __builtin_bit_cast(unsigned, v);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ float rk_key_value(unsigned key)
{
    const unsigned b = (key & 0x80000000u) ? (key & 0x7fffffffu) : ~key;
    return __builtin_bit_cast(float, b);
}

__global__ __launch_bounds__(256) void rk_mr_select(const float *__restrict__ ybuf, long long stride,
                                                    RkKernelRec *__restrict__ recs,
                                                    const int32_t *__restrict__ rank, int k0)
{
    __shared__ int hist[256];
    __shared__ unsigned s_prefix;
    __shared__ int s_rank;
    const int kid = k0 + static_cast<int>(blockIdx.x);
    const int n = recs[kid].nout;
    const float *y = ybuf + static_cast<size_t>(blockIdx.x) * stride;
    const int tid = static_cast<int>(threadIdx.x);
    if (tid == 0) { s_prefix = 0u; s_rank = rank[kid]; }
    unsigned mask = 0u;
    for (int shift = 24; shift >= 0; shift -= 8) {
        hist[tid] = 0;
        __syncthreads();
        const unsigned prefix = s_prefix;
        for (int t = tid; t < n; t += 256) {
            const unsigned key = rk_ordered_key(y[t]);
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
        }
        __syncthreads();
        if (tid == 0) {
            // the bin that holds the wanted rank among the values that match the prefix so far
            int left = s_rank, bin = 0;
            while (bin < 255 && left >= hist[bin]) { left -= hist[bin]; ++bin; }
            s_rank = left;
            s_prefix = prefix | (static_cast<unsigned>(bin) << shift);
        }
        mask |= 255u << shift;
        __syncthreads();
    }
    if (tid == 0) recs[kid].bias = -rk_key_value(s_prefix);
}

}  // namespace

int rk_launch_minirocket_outputs(const rocket_kernels *h, const float *xpad, const int32_t *example_dev, int32_t k0,
                                 int32_t count, int64_t stride, float *ybuf, void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    const dim3 grid(static_cast<unsigned>(count), static_cast<unsigned>((h->L + kTile - 1) / kTile));
    hipLaunchKernelGGL(rk_mr_outputs, grid, dim3(256), 0, stream, xpad, static_cast<int>(h->row_len), h->lead, h->C,
                       h->d_rec, h->d_channels, h->d_weights, example_dev, k0, static_cast<long long>(stride), ybuf);
    return hipGetLastError() == hipSuccess ? ROCKET_OK : ROCKET_EHIP;
}

int rk_launch_minirocket_select(const rocket_kernels *h, const int32_t *rank_dev, int32_t k0, int32_t count,
                                int64_t stride, const float *ybuf, void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    hipLaunchKernelGGL(rk_mr_select, dim3(static_cast<unsigned>(count)), dim3(256), 0, stream, ybuf,
                       static_cast<long long>(stride), const_cast<RkKernelRec *>(h->d_rec), rank_dev, k0);
    return hipGetLastError() == hipSuccess ? ROCKET_OK : ROCKET_EHIP;
}
