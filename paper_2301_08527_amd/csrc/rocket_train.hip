// ROCKET transform for MI355X (gfx950): the small kernels around a training step through
// softPPV (paper section 3.2 makes the pooling differentiable; section 6 names training the
// kernel weights as the next thing to try).  The heavy parts of a step are the transform and
// the backward kernel; here are the loss gradient of a linear head and the parameter update.
//
//   rk_mse_grad   : G[b][i] = (2/B) (pred_b - y_b) coef[i]  and  loss = (1/B) sum_b (pred_b - y_b)^2
//   rk_sgd_update : w <- w - lr*gw, b <- b - lr*gb on the handle's device parameters, with an
//                   optional re-centring of every (kernel, channel) weight row
#include <hip/hip_runtime.h>

#include "rocket_internal.hpp"

// grid (ceil(p/256), B).  Block (0,0) also writes the loss (B is a batch size: a short loop).
__global__ __launch_bounds__(256) void rk_mse_grad(const double *__restrict__ pred, const float *__restrict__ targets,
                                                   const double *__restrict__ coef, int B, int p,
                                                   float *__restrict__ grad_out, double *__restrict__ loss)
{
    const int b = blockIdx.y;
    const int i = blockIdx.x * 256 + threadIdx.x;
    const double r = pred[b] - static_cast<double>(targets[b]);
    if (i < p) grad_out[static_cast<size_t>(b) * p + i] = static_cast<float>((2.0 / B) * r * coef[i]);
    if (loss && blockIdx.x == 0 && b == 0 && threadIdx.x == 0) {
        double s = 0.0;
        for (int q = 0; q < B; ++q) {
            const double e = pred[q] - static_cast<double>(targets[q]);
            s += e * e;
        }
        *loss = s / B;
    }
}

// One thread per kernel: its n_ch rows of `length` weights and its bias.
__global__ __launch_bounds__(256) void rk_sgd_update(RkKernelRec *__restrict__ recs, float *__restrict__ weights,
                                                     const float *__restrict__ gw, const float *__restrict__ gb,
                                                     int K, float lr, int recentre)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= K) return;
    RkKernelRec rec = recs[k];
    for (int c = 0; c < rec.nch; ++c) {
        float *row = weights + rec.w_off + c * rec.len;
        const float *g = gw + rec.w_off + c * rec.len;
        float sum = 0.f;
        for (int j = 0; j < rec.len; ++j) {
            const float v = fmaf(-lr, g[j], row[j]);
            row[j] = v;
            sum += v;
        }
        if (recentre) {
            const float mean = sum / static_cast<float>(rec.len);
            for (int j = 0; j < rec.len; ++j) row[j] -= mean;
        }
    }
    recs[k].bias = fmaf(-lr, gb[k], rec.bias);
}

int rk_launch_mse_grad(const double *pred, const float *targets, const double *coef, int32_t B, int32_t p,
                       float *grad_out, double *loss, void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    hipLaunchKernelGGL(rk_mse_grad, dim3(static_cast<unsigned>((p + 255) / 256), static_cast<unsigned>(B)), dim3(256), 0,
                       stream, pred, targets, coef, B, p, grad_out, loss);
    return hipGetLastError() == hipSuccess ? ROCKET_OK : ROCKET_EHIP;
}

int rk_launch_sgd_update(const rocket_kernels *h, const float *gw, const float *gb, float lr, int recentre,
                         void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    hipLaunchKernelGGL(rk_sgd_update, dim3(static_cast<unsigned>((h->K + 255) / 256)), dim3(256), 0, stream,
                       const_cast<RkKernelRec *>(h->d_rec), h->d_weights, gw, gb, h->K, lr, recentre);
    return hipGetLastError() == hipSuccess ? ROCKET_OK : ROCKET_EHIP;
}
