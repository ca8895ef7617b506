// ROCKET transform for MI355X (gfx950): forward kernel for short series, one
// 64-lane wavefront per (series, kernel).  With a few thousand outputs or fewer a
// 256-lane workgroup would leave most lanes without a strip; a single wavefront
// fills its lanes with shorter strips and needs no cross-wavefront reduction.
#include "rocket_forward_impl.hpp"

int rk_launch_forward_short(const rocket_kernels *h, const float *xpad, int32_t B, uint32_t mask, float nl, float ns,
                            float *partials, void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    const int J = static_cast<int>(h->jobs.size());
    const int spread = 0;   // measured: the per-XCD series mapping makes the short-series launch 2 % slower
    hipLaunchKernelGGL(rk_forward<64>, dim3(static_cast<unsigned>(rk_grid_groups(B, J, spread))), dim3(64), 0, stream, xpad,
                       static_cast<int>(h->row_len), h->lead, h->L, h->C, J, h->d_rec, h->d_jobs, h->d_channels,
                       h->d_weights, mask, nl, ns, partials, B, spread);
    return hipGetLastError() == hipSuccess ? ROCKET_OK : ROCKET_EHIP;
}
