// ROCKET transform for MI355X (gfx950): measurement support.  The transform's multiply-adds are
// plain (one per lane) v_fma_f32 / v_fmac_f32 instructions; this kernel issues nothing else, from
// enough independent accumulators and wavefronts to keep every vector ALU busy, so its rate is the
// ceiling that such code can reach on the device it runs on.  The data sheet's FP32 vector peak
// assumes the packed two-per-lane form and is twice that.
#include <hip/hip_runtime.h>

#include "rocket_internal.hpp"

namespace {

constexpr int kAcc = 16;          // independent dependency chains per lane
constexpr int kInner = 8;         // unrolled rounds per loop iteration
constexpr int kIters = 4096;
constexpr int kGroups = 256 * 16; // workgroups of 256 lanes

__global__ __launch_bounds__(256) void rk_fma_chain(int iters, float a, float b, float *sink)
{
    float acc[kAcc];
#pragma unroll
    for (int i = 0; i < kAcc; ++i) acc[i] = static_cast<float>(threadIdx.x) * 0.001f + static_cast<float>(i);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < kInner; ++r) {
#pragma unroll
            for (int i = 0; i < kAcc; ++i) acc[i] = fmaf(acc[i], a, b);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < kAcc; ++i) s += acc[i];
    if (s == 12345.678f) *sink = s;     // never true for the arguments used; keeps the chains alive
}

}  // namespace

extern "C" int rocket_calibrate_fma(double *tflops, void *hip_stream)
{
    if (!tflops) return rk_fail(ROCKET_EINVAL, "rocket_calibrate_fma: NULL pointer");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    float *sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t err = hipMalloc(&sink, 256);
    if (err == hipSuccess) err = hipEventCreate(&e0);
    if (err == hipSuccess) err = hipEventCreate(&e1);
    float ms = 0.f;
    if (err == hipSuccess) {
        // a*x + b with |a| < 1 stays bounded: no overflow, no denormals
        hipLaunchKernelGGL(rk_fma_chain, dim3(kGroups), dim3(256), 0, stream, kIters / 8, 0.999f, 0.001f, sink);   // warm-up
        err = hipEventRecord(e0, stream);
        hipLaunchKernelGGL(rk_fma_chain, dim3(kGroups), dim3(256), 0, stream, kIters, 0.999f, 0.001f, sink);
        if (err == hipSuccess) err = hipEventRecord(e1, stream);
        if (err == hipSuccess) err = hipEventSynchronize(e1);
        if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
        if (err == hipSuccess) err = hipGetLastError();
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (sink) (void)hipFree(sink);
    if (err != hipSuccess) return rk_fail(ROCKET_EHIP, std::string("rocket_calibrate_fma: ") + hipGetErrorString(err));
    const double flop = 2.0 * kAcc * kInner * static_cast<double>(kIters) * 256.0 * kGroups;
    *tflops = flop / (static_cast<double>(ms) * 1e-3) / 1e12;
    return ROCKET_OK;
}
