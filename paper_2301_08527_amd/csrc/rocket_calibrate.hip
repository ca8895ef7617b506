// ROCKET transform for MI355X (gfx950): measurement support.  The transform's multiply-adds are
// plain (one per lane) v_fma_f32 / v_fmac_f32 instructions; this kernel issues nothing else, from
// enough independent accumulators and wavefronts to keep every vector ALU busy, so its rate is the
// ceiling that such code can reach on the device it runs on.  The data sheet's FP32 vector peak
// assumes the packed two-per-lane form and is twice that.
#include <hip/hip_runtime.h>

#include <vector>

#include "rocket_internal.hpp"
#include "rocket_device.hpp"

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


// ------------------------------------------------------------------ the other units
//
// Rates of the units that bound the transform's kernels, measured with kernels that use one unit each:
// buffer loads into registers from a footprint that stays in a CU's L1 and from one that streams out of L2,
// the same as 16-byte loads, 16-byte loads that write LDS directly, LDS reads, and the FP32 matrix
// instruction with the smallest tile (4x4x1, 16 blocks), alone and beside vector multiply-adds.

namespace {

typedef float rk_f4 __attribute__((ext_vector_type(4)));
typedef int rk_i4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void *rk_lds_ptr;

constexpr int kLoadGroups = 256 * 6;     // workgroups of 256 lanes
constexpr int kLoadIters = 1500;
constexpr int kRowsPerIter = 16;         // dword loads per lane and iteration (4 as 16-byte loads)

__device__ __forceinline__ __amdgpu_buffer_rsrc_t rk_cal_buffer(const void *p, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, static_cast<int>(bytes), 0x00020000);
}

// Every workgroup reads `region_bytes` bytes over and over, block b the region b % nregions; one region of a
// few KB stays in L1, many regions of 1 MB stream out of L2.  W = dwords per lane and load.
template <int W>
__global__ __launch_bounds__(256) void rk_cal_loads(const float *base, unsigned region_bytes, unsigned nregions, int iters,
                                                    float *sink)
{
    constexpr int NL = kRowsPerIter / W;
    const unsigned lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const __amdgpu_buffer_rsrc_t r =
        rk_cal_buffer(reinterpret_cast<const char *>(base) + static_cast<size_t>(blockIdx.x % nregions) * region_bytes, region_bytes);
    const unsigned rowb = 256u * W, voff = lane * 4u * W;
    unsigned so = (wave * NL * rowb) % region_bytes;
    float acc = 0.f;
    for (int it = 0; it < iters; ++it) {
        float v[NL * W];
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            unsigned s = so + i * rowb;
            if (s >= region_bytes) s -= region_bytes;
            if constexpr (W == 1) {
                v[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff, s, 0));
            } else {
                const rk_i4 q = __builtin_amdgcn_raw_buffer_load_b128(r, voff, s, 0);
                v[4 * i] = __builtin_bit_cast(float, q.x); v[4 * i + 1] = __builtin_bit_cast(float, q.y);
                v[4 * i + 2] = __builtin_bit_cast(float, q.z); v[4 * i + 3] = __builtin_bit_cast(float, q.w);
            }
        }
#pragma unroll
        for (int i = 0; i < NL * W; ++i) acc += v[i];
        so += NL * rowb;
        while (so >= region_bytes) so -= region_bytes;
    }
    if (acc == 12345.678f) *sink = acc;
}

// 16-byte buffer loads with the LDS modifier: four per iteration and wavefront into the wavefront's own 4 KB of
// LDS (lane l's 16 bytes land at byte 16*l of the 1 KB block the instruction names), then a wait for them.
__global__ __launch_bounds__(256) void rk_cal_loads_to_lds(const float *base, unsigned region_bytes, unsigned nregions, int iters,
                                                           float *sink)
{
    __shared__ __attribute__((aligned(16))) char slab[4][4096];
    const unsigned lane = threadIdx.x & 63;
    const unsigned wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const __amdgpu_buffer_rsrc_t r =
        rk_cal_buffer(reinterpret_cast<const char *>(base) + static_cast<size_t>(blockIdx.x % nregions) * region_bytes, region_bytes);
    unsigned so = (wave * 4096u) % region_bytes;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            unsigned s = so + i * 1024u;
            if (s >= region_bytes) s -= region_bytes;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (rk_lds_ptr)(&slab[wave][i * 1024]), 16, lane * 16u, s, 0, 0);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        so += 4096u;
        while (so >= region_bytes) so -= region_bytes;
    }
    if (iters < 0) *sink = *reinterpret_cast<const float *>(&slab[wave][lane * 4]);
}

// LDS reads, one dword per lane and read, consecutive lanes at consecutive words.
__global__ __launch_bounds__(256) void rk_cal_lds_reads(int iters, float *sink)
{
    __shared__ float words[8192];
    for (int i = threadIdx.x; i < 8192; i += 256) words[i] = static_cast<float>(i);
    __syncthreads();
    const unsigned lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float acc = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kRowsPerIter; ++i) acc += words[(wave * 2048 + lane + i * 64 + it) & 8191u];
    }
    if (acc == 12345.678f) *sink = acc;
}

// mode 0: every wavefront issues the 4x4x1 FP32 matrix instruction on 8 independent accumulator tiles;
// mode 1: even wavefronts do that, odd wavefronts run plain multiply-add chains; mode 2: only the even ones
// work; mode 3: only the odd ones.
__global__ __launch_bounds__(256) void rk_cal_matrix(int iters, float a0, float b0, int mode, float *sink)
{
    const unsigned wave = threadIdx.x >> 6;
    const bool matrix_wave = mode == 0 || (wave & 1) == 0;
    float s = 0.f;
    if (matrix_wave) {
        if (mode == 3) return;
        rk_f4 acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = rk_f4{0.f, 0.f, 0.f, 0.f};
        const float a = a0 + threadIdx.x * 1e-6f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 8; ++r) {
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_4x4x1f32(a, b0, acc[i], 0, 0, 0);
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) s += acc[i].x + acc[i].y + acc[i].z + acc[i].w;
    } else {
        if (mode == 2) return;
        float v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = threadIdx.x * 0.001f + i;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int r = 0; r < 8; ++r) {
#pragma unroll
                for (int i = 0; i < 16; ++i) v[i] = fmaf(v[i], 0.999f, 0.001f);
            }
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) s += v[i];
    }
    if (s == 12345.678f) *sink = s;
}

// One forward strip per wavefront and pass, as rk_segment forms it (32 rows x 64 columns, kernel length 9, four
// channels, rows 1,024 floats apart, max + PPV pooling), in two forms that give bit-identical outputs:
//   MATRIX = false: 40 loads and 288 plain multiply-adds per channel
//   MATRIX = true : the same 40 loads, then 96 v_mfma_f32_4x4x1_16b_f32 in Toeplitz form -- a block is 4 output rows
//                   x 4 neighbouring columns, one step per input row; lane l supplies its own column's sample as B
//                   and w[delta - l % 4] as A (the banded weight operand, built with quad shifts), and receives
//                   the four rows of its own column
// Their rates answer whether the matrix cores would speed the conv up.  The weights arrive by value.
struct RkCalWeights { float w[4][9]; };
constexpr int kStripRows = 32, kStripLen = 9, kStripWin = kStripRows + kStripLen - 1, kStripCh = 4;
constexpr int kStripD = 1024, kStripPasses = 24, kStripGroups = 256 * 8;
typedef float rk_f4 __attribute__((ext_vector_type(4)));

template <bool MATRIX>
__global__ __launch_bounds__(256) void rk_cal_strip(const float *x, RkCalWeights wts, float threshold,
                                                    float *__restrict__ lane_max, int *__restrict__ wave_count)
{
    const unsigned lane = threadIdx.x & 63u;
    const unsigned gw = blockIdx.x * 4u + static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6)));
    const unsigned row_bytes = 16u << 20;             // one channel: 4,096 rows of 1,024 floats
    const unsigned dbytes = kStripD * 4u;
    float vmax = -INFINITY;
    int cnt = 0;
    for (int s = 0; s < kStripPasses; ++s) {
        const unsigned col0 = ((gw * kStripPasses + static_cast<unsigned>(s)) * 64u) % kStripD;
        const unsigned voff = (col0 + lane) * 4u;
        float acc[kStripRows];
#pragma unroll
        for (int i = 0; i < kStripRows; ++i) acc[i] = 0.f;
        for (int c = 0; c < kStripCh; ++c) {
            const __amdgpu_buffer_rsrc_t r = rk_row_buffer(reinterpret_cast<const char *>(x) + static_cast<size_t>(c) * row_bytes, row_bytes);
            float w[kStripLen];
#pragma unroll
            for (int j = 0; j < kStripLen; ++j) w[j] = wts.w[c][j];
            float xs[kStripWin];
            uint32_t soff = 0;
            rk_static_for<0, kStripWin>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                xs[i] = rk_load(r, voff, soff);
                soff = rk_advance(soff, dbytes);
            });
            if constexpr (!MATRIX) {
                rk_static_for<0, kStripWin>([&](auto ic) {
                    constexpr int i = decltype(ic)::value;
                    rk_taps<kStripLen, kStripRows, i>(w, xs[i], acc);
                });
            } else {
                float wt[kStripLen + 3];
                const bool first = (lane & 3u) == 0u;
                float run = 0.f;
                rk_static_for<0, kStripLen + 3>([&](auto dc) {
                    constexpr int dl = decltype(dc)::value;
                    const float shifted = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(
                        0, __builtin_bit_cast(int, run), 0x90 /* quad_perm [0,0,1,2] */, 0xF, 0xF, false));
                    float fresh = 0.f;
                    if constexpr (dl < kStripLen) fresh = w[dl];
                    run = first ? fresh : shifted;
                    wt[dl] = run;
                });
                rk_f4 a4[kStripRows / 4];
#pragma unroll
                for (int m = 0; m < kStripRows / 4; ++m) a4[m] = rk_f4{acc[4 * m], acc[4 * m + 1], acc[4 * m + 2], acc[4 * m + 3]};
                __builtin_amdgcn_sched_barrier(0);    // all loads of the channel are requested before the first matrix instruction
                rk_static_for<0, kStripWin>([&](auto ic) {
                    constexpr int u = decltype(ic)::value;
                    rk_static_for<0, kStripRows / 4>([&](auto mc) {
                        constexpr int m = decltype(mc)::value;
                        constexpr int dl = u - 4 * m;
                        if constexpr (dl >= 0 && dl < kStripLen + 3)
                            a4[m] = __builtin_amdgcn_mfma_f32_4x4x1f32(wt[dl], xs[u], a4[m], 0, 0, 0);
                    });
                });
#pragma unroll
                for (int m = 0; m < kStripRows / 4; ++m) {
                    acc[4 * m] = a4[m][0]; acc[4 * m + 1] = a4[m][1]; acc[4 * m + 2] = a4[m][2]; acc[4 * m + 3] = a4[m][3];
                }
            }
        }
#pragma unroll
        for (int i = 0; i < kStripRows; ++i) {
            vmax = fmaxf(vmax, acc[i]);
            cnt += __builtin_popcountll(__ballot(acc[i] > threshold));
        }
    }
    lane_max[blockIdx.x * 256 + threadIdx.x] = vmax;
    if (lane == 0) wave_count[gw] = cnt;
}

// pseudo-random samples in [-1, 1) for the strips (the other micro-kernels do not care what they load)
__global__ __launch_bounds__(256) void rk_cal_fill(float *x, size_t n)
{
    for (size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x; i < n; i += static_cast<size_t>(gridDim.x) * 256) {
        uint32_t h = static_cast<uint32_t>(i) * 2654435761u;
        h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
        x[i] = static_cast<float>(h >> 8) * (1.0f / 8388608.0f) - 1.0f;
    }
}

}  // namespace

extern "C" int rocket_calibrate_units(double *out, int32_t count, void *hip_stream)
{
    if (!out || count < ROCKET_CAL_COUNT) return rk_fail(ROCKET_EINVAL, "rocket_calibrate_units: out must hold ROCKET_CAL_COUNT values");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const size_t bytes = static_cast<size_t>(64) << 20;
    float *buf = nullptr, *sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t err = hipMalloc(&buf, bytes);
    if (err == hipSuccess) err = hipMalloc(&sink, 256);
    if (err == hipSuccess) hipLaunchKernelGGL(rk_cal_fill, dim3(4096), dim3(256), 0, stream, buf, bytes / 4);
    if (err == hipSuccess) err = hipEventCreate(&e0);
    if (err == hipSuccess) err = hipEventCreate(&e1);
    // runs `launch` twice (the first run warms caches and clocks) and returns the second run's milliseconds
    auto timed = [&](auto launch, double &ms_out) {
        if (err != hipSuccess) return;
        launch();
        err = hipEventRecord(e0, stream);
        launch();
        if (err == hipSuccess) err = hipEventRecord(e1, stream);
        if (err == hipSuccess) err = hipEventSynchronize(e1);
        float ms = 0.f;
        if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
        if (err == hipSuccess) err = hipGetLastError();
        ms_out = ms;
    };
    const double load_bytes = 4.0 * kLoadGroups * kLoadIters * kRowsPerIter * 256.0;   // per launch, all wavefronts
    double ms = 0.0;
    auto gbps = [&](double b) { return ms > 0.0 ? b / (ms * 1e-3) / 1e9 : 0.0; };
    timed([&] { hipLaunchKernelGGL((rk_cal_loads<1>), dim3(kLoadGroups), dim3(256), 0, stream, buf, 4096u, 1u, kLoadIters, sink); }, ms);
    out[ROCKET_CAL_LOAD_B32_L1] = gbps(load_bytes);
    timed([&] { hipLaunchKernelGGL((rk_cal_loads<1>), dim3(kLoadGroups), dim3(256), 0, stream, buf, 1u << 20, 64u, kLoadIters, sink); }, ms);
    out[ROCKET_CAL_LOAD_B32_L2] = gbps(load_bytes);
    timed([&] { hipLaunchKernelGGL((rk_cal_loads<4>), dim3(kLoadGroups), dim3(256), 0, stream, buf, 16384u, 1u, kLoadIters, sink); }, ms);
    out[ROCKET_CAL_LOAD_B128_L1] = gbps(load_bytes);
    timed([&] { hipLaunchKernelGGL((rk_cal_loads<4>), dim3(kLoadGroups), dim3(256), 0, stream, buf, 1u << 20, 64u, kLoadIters, sink); }, ms);
    out[ROCKET_CAL_LOAD_B128_L2] = gbps(load_bytes);
    timed([&] { hipLaunchKernelGGL(rk_cal_loads_to_lds, dim3(kLoadGroups), dim3(256), 0, stream, buf, 1u << 20, 64u, kLoadIters, sink); }, ms);
    out[ROCKET_CAL_LOAD_B128_TO_LDS] = gbps(4.0 * kLoadGroups * kLoadIters * 4096.0);
    timed([&] { hipLaunchKernelGGL(rk_cal_lds_reads, dim3(kLoadGroups), dim3(256), 0, stream, kLoadIters, sink); }, ms);
    out[ROCKET_CAL_LDS_READ_B32] = gbps(load_bytes);
    const int mgroups = 256 * 8, miters = 2000;
    const double mflop = 64.0 * 512.0 * miters, vflop = 128.0 * 128.0 * miters;   // per wavefront: matrix / vector work
    auto tflops = [&](double f) { return ms > 0.0 ? f / (ms * 1e-3) / 1e12 : 0.0; };
    timed([&] { hipLaunchKernelGGL(rk_cal_matrix, dim3(mgroups), dim3(256), 0, stream, miters, 1.0001f, 0.5f, 0, sink); }, ms);
    out[ROCKET_CAL_MFMA_F32_4X4X1] = tflops(mgroups * 4.0 * mflop);
    timed([&] { hipLaunchKernelGGL(rk_cal_matrix, dim3(mgroups), dim3(256), 0, stream, miters, 1.0001f, 0.5f, 2, sink); }, ms);
    const double ms_matrix_half = ms;
    timed([&] { hipLaunchKernelGGL(rk_cal_matrix, dim3(mgroups), dim3(256), 0, stream, miters, 1.0001f, 0.5f, 3, sink); }, ms);
    const double ms_vector_half = ms;
    timed([&] { hipLaunchKernelGGL(rk_cal_matrix, dim3(mgroups), dim3(256), 0, stream, miters, 1.0001f, 0.5f, 1, sink); }, ms);
    // 1 = the two kinds of wavefront take as long together as one after the other (no overlap); 0.5 would be full overlap
    out[ROCKET_CAL_MFMA_VALU_SERIAL] = (ms_matrix_half + ms_vector_half) > 0.0 ? ms / (ms_matrix_half + ms_vector_half) : 0.0;
    // the conv strip in its two forms (useful multiply-adds counted); the 64 MB buffer is the four channels
    RkCalWeights cw;
    for (int c = 0; c < 4; ++c)
        for (int j = 0; j < 9; ++j) cw.w[c][j] = 0.125f * static_cast<float>((c * 9 + j) % 7 - 3);
    const double sflop = 2.0 * kStripGroups * 4.0 * kStripPasses * 64.0 * kStripRows * kStripLen * kStripCh;
    const size_t lanes = static_cast<size_t>(kStripGroups) * 256, waves = static_cast<size_t>(kStripGroups) * 4;
    float *res = nullptr;                 // per form: the lanes' maxima, then the wavefronts' counts
    if (err == hipSuccess) err = hipMalloc(&res, 2 * (lanes + waves) * 4);
    float *max_a = res, *max_b = res + lanes + waves;
    int *cnt_a = reinterpret_cast<int *>(res + lanes), *cnt_b = reinterpret_cast<int *>(max_b + lanes);
    timed([&] { hipLaunchKernelGGL((rk_cal_strip<false>), dim3(kStripGroups), dim3(256), 0, stream, buf, cw, 0.1f, max_a, cnt_a); }, ms);
    out[ROCKET_CAL_STRIP_VALU] = tflops(sflop);
    timed([&] { hipLaunchKernelGGL((rk_cal_strip<true>), dim3(kStripGroups), dim3(256), 0, stream, buf, cw, 0.1f, max_b, cnt_b); }, ms);
    out[ROCKET_CAL_STRIP_MFMA] = tflops(sflop);
    bool same = true;
    if (err == hipSuccess) {
        std::vector<uint32_t> host(2 * (lanes + waves));
        err = hipMemcpy(host.data(), res, host.size() * 4, hipMemcpyDeviceToHost);
        for (size_t i = 0; i < lanes + waves && err == hipSuccess; ++i) same = same && host[i] == host[lanes + waves + i];
    }
    if (res) (void)hipFree(res);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (buf) (void)hipFree(buf);
    if (sink) (void)hipFree(sink);
    if (err != hipSuccess) return rk_fail(ROCKET_EHIP, std::string("rocket_calibrate_units: ") + hipGetErrorString(err));
    if (!same) return rk_fail(ROCKET_EHIP, "rocket_calibrate_units: the matrix form of the conv strip does not reproduce the vector form");
    return ROCKET_OK;
}
