// ROCKET transform for MI355X (gfx950): the PPV features of MINIROCKET-style kernels, one group at a time.
//
// The paper's related-work section says of MINIROCKET that its weights take two values from a predetermined
// set, so that the convolution can be done by additions, and that it pools with PPV only (Eq. 1-2).  In this
// build's kernel set (rocket.h) the 84 kernels of a group share dilation d, padding and channel subset and
// differ only in which three of their nine weights are 2 (the other six are -1).  With s[t] the sum of the
// group's channels at (zero-padded) sample t and T_j = s[t + j d], kernel (a, b, c) gives
//     y = 3 (T_a + T_b + T_c) - (T_0 + ... + T_8),   so   3 y = U_a + U_b + U_c  with  U_j = 9 T_j - sum_j T_j.
// Per position the nine U_j are formed once (one rounding each, on the small difference) and every kernel
// costs one addition (U_a + U_b is shared by the kernels with the same first two positions) and one
// comparison 3 y > -3 bias; the generic kernel spends 9 n_ch multiply-adds on the same output.
//
// rk_mr_forward: one workgroup (four wavefronts) per (series, tile of positions of one group).  The
// channel-summed samples that the tile needs are staged in LDS once: for d <= 256 a tile is a run of
// consecutive positions and LDS holds that run plus 8 d samples; for larger d the positions are viewed as rows
// of d (position = row d + column) and a tile is a block of rows x columns, LDS holding rows + 8 rows of it.
// Either way tap j of the position at LDS index q is at q + j * stride (stride = d, or the block's width).
// The 84 kernels are taken in two passes of 42 over the staged tile so that 42 counters fit the scalar
// registers (v_cmp + s_bcnt1 + s_add per output) beside 42 thresholds in vector registers.  Counts are
// integers and added with atomics: the result does not depend on the order.  The tile holds 6,144 samples
// (24 KB: six workgroups per CU); 8,192 and 12,288 measured 15 and 40 % slower, 4,096 10 % slower.
// rk_mr_features: PPV = count / n per (series, kernel).
#include <hip/hip_runtime.h>

#include <type_traits>

#include "rocket_internal.hpp"
#include "rocket_device.hpp"

namespace {

struct MrTriples {
    int a[kMrSet], b[kMrSet], c[kMrSet];
};
constexpr MrTriples mr_triples()
{
    MrTriples s{};
    int k = 0;
    for (int a = 0; a < kMrLen; ++a)
        for (int b = a + 1; b < kMrLen; ++b)
            for (int c = b + 1; c < kMrLen; ++c, ++k) { s.a[k] = a; s.b[k] = b; s.c[k] = c; }
    return s;
}
constexpr MrTriples kTriples = mr_triples();
constexpr int kHalf = kMrSet / 2;

// Kernels [LO, LO + kHalf) of the group over the staged tile.  `items` = rows x chunks of 64 columns, dealt to
// the four wavefronts in turn; `limit0` = valid columns of row 0 and `limit_step` what a row adds to it
// (rows of the d-column view end where the output ends), `width_valid` the block's own valid columns.
template <int LO>
__device__ __forceinline__ void rk_mr_pass(const float *tile, int stride, int width, int rows, int width_valid,
                                           int limit0, int limit_step, const RkKernelRec *__restrict__ grec,
                                           int *__restrict__ wave_counts, int wave, int lane)
{
    float thr[kHalf];
    int cnt[kHalf];
    rk_static_for<0, kHalf>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        thr[i] = -3.f * grec[LO + i].bias;
        cnt[i] = 0;
    });
    const int chunks = width / 64;
    int row = 0, chunk = wave;
    while (chunk >= chunks) { chunk -= chunks; ++row; }
    while (row < rows) {
        const int col = chunk * 64 + lane;
        const int limit = min(width_valid, limit0 + row * limit_step);
        if (chunk * 64 < limit) {   // wave-uniform, so the counters stay scalar; lanes past the limit are given
            const bool ok = col < limit;   // U = -inf, which no threshold lies below
            const float *q = tile + row * width + col;
            float T[kMrLen], U[kMrLen];
            rk_static_for<0, kMrLen>([&](auto jc) {
                constexpr int j = decltype(jc)::value;
                T[j] = q[j * stride];
            });
            const float total = (((T[0] + T[1]) + (T[2] + T[3])) + ((T[4] + T[5]) + (T[6] + T[7]))) + T[8];
            rk_static_for<0, kMrLen>([&](auto jc) {
                constexpr int j = decltype(jc)::value;
                U[j] = ok ? fmaf(9.f, T[j], -total) : -INFINITY;
            });
            rk_static_for<0, kHalf>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                constexpr int a = kTriples.a[LO + i], b = kTriples.b[LO + i], c = kTriples.c[LO + i];
                const float y3 = (U[a] + U[b]) + U[c];
                cnt[i] += __builtin_popcountll(__ballot(y3 > thr[i]));
            });
        }
        chunk += 4;
        while (chunk >= chunks) { chunk -= chunks; ++row; }
    }
    if (lane == 0) {
        rk_static_for<0, kHalf>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            wave_counts[wave * kHalf + i] = cnt[i];
        });
    }
}

// Fills the LDS tile of a work item with the sum of the group's NCH channels (added in the order of the
// channel list).  Sample index i of a padded row seen through `series` is x[i - pad]; the outputs need
// i < reach = n + 8 d, and the zeros that follow the samples of a row extend at least that far.
template <int NCH>
__device__ __forceinline__ void rk_mr_stage(float *tile, const float *series, const int32_t *__restrict__ chan,
                                            int row_len, const RkMrJob &job, int d, int reach, int tid)
{
    const float *rows[NCH];
    rk_static_for<0, NCH>([&](auto cc) {
        constexpr int c = decltype(cc)::value;
        rows[c] = series + static_cast<size_t>(chan[c]) * row_len;
    });
    auto sum_at = [&](unsigned i) {
        float v[NCH];
        const unsigned at = i * 4u;     // a 32-bit byte offset beside a scalar row address: no 64-bit vector arithmetic
        rk_static_for<0, NCH>([&](auto cc) {
            constexpr int c = decltype(cc)::value;
            v[c] = *reinterpret_cast<const float *>(reinterpret_cast<const char *>(rows[c]) + at);
        });
        float s = v[0];
        rk_static_for<1, NCH>([&](auto cc) { constexpr int c = decltype(cc)::value; s += v[c]; });
        return s;
    };
    if (job.mode == 0) {
        // positions [first, first + count): LDS index = position - first
        const int total = job.count + (kMrLen - 1) * d;
        for (int u = tid; u < total; u += 256) tile[u] = sum_at(static_cast<unsigned>(job.first + u));
    } else {
        // output rows [first, first + rows) x columns [col0, col0 + width): LDS index = row * width + column
        for (int u = 0; u < job.rows + (kMrLen - 1); ++u) {
            const int base = (job.first + u) * d + job.col0;
            for (int c0 = tid; c0 < job.width; c0 += 256) {
                const int i = base + c0;
                tile[u * job.width + c0] = i < reach ? sum_at(static_cast<unsigned>(i)) : 0.f;
            }
        }
    }
}

__global__ __launch_bounds__(256) void rk_mr_forward(const float *__restrict__ xpad, int row_len, int lead, int C,
                                                     const RkKernelRec *__restrict__ recs,
                                                     const int32_t *__restrict__ channels,
                                                     const RkMrJob *__restrict__ jobs, int njobs, int B, int spread,
                                                     int K, int *__restrict__ counts)
{
    __shared__ float tile[kMrTileFloats + 64];   // lanes past the end of a tile's last 64 positions read (and discard) up to 63 more
    __shared__ int wave_counts[2][4 * kHalf];
    int b, item;
    if (!rk_block_to_pair(njobs, B, spread, b, item)) return;
    const RkMrJob job = jobs[item];
    const RkKernelRec *grec = recs + static_cast<size_t>(job.group) * kMrSet;
    const RkKernelRec rec = grec[0];
    const int d = rec.dil, n = rec.nout, nch = rec.nch;
    const int tid = static_cast<int>(threadIdx.x);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const float *series = xpad + static_cast<size_t>(b) * C * row_len + (lead - rec.pad);
    const int32_t *chan = channels + rec.ch_off;
    const int reach = n + (kMrLen - 1) * d;

    int stride, width, rows, width_valid, limit0, limit_step;
    if (job.mode == 0) {
        stride = d; width = job.width; rows = 1; width_valid = job.count; limit0 = job.count; limit_step = 0;
    } else {
        stride = job.width; width = job.width; rows = job.rows;
        width_valid = min(job.width, d - job.col0);
        limit0 = n - job.first * d - job.col0;     // valid columns of the block's first row if the output ended in it
        limit_step = -d;
    }
    switch (nch) {    // the channel count is a template parameter of the staging loops: loads back to back, no branches
    case 1: rk_mr_stage<1>(tile, series, chan, row_len, job, d, reach, tid); break;
    case 2: rk_mr_stage<2>(tile, series, chan, row_len, job, d, reach, tid); break;
    case 3: rk_mr_stage<3>(tile, series, chan, row_len, job, d, reach, tid); break;
    case 4: rk_mr_stage<4>(tile, series, chan, row_len, job, d, reach, tid); break;
    case 5: rk_mr_stage<5>(tile, series, chan, row_len, job, d, reach, tid); break;
    case 6: rk_mr_stage<6>(tile, series, chan, row_len, job, d, reach, tid); break;
    case 7: rk_mr_stage<7>(tile, series, chan, row_len, job, d, reach, tid); break;
    case 8: rk_mr_stage<8>(tile, series, chan, row_len, job, d, reach, tid); break;
    default: rk_mr_stage<9>(tile, series, chan, row_len, job, d, reach, tid); break;
    }
    __syncthreads();
    rk_mr_pass<0>(tile, stride, width, rows, width_valid, limit0, limit_step, grec, wave_counts[0], wave, lane);
    rk_mr_pass<kHalf>(tile, stride, width, rows, width_valid, limit0, limit_step, grec, wave_counts[1], wave, lane);
    __syncthreads();
    if (tid < kMrSet) {
        const int *w = wave_counts[tid / kHalf] + tid % kHalf;
        const int sum = (w[0] + w[kHalf]) + (w[2 * kHalf] + w[3 * kHalf]);
        if (sum != 0) atomicAdd(counts + static_cast<size_t>(b) * K + static_cast<size_t>(job.group) * kMrSet + tid, sum);
    }
}

__global__ __launch_bounds__(256) void rk_mr_clear(int *__restrict__ counts, int total)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < total) counts[i] = 0;
}

// PPV (Eq. 2): the positive count over the kernel's own output length
__global__ __launch_bounds__(256) void rk_mr_features(const int *__restrict__ counts, int B, int K,
                                                      const RkKernelRec *__restrict__ recs, float *__restrict__ out)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= B * K) return;
    const int kid = i % K;
    out[i] = static_cast<float>(static_cast<double>(counts[i]) / static_cast<double>(recs[kid].nout));
}

}  // namespace

int rk_launch_minirocket_clear(const rocket_kernels *h, int32_t B, int32_t *counts, void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    const int total = B * h->K;
    hipLaunchKernelGGL(rk_mr_clear, dim3((total + 255) / 256), dim3(256), 0, stream, counts, total);
    return hipGetLastError() == hipSuccess ? ROCKET_OK : ROCKET_EHIP;
}

int rk_launch_minirocket_forward(const rocket_kernels *h, const float *xpad, int32_t B, int32_t *counts, void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    const int njobs = static_cast<int>(h->mr_jobs.size());
    const int spread = rk_spread(h, B);
    const int64_t groups = rk_grid_groups(B, njobs, spread);
    hipLaunchKernelGGL(rk_mr_forward, dim3(static_cast<unsigned>(groups)), dim3(256), 0, stream, xpad,
                       static_cast<int>(h->row_len), h->lead, h->C, h->d_rec, h->d_channels, h->d_mr_jobs, njobs, B,
                       spread, h->K, counts);
    return hipGetLastError() == hipSuccess ? ROCKET_OK : ROCKET_EHIP;
}

int rk_launch_minirocket_features(const rocket_kernels *h, const int32_t *counts, int32_t B, float *out, void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    const int total = B * h->K;
    hipLaunchKernelGGL(rk_mr_features, dim3((total + 255) / 256), dim3(256), 0, stream, counts, B, h->K, h->d_rec, out);
    return hipGetLastError() == hipSuccess ? ROCKET_OK : ROCKET_EHIP;
}
