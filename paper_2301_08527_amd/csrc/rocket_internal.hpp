// Internal declarations shared by the host sampler and the HIP translation units.
#pragma once
#include <cstdint>
#include <string>
#include <utility>
#include <vector>

#include "rocket.h"

// Constants shared by the host planner and the kernels.
#ifndef RK_LDS_ROWS
#define RK_LDS_ROWS 17
#endif
#ifndef RK_LDS_MAXD
#define RK_LDS_MAXD 16
#endif
constexpr int kThreads = 256;                 // lanes of the standard workgroup
constexpr int kLdsRows = RK_LDS_ROWS;         // rows per band in the LDS path
constexpr int kLdsMaxD = RK_LDS_MAXD;         // dilations below this take the LDS path
constexpr int kXcds = 8;                       // accelerator dies (XCDs) of the chip, each with its own L2
constexpr int kFewMinD = 256;                 // few-rows path: smallest dilation ...
constexpr int kFewRowsMax = 24;               // ... and largest number of output rows
#ifndef RK_TILE_POSITIONS
#define RK_TILE_POSITIONS 16384
#endif
constexpr int64_t kTilePositions = RK_TILE_POSITIONS;   // smallest time tile of a forward job, in output positions

// MINIROCKET-style kernel set: groups of kMrSet kernels of length kMrLen (rocket.h)
constexpr int kMrSet = 84;
constexpr int kMrLen = 9;
#ifndef RK_MR_TILE
#define RK_MR_TILE 6144
#endif
#ifndef RK_MR_LINEAR_MAXD
#define RK_MR_LINEAR_MAXD 256
#endif
constexpr int kMrTileFloats = RK_MR_TILE;          // channel-summed samples that one workgroup of the group kernel stages in LDS
constexpr int kMrLinearMaxD = RK_MR_LINEAR_MAXD;   // up to this dilation a tile is a run of consecutive positions
static_assert(kMrTileFloats >= 16 * kMrLinearMaxD && kMrTileFloats >= 9 * 256, "a tile must hold its halo and at least one row of outputs");

// One work item of the group kernel (32 bytes).  mode 0: positions [first, first + count) of the group's
// output, `width` = count rounded up to 64.  mode 1: rows [first, first + rows) x columns [col0, col0 + width)
// of the output viewed as rows of d positions.
struct RkMrJob {
    int32_t group, mode, first, count, col0, width, rows, reserved;
};

// One packed record per kernel as the device code reads it (32 bytes).
struct RkKernelRec {
    int32_t len, dil, pad, nout;
    float bias;
    int32_t nch;
    int32_t ch_off;  // into channels[]
    int32_t w_off;   // into weights[]
};

// One forward work item: rows [row0, row1) of kernel `kernel` (rows of d consecutive
// output positions); 16 bytes.
struct RkJob {
    int32_t kernel;
    int32_t row0, row1;
    int32_t flags;   // bit 0: also owns the partial last row; bit 1: covers the whole kernel
};

struct rocket_kernels {
    int32_t K = 0, C = 0, L = 0;
    std::vector<int32_t> length, dilation, padding, n_ch, channels;
    std::vector<float> bias, weights;
    std::vector<int64_t> ch_off, w_off;

    // plan: forward / backward jobs and padded row geometry
    // forward plan: every kernel's rows cut into time tiles; jobs sorted by time window so
    // that workgroups running together read the same stretch of the series
    std::vector<RkJob> jobs;
    std::vector<int32_t> kjob_off, kjob_idx;   // jobs of kernel k: kjob_idx[kjob_off[k] .. kjob_off[k+1])
    // backward pass: job j owns words [bjob_off[j], bjob_off[j+1]) of a series' row of partial
    // results (its kernel's n_ch*len gradient sums + 4 words)
    std::vector<int32_t> bjob_off;
    int32_t pad_max = 0;     // largest padding of any kernel
    int32_t lead = 0;        // zeros in front of every padded row (multiple of 64)
    int64_t row_len = 0;     // floats per padded row (multiple of 64)
    double conv_fma = 0.0;   // sum_k n_k * n_ch_k * len_k
    double outputs = 0.0;    // sum_k n_k
    int32_t max_terms = 0;   // largest n_ch * length of any kernel

    // device mirror (allocated on first use on `device`)
    int device = -1;
    void *d_blob = nullptr;
    size_t blob_bytes = 0;
    bool params_dirty = true;    // host parameters are newer than the device mirror
    bool host_stale = false;     // the device mirror was updated in place (training) after the last download
    void *update_stream = nullptr;   // stream of that update
    const RkKernelRec *d_rec = nullptr;
    const RkJob *d_jobs = nullptr;
    const int32_t *d_kjob_off = nullptr;
    const int32_t *d_kjob_idx = nullptr;
    const int32_t *d_bjob_off = nullptr;
    const int32_t *d_channels = nullptr;
    float *d_weights = nullptr;

    // MINIROCKET-style handles (rocket_minirocket_kernels): number of groups while the weights are the
    // predetermined set (0 otherwise), work items of the group kernel and their device copy (own allocation,
    // made at the first rocket_minirocket_transform)
    int32_t mr_groups = 0;
    std::vector<RkMrJob> mr_jobs;
    const RkMrJob *d_mr_jobs = nullptr;

    // optional event pairs around the dominant kernel of each call
    bool profile = false;
    std::vector<std::pair<void *, void *>> events;
};

void rk_set_error(const std::string &msg);
int rk_fail(int code, const std::string &msg);

// sampler.cpp: fills the per-kernel arrays of `h` (K, C, L already set)
void rk_sample_kernels(uint64_t seed, rocket_kernels &h);
// sampler.cpp: the MINIROCKET-style kernel set (groups of 84 two-valued kernels; C, L already set) and the
// (training example, rank) draws of the biases
void rk_sample_minirocket(uint64_t seed, int32_t groups, rocket_kernels &h);
void rk_minirocket_draws(uint64_t seed, const rocket_kernels &h, int32_t n_train, std::vector<int32_t> &example,
                         std::vector<int32_t> &rank);
// rocket_minirocket.hip: bias-free outputs of kernels [k0, k0 + count) on their drawn examples into ybuf (rows of
// `stride` floats), and the selection of the drawn order statistic, whose negative becomes the kernel's bias in
// the device records
int rk_launch_minirocket_outputs(const rocket_kernels *h, const float *xpad, const int32_t *example_dev, int32_t k0,
                                 int32_t count, int64_t stride, float *ybuf, void *stream);
int rk_launch_minirocket_select(const rocket_kernels *h, const int32_t *rank_dev, int32_t k0, int32_t count,
                                int64_t stride, const float *ybuf, void *stream);
// rocket_minirocket_forward.hip: the PPV features of a MINIROCKET-style handle, group by group: clears the
// B x K counters, adds every work item's positive counts to them, turns them into features
int rk_launch_minirocket_clear(const rocket_kernels *h, int32_t B, int32_t *counts, void *stream);
int rk_launch_minirocket_forward(const rocket_kernels *h, const float *xpad, int32_t B, int32_t *counts, void *stream);
int rk_launch_minirocket_features(const rocket_kernels *h, const int32_t *counts, int32_t B, float *out, void *stream);
// rocket_api.hip: offsets, job plan, padded row geometry; returns ROCKET_OK or an error
int rk_finish_handle(rocket_kernels &h);

// Whether a launch over B series uses the per-XCD series mapping (rk_block_to_pair in
// rocket_device.hpp): when the series divide evenly among the XCDs (with 60 series four XCDs
// would get 8 and four 7, and the launch takes as long as 64), and while the kXcds padded series
// that are then in flight together fit in half of the 256 MB Infinity Cache.  (Measured at
// 64 x 20 x 50,000: 1 % faster, 22 % less L2 fill traffic; slower at 8 x 20 x 200,000, whose eight
// padded series are 192 MB, and for the short-series kernel, which does not use it.)
inline int rk_spread(const rocket_kernels *h, int32_t B)
{
    const int64_t series_bytes = static_cast<int64_t>(h->C) * h->row_len * 4;
    return (B % kXcds == 0 && kXcds * series_bytes <= (128LL << 20)) ? 1 : 0;
}
// Workgroups of a launch over B series x `items` work items each.
inline int64_t rk_grid_groups(int32_t B, int64_t items, int spread)
{
    const int64_t series = spread ? static_cast<int64_t>((B + kXcds - 1) / kXcds) * kXcds : B;
    return series * items;
}

// Kernel launchers (rocket_forward.hip, rocket_backward.hip).  `stream` is a hipStream_t.
// They enqueue and return ROCKET_OK, or ROCKET_EHIP if the launch itself was rejected.
int rk_launch_pad(const rocket_kernels *h, const float *x, int32_t B, float *xpad, void *stream);
// rocket_train.hip: loss gradient of a linear head, and the in-place parameter update of
// the handle's device mirror
int rk_launch_mse_grad(const double *pred, const float *targets, const double *coef, int32_t B, int32_t p,
                       float *grad_out, double *loss, void *stream);
int rk_launch_sgd_update(const rocket_kernels *h, const float *gw, const float *gb, float lr, int recentre,
                         void *stream);
// rocket_prologue.hip: the same copy from 8-bit samples, z-normalising every row on the way;
// `stats` is device scratch of 16 bytes per (series, channel) row
int rk_launch_pad_u8(const rocket_kernels *h, const uint8_t *x, int32_t B, float *xpad, void *stats, void *stream);
// forward kernel: one workgroup per (series, job); writes per-job partial results
// (max, positive count, sigmoid sum: three planes of B*J words) into `partials`
int rk_launch_forward(const rocket_kernels *h, const float *xpad, int32_t B, uint32_t mask, float nl, float ns,
                      float *partials, void *stream);
// same kernel with one wavefront per workgroup, for short series
int rk_launch_forward_short(const rocket_kernels *h, const float *xpad, int32_t B, uint32_t mask, float nl, float ns,
                            float *partials, void *stream);
// combines the per-job partials of every (series, kernel) into the feature planes
int rk_launch_finalize(const rocket_kernels *h, const float *partials, int32_t B, uint32_t mask, float *out,
                       void *stream);
int rk_launch_backward(const rocket_kernels *h, const float *xpad, int32_t B, const float *grad_out, int F,
                       int plane_soft, int plane_max, float lambda, float nl, float ns, float *partial, void *stream);
// sums the job partials of every kernel over the jobs and the batch, adds the max plane's
// sub-gradient at the first arg-max, writes grad_w and grad_b
int rk_launch_reduce_jobs(const rocket_kernels *h, const float *partial, const float *xpad, int32_t B,
                          const float *grad_out, int F, int plane_max, float *grad_w, float *grad_b, void *stream);
