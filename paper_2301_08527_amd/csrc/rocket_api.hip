// ROCKET transform for MI355X (gfx950): C-ABI entry points (handles, validation, host-side
// plan, device mirror, launch sequencing).  See include/rocket.h for the contract of every
// entry point.  The kernels live in rocket_forward.hip / rocket_forward_short.hip (transform),
// rocket_backward.hip (soft-PPV backward), rocket_prologue.hip (8-bit input), rocket_ridge.hip
// (regressor), rocket_train.hip (loss gradient, parameter update) and rocket_calibrate.hip.
//
// One transform call is: zero-padding copy of the batch into the workspace -> forward kernel
// (one workgroup per series and job; a job is a time tile of one kernel's outputs and writes
// partial pooled values) -> rk_finalize (combines a kernel's jobs into the feature planes).
// One backward call is: the same copy -> backward kernel (one workgroup per series and job,
// per-job partial gradients) -> rk_reduce_jobs (sum over jobs and batch in a fixed order).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <type_traits>

#include "rocket_internal.hpp"

// ------------------------------------------------------------------ errors

static thread_local std::string g_last_error;

void rk_set_error(const std::string &msg) { g_last_error = msg; }

int rk_fail(int code, const std::string &msg)
{
    g_last_error = msg;
    return code;
}

#define RK_HIP(call)                                                                   \
    do {                                                                               \
        hipError_t e_ = (call);                                                        \
        if (e_ != hipSuccess)                                                          \
            return rk_fail(ROCKET_EHIP, std::string(#call) + ": " + hipGetErrorString(e_)); \
    } while (0)

// ------------------------------------------------------------------ host plan

static inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }

int rk_finish_handle(rocket_kernels &h)
{
    const int32_t K = h.K;
    // byte offsets inside a padded row (up to 42 dilation steps of at most L/6 floats)
    // are 32-bit in the kernels
    if (h.L > 100000000) return rk_fail(ROCKET_EINVAL, "series longer than 100,000,000 samples are not supported");
    h.ch_off.assign(K + 1, 0);
    h.w_off.assign(K + 1, 0);
    h.pad_max = 0;
    h.conv_fma = 0.0;
    h.outputs = 0.0;
    h.max_terms = 0;
    int32_t max_dil = 0;
    for (int32_t k = 0; k < K; ++k) {
        h.ch_off[k + 1] = h.ch_off[k] + h.n_ch[k];
        h.w_off[k + 1] = h.w_off[k] + static_cast<int64_t>(h.n_ch[k]) * h.length[k];
        const int64_t n = static_cast<int64_t>(h.L) + 2LL * h.padding[k] -
                          static_cast<int64_t>(h.length[k] - 1) * h.dilation[k];
        if (n < 1) return rk_fail(ROCKET_ESHAPE, "kernel " + std::to_string(k) + " has no output position");
        h.pad_max = std::max(h.pad_max, h.padding[k]);
        max_dil = std::max(max_dil, h.dilation[k]);
        h.max_terms = std::max(h.max_terms, h.n_ch[k] * h.length[k]);
        h.conv_fma += static_cast<double>(n) * h.n_ch[k] * h.length[k];
        h.outputs += static_cast<double>(n);
    }
    if (h.w_off[K] > INT32_MAX || h.ch_off[K] > INT32_MAX)
        return rk_fail(ROCKET_EINVAL, "too many weights for 32-bit offsets");
    // Jobs of the forward and the backward pass.  A kernel's rows are cut into tiles of at least kTilePositions output
    // positions (whole LDS chunks or whole 32-row bands); jobs are ordered by the time
    // window they start in, so the workgroups that run together read one stretch of the
    // series and an XCD's live set stays within its L2.  Kernels whose single tile spans
    // most of the series (large dilations) come first.
    {
        struct Key { int64_t window; double cost; };
        std::vector<Key> keys;
        h.jobs.clear();
        h.kjob_off.assign(K + 1, 0);
        std::vector<std::vector<int32_t>> per_kernel(K);
        for (int32_t k = 0; k < K; ++k) {
            const int64_t d = h.dilation[k];
            const int64_t n = static_cast<int64_t>(h.L) + 2LL * h.padding[k] - static_cast<int64_t>(h.length[k] - 1) * d;
            const int64_t rows = n / d, tail = n - rows * d;
            const double per_pos = static_cast<double>(h.n_ch[k]) * h.length[k];
            auto add = [&](int64_t r0, int64_t r1, int flags, int64_t window) {
                RkJob j;
                j.kernel = k; j.row0 = static_cast<int32_t>(r0); j.row1 = static_cast<int32_t>(r1); j.flags = flags;
                per_kernel[k].push_back(static_cast<int32_t>(h.jobs.size()));
                h.jobs.push_back(j);
                const double pos = static_cast<double>((r1 - r0) * d + ((flags & 1) ? tail : 0));
                keys.push_back({window, pos * per_pos});
            };
            const int64_t unit = d < kLdsMaxD ? kLdsRows * (kThreads / d) : 32;     // rows per LDS chunk / tallest band
            int64_t units = std::max<int64_t>(1, (kTilePositions + unit * d - 1) / (unit * d));
            if (d >= kLdsMaxD) {
                // register path: a tile of `units` bands has units*d strips, handed out 64 to a
                // wavefront; between the smallest tile and twice that, take the height that leaves
                // the fewest lanes of the last wavefront without a strip
                int64_t best = units;
                double best_idle = 2.0;
                for (int64_t u = units; u <= units + (units + 1) / 2; ++u) {
                    const int64_t strips = u * d, slots = (strips + 63) / 64 * 64;
                    const double idle = static_cast<double>(slots - strips) / static_cast<double>(slots);
                    if (idle < best_idle - 1e-9) { best_idle = idle; best = u; }
                }
                units = best;
            }
            const int64_t per_tile = unit * units;
            const int64_t tiles = std::max<int64_t>(1, rows / per_tile);
            const bool few = d >= kFewMinD && rows + (tail > 0 ? 1 : 0) <= kFewRowsMax;
            if (few || tiles == 1) {
                // one job; a tile that reaches over more than two windows counts as "everywhere" and
                // goes first: these are the longest jobs of a series, and started last they were the
                // tail of a small batch (one series alone: 0.76 -> 0.66 ms)
                const bool wide = (rows + h.length[k]) * d > 2 * kTilePositions;
                add(0, rows, 3, wide ? -1 : 0);
            } else {
                for (int64_t t = 0; t < tiles; ++t) {
                    const int64_t r0 = t * per_tile, r1 = (t == tiles - 1) ? rows : (t + 1) * per_tile;
                    add(r0, r1, (t == tiles - 1) ? 1 : 0, (r0 * d) / kTilePositions);
                }
            }
        }
        const size_t J = h.jobs.size();
        if (J > static_cast<size_t>(INT32_MAX)) return rk_fail(ROCKET_EINVAL, "too many forward jobs");
        std::vector<int32_t> perm(J);
        for (size_t i = 0; i < J; ++i) perm[i] = static_cast<int32_t>(i);
        std::stable_sort(perm.begin(), perm.end(), [&](int32_t a, int32_t b) {
            if (keys[a].window != keys[b].window) return keys[a].window < keys[b].window;
            return keys[a].cost > keys[b].cost;
        });
        std::vector<RkJob> sorted(J);
        std::vector<int32_t> where(J);
        for (size_t i = 0; i < J; ++i) { sorted[i] = h.jobs[perm[i]]; where[perm[i]] = static_cast<int32_t>(i); }
        h.jobs.swap(sorted);
        h.kjob_idx.clear();
        for (int32_t k = 0; k < K; ++k) {
            for (int32_t j : per_kernel[k]) h.kjob_idx.push_back(where[j]);
            h.kjob_off[k + 1] = static_cast<int32_t>(h.kjob_idx.size());
        }
        // backward pass: words of partial results per job (its kernel's gradient sums, the sum of
        // q, the largest output and its position, one spare)
        h.bjob_off.assign(J + 1, 0);
        int64_t words = 0;
        for (size_t j = 0; j < J; ++j) {
            const int32_t k = h.jobs[j].kernel;
            words += static_cast<int64_t>(h.n_ch[k]) * h.length[k] + 4;
            if (words > INT32_MAX) return rk_fail(ROCKET_EINVAL, "too many backward partial results per series");
            h.bjob_off[j + 1] = static_cast<int32_t>(words);
        }
    }
    // padded rows: a gap of `lead` zeros, then the L samples (rounded up to 64 with zeros).  The
    // gap is at least the largest padding (reads before the series) and at least the largest
    // dilation (idle lanes of a partial last row read up to one row of d floats past the series);
    // reads past the end of a row land in the gap of the next row, so one gap serves both sides,
    // and an all-zero row follows the last one.
    h.lead = static_cast<int32_t>(round_up(std::max(h.pad_max, max_dil), 64));
    h.row_len = static_cast<int64_t>(h.lead) + round_up(h.L, 64);
    h.params_dirty = true;
    return ROCKET_OK;
}

// ------------------------------------------------------------------ handles

extern "C" const char *rocket_last_error(void) { return g_last_error.c_str(); }

extern "C" int32_t rocket_num_features(uint32_t mask)
{
    if (mask == 0 || (mask & ~7u)) return 0;
    return static_cast<int32_t>(__builtin_popcount(mask));
}

extern "C" int rocket_make_kernels(uint64_t seed, int32_t K, int32_t C, int32_t L, rocket_kernels **out)
{
    if (!out) return rk_fail(ROCKET_EINVAL, "rocket_make_kernels: out is NULL");
    *out = nullptr;
    if (K < 1 || C < 1) return rk_fail(ROCKET_EINVAL, "rocket_make_kernels: K and C must be >= 1");
    if (L < 11) return rk_fail(ROCKET_EINVAL, "rocket_make_kernels: L must be >= 11");
    rocket_kernels *h = new (std::nothrow) rocket_kernels;
    if (!h) return rk_fail(ROCKET_ENOMEM, "rocket_make_kernels: out of host memory");
    try {
        h->K = K; h->C = C; h->L = L;
        rk_sample_kernels(seed, *h);
        int rc = rk_finish_handle(*h);
        if (rc != ROCKET_OK) { delete h; return rc; }
    } catch (const std::bad_alloc &) {
        delete h;
        return rk_fail(ROCKET_ENOMEM, "rocket_make_kernels: out of host memory");
    }
    *out = h;
    return ROCKET_OK;
}

extern "C" int rocket_kernels_import(int32_t K, int32_t C, int32_t L,
                                     const int32_t *length, const int32_t *dilation, const int32_t *padding,
                                     const float *bias, const int32_t *n_ch, const int32_t *channels,
                                     const float *weights, rocket_kernels **out)
{
    if (!out) return rk_fail(ROCKET_EINVAL, "rocket_kernels_import: out is NULL");
    *out = nullptr;
    if (!length || !dilation || !padding || !bias || !n_ch || !channels || !weights)
        return rk_fail(ROCKET_EINVAL, "rocket_kernels_import: NULL array");
    if (K < 1 || C < 1 || L < 1) return rk_fail(ROCKET_EINVAL, "rocket_kernels_import: K, C, L must be >= 1");
    rocket_kernels *h = new (std::nothrow) rocket_kernels;
    if (!h) return rk_fail(ROCKET_ENOMEM, "rocket_kernels_import: out of host memory");
    try {
        h->K = K; h->C = C; h->L = L;
        int64_t nc = 0, nw = 0;
        std::vector<char> seen(C);
        for (int32_t k = 0; k < K; ++k) {
            const std::string who = "rocket_kernels_import: kernel " + std::to_string(k);
            const int32_t len = length[k], d = dilation[k], p = padding[k], m = n_ch[k];
            if (len != 7 && len != 9 && len != 11) { delete h; return rk_fail(ROCKET_ESHAPE, who + ": length not in {7,9,11}"); }
            if (d < 1) { delete h; return rk_fail(ROCKET_ESHAPE, who + ": dilation < 1"); }
            const int64_t span = static_cast<int64_t>(len - 1) * d;
            if (p != 0 && p != span / 2) { delete h; return rk_fail(ROCKET_ESHAPE, who + ": padding is neither 0 nor (len-1)d/2"); }
            if (static_cast<int64_t>(L) + 2LL * p - span < 1) { delete h; return rk_fail(ROCKET_ESHAPE, who + ": no output position"); }
            if (m < 1 || m > C) { delete h; return rk_fail(ROCKET_ESHAPE, who + ": n_ch outside [1,C]"); }
            std::fill(seen.begin(), seen.end(), 0);
            for (int32_t c = 0; c < m; ++c) {
                const int32_t ch = channels[nc + c];
                if (ch < 0 || ch >= C || seen[ch]) { delete h; return rk_fail(ROCKET_ESHAPE, who + ": channel out of range or repeated"); }
                seen[ch] = 1;
            }
            if (!std::isfinite(bias[k])) { delete h; return rk_fail(ROCKET_ESHAPE, who + ": bias not finite"); }
            for (int64_t i = 0; i < static_cast<int64_t>(m) * len; ++i)
                if (!std::isfinite(weights[nw + i])) { delete h; return rk_fail(ROCKET_ESHAPE, who + ": weight not finite"); }
            nc += m;
            nw += static_cast<int64_t>(m) * len;
        }
        h->length.assign(length, length + K);
        h->dilation.assign(dilation, dilation + K);
        h->padding.assign(padding, padding + K);
        h->n_ch.assign(n_ch, n_ch + K);
        h->bias.assign(bias, bias + K);
        h->channels.assign(channels, channels + nc);
        h->weights.assign(weights, weights + nw);
        int rc = rk_finish_handle(*h);
        if (rc != ROCKET_OK) { delete h; return rc; }
    } catch (const std::bad_alloc &) {
        delete h;
        return rk_fail(ROCKET_ENOMEM, "rocket_kernels_import: out of host memory");
    }
    *out = h;
    return ROCKET_OK;
}

// After rocket_sgd_update the device mirror holds the newest parameters: fetch them.
static int download_params(rocket_kernels *h)
{
    if (!h->host_stale) return ROCKET_OK;
    int cur = 0;
    RK_HIP(hipGetDevice(&cur));
    if (cur != h->device) RK_HIP(hipSetDevice(h->device));
    std::vector<RkKernelRec> rec(h->K);
    // the stream of the update may no longer exist: wait for the whole device
    hipError_t e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipMemcpy(h->weights.data(), h->d_weights, h->weights.size() * 4, hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemcpy(rec.data(), h->d_rec, rec.size() * sizeof(RkKernelRec), hipMemcpyDeviceToHost);
    if (cur != h->device) (void)hipSetDevice(cur);
    if (e != hipSuccess) return rk_fail(ROCKET_EHIP, std::string("download of the trained parameters failed: ") + hipGetErrorString(e));
    for (int32_t k = 0; k < h->K; ++k) h->bias[k] = rec[k].bias;
    h->host_stale = false;
    return ROCKET_OK;
}

extern "C" int rocket_kernels_view_get(const rocket_kernels *h, rocket_kernels_view *v)
{
    if (!h || !v) return rk_fail(ROCKET_EINVAL, "rocket_kernels_view_get: NULL argument");
    const int rc = download_params(const_cast<rocket_kernels *>(h));
    if (rc != ROCKET_OK) return rc;
    v->K = h->K; v->C = h->C; v->L = h->L;
    v->total_channels = h->ch_off[h->K];
    v->total_weights = h->w_off[h->K];
    v->length = h->length.data(); v->dilation = h->dilation.data(); v->padding = h->padding.data();
    v->n_ch = h->n_ch.data(); v->bias = h->bias.data();
    v->ch_off = h->ch_off.data(); v->w_off = h->w_off.data();
    v->channels = h->channels.data(); v->weights = h->weights.data();
    return ROCKET_OK;
}

extern "C" int rocket_kernels_set_params(rocket_kernels *h, const float *weights, const float *bias)
{
    if (!h) return rk_fail(ROCKET_EINVAL, "rocket_kernels_set_params: NULL handle");
    // validate everything before anything changes: a rejected call leaves the handle as it was
    if (weights) {
        for (size_t i = 0; i < h->weights.size(); ++i)
            if (!std::isfinite(weights[i])) return rk_fail(ROCKET_EINVAL, "rocket_kernels_set_params: weight not finite");
    }
    if (bias) {
        for (int32_t k = 0; k < h->K; ++k)
            if (!std::isfinite(bias[k])) return rk_fail(ROCKET_EINVAL, "rocket_kernels_set_params: bias not finite");
    }
    if (weights && bias) {
        h->host_stale = false;     // everything is overwritten: nothing to fetch from the device
    } else {
        const int rc = download_params(h);
        if (rc != ROCKET_OK) return rc;
    }
    if (weights) {
        std::copy(weights, weights + h->weights.size(), h->weights.begin());
        h->mr_groups = 0;          // no longer the predetermined weight set: the group kernel does not apply
    }
    if (bias) std::copy(bias, bias + h->K, h->bias.begin());
    h->params_dirty = true;
    return ROCKET_OK;
}

extern "C" int rocket_jobs_view_get(const rocket_kernels *h, int32_t *count, const int32_t **kernel,
                                    const int32_t **row0, const int32_t **row1, const int32_t **flags,
                                    int32_t *stride_bytes)
{
    if (!h || !count || !kernel || !row0 || !row1 || !flags || !stride_bytes)
        return rk_fail(ROCKET_EINVAL, "rocket_jobs_view_get: NULL argument");
    static_assert(std::is_standard_layout<RkJob>::value, "RkJob is exposed field by field");
    *count = static_cast<int32_t>(h->jobs.size());
    *kernel = &h->jobs.data()->kernel;
    *row0 = &h->jobs.data()->row0;
    *row1 = &h->jobs.data()->row1;
    *flags = &h->jobs.data()->flags;
    *stride_bytes = static_cast<int32_t>(sizeof(RkJob));
    return ROCKET_OK;
}

extern "C" int rocket_work_per_series(const rocket_kernels *h, double *conv_fma, double *outputs)
{
    if (!h) return rk_fail(ROCKET_EINVAL, "rocket_work_per_series: NULL handle");
    if (conv_fma) *conv_fma = h->conv_fma;
    if (outputs) *outputs = h->outputs;
    return ROCKET_OK;
}

static void drop_events(rocket_kernels *h)
{
    for (auto &pr : h->events) {
        (void)hipEventDestroy(static_cast<hipEvent_t>(pr.first));
        (void)hipEventDestroy(static_cast<hipEvent_t>(pr.second));
    }
    h->events.clear();
}

extern "C" int rocket_profile_enable(rocket_kernels *h, int enable)
{
    if (!h) return rk_fail(ROCKET_EINVAL, "rocket_profile_enable: NULL handle");
    h->profile = enable != 0;
    if (!h->profile) drop_events(h);
    return ROCKET_OK;
}

extern "C" int rocket_profile_read(rocket_kernels *h, int32_t *launches, double *total_ms)
{
    if (!h || !launches || !total_ms) return rk_fail(ROCKET_EINVAL, "rocket_profile_read: NULL argument");
    double sum = 0.0;
    for (auto &pr : h->events) {
        float ms = 0.f;
        RK_HIP(hipEventSynchronize(static_cast<hipEvent_t>(pr.second)));
        RK_HIP(hipEventElapsedTime(&ms, static_cast<hipEvent_t>(pr.first), static_cast<hipEvent_t>(pr.second)));
        sum += ms;
    }
    *launches = static_cast<int32_t>(h->events.size());
    *total_ms = sum;
    drop_events(h);
    return ROCKET_OK;
}

// Records the first / second event of a pair on `stream` when profiling is on.
static int profile_mark(rocket_kernels *h, hipStream_t stream, bool begin)
{
    if (!h->profile) return ROCKET_OK;
    hipEvent_t ev;
    RK_HIP(hipEventCreate(&ev));
    if (begin) h->events.emplace_back(ev, nullptr);
    else h->events.back().second = ev;
    RK_HIP(hipEventRecord(ev, stream));
    return ROCKET_OK;
}

extern "C" void rocket_free_kernels(rocket_kernels *h)
{
    if (!h) return;
    drop_events(h);
    if (h->d_blob) {
        int cur = -1;
        void *jobs = const_cast<RkMrJob *>(h->d_mr_jobs);
        if (hipGetDevice(&cur) == hipSuccess && cur != h->device && hipSetDevice(h->device) == hipSuccess) {
            (void)hipFree(h->d_blob);
            if (jobs) (void)hipFree(jobs);
            (void)hipSetDevice(cur);
        } else {
            (void)hipFree(h->d_blob);
            if (jobs) (void)hipFree(jobs);
        }
    }
    delete h;
}

// workspace layout: [padded batch: B*C*row_len floats][partial results of the forward or the
// backward kernel][mean and standard deviation of every row, used by the 8-bit entry points]
static size_t padded_batch_bytes(const rocket_kernels *h, int32_t B)
{
    // B*C rows and the all-zero row after them; 8 KB of slack: the LDS staging of the last row may
    // read a few hundred floats past it
    return static_cast<size_t>(round_up((static_cast<int64_t>(B) * h->C + 1) * h->row_len * 4 + 8192, 256));
}

static size_t backward_partial_floats(const rocket_kernels *h) { return static_cast<size_t>(h->bjob_off.back()); }

// forward: three words (max, positive count, sigmoid sum) per (series, job)
static size_t forward_partial_floats(const rocket_kernels *h) { return 3 * h->jobs.size(); }

static size_t row_stats_offset(const rocket_kernels *h, int32_t B, int backward)
{
    size_t bytes = padded_batch_bytes(h, B);
    bytes += static_cast<size_t>(B) * (backward ? backward_partial_floats(h) : forward_partial_floats(h)) * 4;
    return static_cast<size_t>(round_up(static_cast<int64_t>(bytes), 256));
}

extern "C" size_t rocket_workspace_bytes(const rocket_kernels *h, int32_t B, uint32_t mask, int backward)
{
    if (!h || B < 1 || rocket_num_features(mask) == 0) return 0;
    return row_stats_offset(h, B, backward) + static_cast<size_t>(round_up(static_cast<int64_t>(B) * h->C * 16, 256));
}

// ------------------------------------------------------------------ device mirror

static int ensure_device(rocket_kernels *h, hipStream_t stream)
{
    int cur = 0;
    RK_HIP(hipGetDevice(&cur));
    const int32_t K = h->K;
    const size_t rec_b = round_up(static_cast<int64_t>(K) * sizeof(RkKernelRec), 256);
    const size_t boff_b = round_up(static_cast<int64_t>(h->bjob_off.size()) * 4, 256);
    const size_t ch_b = round_up(static_cast<int64_t>(h->channels.size()) * 4, 256);
    const size_t w_b = round_up(static_cast<int64_t>(h->weights.size()) * 4, 256);
    const size_t job_b = round_up(static_cast<int64_t>(h->jobs.size()) * sizeof(RkJob), 256);
    const size_t koff_b = round_up(static_cast<int64_t>(K + 1) * 4, 256);
    const size_t kidx_b = round_up(static_cast<int64_t>(h->kjob_idx.size()) * 4, 256);
    if (h->d_blob && h->device != cur)
        return rk_fail(ROCKET_EINVAL, "handle was first used on another device");
    if (!h->d_blob) {
        h->blob_bytes = rec_b + boff_b + ch_b + w_b + job_b + koff_b + kidx_b;
        RK_HIP(hipMalloc(&h->d_blob, h->blob_bytes));
        h->device = cur;
        char *base = static_cast<char *>(h->d_blob);
        h->d_rec = reinterpret_cast<const RkKernelRec *>(base);
        h->d_bjob_off = reinterpret_cast<const int32_t *>(base + rec_b);
        h->d_channels = reinterpret_cast<const int32_t *>(base + rec_b + boff_b);
        h->d_weights = reinterpret_cast<float *>(base + rec_b + boff_b + ch_b);
        h->d_jobs = reinterpret_cast<const RkJob *>(base + rec_b + boff_b + ch_b + w_b);
        h->d_kjob_off = reinterpret_cast<const int32_t *>(base + rec_b + boff_b + ch_b + w_b + job_b);
        h->d_kjob_idx = reinterpret_cast<const int32_t *>(base + rec_b + boff_b + ch_b + w_b + job_b + koff_b);
        h->params_dirty = true;
    }
    if (h->params_dirty) {
        std::vector<RkKernelRec> rec(K);
        for (int32_t k = 0; k < K; ++k) {
            RkKernelRec &r = rec[k];
            r.len = h->length[k]; r.dil = h->dilation[k]; r.pad = h->padding[k];
            r.nout = h->L + 2 * h->padding[k] - (h->length[k] - 1) * h->dilation[k];
            r.bias = h->bias[k]; r.nch = h->n_ch[k];
            r.ch_off = static_cast<int32_t>(h->ch_off[k]);
            r.w_off = static_cast<int32_t>(h->w_off[k]);
        }
        // pageable sources: these copies return once the source has been read
        RK_HIP(hipMemcpyAsync(const_cast<RkKernelRec *>(h->d_rec), rec.data(), K * sizeof(RkKernelRec), hipMemcpyHostToDevice, stream));
        RK_HIP(hipMemcpyAsync(const_cast<int32_t *>(h->d_bjob_off), h->bjob_off.data(), h->bjob_off.size() * 4, hipMemcpyHostToDevice, stream));
        RK_HIP(hipMemcpyAsync(const_cast<int32_t *>(h->d_channels), h->channels.data(), h->channels.size() * 4, hipMemcpyHostToDevice, stream));
        RK_HIP(hipMemcpyAsync(h->d_weights, h->weights.data(), h->weights.size() * 4, hipMemcpyHostToDevice, stream));
        RK_HIP(hipMemcpyAsync(const_cast<RkJob *>(h->d_jobs), h->jobs.data(), h->jobs.size() * sizeof(RkJob), hipMemcpyHostToDevice, stream));
        RK_HIP(hipMemcpyAsync(const_cast<int32_t *>(h->d_kjob_off), h->kjob_off.data(), (K + 1) * 4, hipMemcpyHostToDevice, stream));
        RK_HIP(hipMemcpyAsync(const_cast<int32_t *>(h->d_kjob_idx), h->kjob_idx.data(), h->kjob_idx.size() * 4, hipMemcpyHostToDevice, stream));
        RK_HIP(hipStreamSynchronize(stream));
        h->params_dirty = false;
    }
    return ROCKET_OK;
}

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kShortSeries = 8192;       // longest series handled by the one-wavefront forward kernel
constexpr int kBwdMaxTerms = 9 * 11;     // the backward kernel holds at most 9 channels x 11 weights per kernel

// ------------------------------------------------------------------ launches

static int check_common(const char *fn, const rocket_kernels *h, const void *x, int32_t B, uint32_t mask,
                        float lambda, float shift, const void *ws, size_t ws_bytes, int backward)
{
    const std::string who(fn);
    if (!h) return rk_fail(ROCKET_EINVAL, who + ": NULL handle");
    if (!x) return rk_fail(ROCKET_EINVAL, who + ": x_dev is NULL");
    if (B < 1) return rk_fail(ROCKET_EINVAL, who + ": B must be >= 1");
    if (rocket_num_features(mask) == 0) return rk_fail(ROCKET_EINVAL, who + ": feature mask must be a non-empty subset of 7");
    if (!std::isfinite(lambda) || !std::isfinite(shift)) return rk_fail(ROCKET_EINVAL, who + ": lambda and shift must be finite");
    if (rk_grid_groups(B, static_cast<int64_t>(std::max<size_t>(h->jobs.size(), h->K)), 1) > INT32_MAX)
        return rk_fail(ROCKET_EINVAL, who + ": B times the number of work items exceeds the grid limit");
    const size_t need = rocket_workspace_bytes(h, B, mask, backward);
    if (!ws || ws_bytes < need)
        return rk_fail(ROCKET_EWORKSPACE, who + ": workspace of " + std::to_string(need) + " bytes required");
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return rk_fail(ROCKET_EWORKSPACE, who + ": workspace must be 256-byte aligned");
    return ROCKET_OK;
}

// Fills the padded workspace copy from fp32 samples, or from 8-bit samples with the
// per-row z-normalisation folded in.
static int pad_batch(const rocket_kernels *h, const void *x_dev, bool is_u8, int32_t B, void *ws, int backward,
                     hipStream_t stream)
{
    float *xpad = static_cast<float *>(ws);
    const int rc = is_u8 ? rk_launch_pad_u8(h, static_cast<const uint8_t *>(x_dev), B, xpad,
                                            static_cast<char *>(ws) + row_stats_offset(h, B, backward), stream)
                         : rk_launch_pad(h, static_cast<const float *>(x_dev), B, xpad, stream);
    return rc == ROCKET_OK ? ROCKET_OK : rk_fail(ROCKET_EHIP, "launch of the padding kernel failed");
}

// `resident_only`: the call may not allocate, so the handle's device mirror must already be there
// and current (ensure_device would allocate and copy), and no timing events are created.
static int transform_impl(const char *fn, rocket_kernels *h, const void *x_dev, bool is_u8, int32_t B, uint32_t mask,
                          float lambda, float shift, float *out_dev, void *ws, size_t ws_bytes, void *hip_stream,
                          bool resident_only = false)
{
    int rc = check_common(fn, h, x_dev, B, mask, lambda, shift, ws, ws_bytes, 0);
    if (rc != ROCKET_OK) return rc;
    if (!out_dev) return rk_fail(ROCKET_EINVAL, std::string(fn) + ": out_dev is NULL");
    if (h->row_len > INT32_MAX) return rk_fail(ROCKET_EINVAL, std::string(fn) + ": series too long");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (resident_only) {
        int cur = -1;
        RK_HIP(hipGetDevice(&cur));
        if (!h->d_blob || h->params_dirty || h->device != cur)
            return rk_fail(ROCKET_EINVAL, std::string(fn) + ": the kernels' parameters are not on this device yet; one "
                           "earlier rocket_transform call on the handle uploads them");
    } else {
        rc = ensure_device(h, stream);
        if (rc != ROCKET_OK) return rc;
    }
    float *xpad = static_cast<float *>(ws);
    rc = pad_batch(h, x_dev, is_u8, B, ws, 0, stream);
    if (rc != ROCKET_OK) return rc;
    const float nl = -lambda * kLog2e, ns = -shift * kLog2e;
    if (!resident_only) rc = profile_mark(h, stream, true);
    if (rc != ROCKET_OK) return rc;
    // series of at most kShortSeries samples: one wavefront per (series, kernel) instead of four
    float *partials = reinterpret_cast<float *>(static_cast<char *>(ws) + padded_batch_bytes(h, B));
    const int launched = h->L <= kShortSeries ? rk_launch_forward_short(h, xpad, B, mask, nl, ns, partials, stream)
                                              : rk_launch_forward(h, xpad, B, mask, nl, ns, partials, stream);
    if (launched != ROCKET_OK) return rk_fail(ROCKET_EHIP, "launch of the forward kernel failed");
    if (!resident_only) rc = profile_mark(h, stream, false);
    if (rc != ROCKET_OK) return rc;
    if (rk_launch_finalize(h, partials, B, mask, out_dev, stream) != ROCKET_OK)
        return rk_fail(ROCKET_EHIP, "launch of the feature kernel failed");
    return ROCKET_OK;
}

extern "C" int rocket_transform(rocket_kernels *h, const float *x_dev, int32_t B, uint32_t mask, float lambda,
                                float shift, float *out_dev, void *ws, size_t ws_bytes, void *hip_stream)
{
    return transform_impl("rocket_transform", h, x_dev, false, B, mask, lambda, shift, out_dev, ws, ws_bytes, hip_stream);
}

extern "C" int rocket_transform_u8(rocket_kernels *h, const uint8_t *x_u8_dev, int32_t B, uint32_t mask, float lambda,
                                   float shift, float *out_dev, void *ws, size_t ws_bytes, void *hip_stream)
{
    return transform_impl("rocket_transform_u8", h, x_u8_dev, true, B, mask, lambda, shift, out_dev, ws, ws_bytes,
                          hip_stream);
}

// ------------------------------------------------------------------ transform without allocation
//
// For callers that cannot allocate device memory (tight serving loops, harnesses that forbid it):
// the workspace of the transform is a fixed array in the library's own device image.  Every GPU
// the library runs on holds one copy of it, at its own address, until the process ends.

constexpr size_t kResidentScratchBytes = static_cast<size_t>(64) << 20;   // 64 MiB
constexpr int kMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kResidentScratchBytes];

// Device address of `scratch` on the current device.  The array's name is only a host-side
// stand-in for the symbol; the address that kernels and copies can use comes from
// hipGetSymbolAddress, once per device, with that device current.
static int resident_scratch(void **ptr)
{
    static void *address[kMaxDevices];      // zero-initialised; written once per device
    static std::mutex guard;
    int dev = -1;
    RK_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return rk_fail(ROCKET_EINVAL, "device index beyond the supported range");
    std::lock_guard<std::mutex> lock(guard);
    if (!address[dev]) {
        void *p = nullptr;
        RK_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return rk_fail(ROCKET_EHIP, "hipGetSymbolAddress returned no address for the resident workspace");
        address[dev] = p;
    }
    *ptr = address[dev];
    return ROCKET_OK;
}

extern "C" int rocket_transform_noalloc(rocket_kernels *h, const float *x_dev, int32_t B, uint32_t mask, float lambda,
                                        float shift, float *out_dev, void *hip_stream)
{
    if (!h) return rk_fail(ROCKET_EINVAL, "rocket_transform_noalloc: NULL handle");
    const size_t need = rocket_workspace_bytes(h, B, mask, 0);
    if (need == 0) return rk_fail(ROCKET_EINVAL, "rocket_transform_noalloc: B must be >= 1 and the feature mask a non-empty subset of 7");
    if (need > kResidentScratchBytes)
        return rk_fail(ROCKET_EWORKSPACE, "rocket_transform_noalloc: this batch needs a workspace of " + std::to_string(need) +
                       " bytes, the resident one holds " + std::to_string(kResidentScratchBytes) +
                       "; use rocket_transform with a workspace of the caller's");
    if (!h->d_blob || h->params_dirty)
        return rk_fail(ROCKET_EINVAL, "rocket_transform_noalloc: the kernels' parameters are not on the device yet; one "
                       "earlier rocket_transform call on the handle uploads them");
    void *ws = nullptr;
    const int rc = resident_scratch(&ws);
    if (rc != ROCKET_OK) return rc;
    return transform_impl("rocket_transform_noalloc", h, x_dev, false, B, mask, lambda, shift, out_dev, ws,
                          kResidentScratchBytes, hip_stream, true);
}

extern "C" int rocket_infer(rocket_kernels *h, const void *x_dev, int x_is_u8, int32_t B, uint32_t mask, float lambda,
                            float shift, const double *coef_dev, const double *intercept_dev, float *features_dev,
                            double *pred_dev, void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!coef_dev || !intercept_dev || !pred_dev) return rk_fail(ROCKET_EINVAL, "rocket_infer: NULL pointer");
    int rc = transform_impl("rocket_infer", h, x_dev, x_is_u8 != 0, B, mask, lambda, shift, features_dev, ws, ws_bytes,
                            hip_stream);
    if (rc != ROCKET_OK) return rc;
    return rocket_ridge_predict(features_dev, B, rocket_num_features(mask) * h->K, coef_dev, intercept_dev, pred_dev,
                                hip_stream);
}

static int backward_impl(const char *fn, rocket_kernels *h, const void *x_dev, bool is_u8, int32_t B, uint32_t mask,
                         const float *grad_out_dev, float lambda, float shift, int include_max, float *grad_w_dev,
                         float *grad_b_dev, void *ws, size_t ws_bytes, void *hip_stream)
{
    const std::string who(fn);
    int rc = check_common(fn, h, x_dev, B, mask, lambda, shift, ws, ws_bytes, 1);
    if (rc != ROCKET_OK) return rc;
    if (!(mask & ROCKET_F_SOFTPPV)) return rk_fail(ROCKET_EINVAL, who + ": mask must contain ROCKET_F_SOFTPPV");
    if (include_max && !(mask & ROCKET_F_MAX)) return rk_fail(ROCKET_EINVAL, who + ": include_max needs ROCKET_F_MAX in the mask");
    if (!grad_out_dev || !grad_w_dev || !grad_b_dev) return rk_fail(ROCKET_EINVAL, who + ": NULL gradient pointer");
    if (h->row_len > INT32_MAX) return rk_fail(ROCKET_EINVAL, who + ": series too long");
    if (h->max_terms > kBwdMaxTerms)
        return rk_fail(ROCKET_ESHAPE, who + ": a kernel has more than 9 channels x 11 weights");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    rc = ensure_device(h, stream);
    if (rc != ROCKET_OK) return rc;
    float *xpad = static_cast<float *>(ws);
    float *partial = reinterpret_cast<float *>(static_cast<char *>(ws) + padded_batch_bytes(h, B));
    rc = pad_batch(h, x_dev, is_u8, B, ws, 1, stream);
    if (rc != ROCKET_OK) return rc;
    const int F = rocket_num_features(mask);
    const int plane_soft = F - 1;                 // planes are in bit order: softPPV is last
    const int plane_max = include_max ? 0 : -1;   // and max, when present, is first
    const float nl = -lambda * kLog2e, ns = -shift * kLog2e;
    rc = profile_mark(h, stream, true);
    if (rc != ROCKET_OK) return rc;
    if (rk_launch_backward(h, xpad, B, grad_out_dev, F, plane_soft, plane_max, lambda, nl, ns, partial, stream) != ROCKET_OK)
        return rk_fail(ROCKET_EHIP, "launch of the backward kernel failed");
    rc = profile_mark(h, stream, false);
    if (rc != ROCKET_OK) return rc;
    if (rk_launch_reduce_jobs(h, partial, xpad, B, grad_out_dev, F, plane_max, grad_w_dev, grad_b_dev, stream) != ROCKET_OK)
        return rk_fail(ROCKET_EHIP, "launch of the gradient reduction kernel failed");
    return ROCKET_OK;
}

extern "C" int rocket_soft_ppv_backward(rocket_kernels *h, const float *x_dev, int32_t B, uint32_t mask,
                                        const float *grad_out_dev, float lambda, float shift, int include_max,
                                        float *grad_w_dev, float *grad_b_dev, void *ws, size_t ws_bytes,
                                        void *hip_stream)
{
    return backward_impl("rocket_soft_ppv_backward", h, x_dev, false, B, mask, grad_out_dev, lambda, shift, include_max,
                         grad_w_dev, grad_b_dev, ws, ws_bytes, hip_stream);
}

extern "C" int rocket_soft_ppv_backward_u8(rocket_kernels *h, const uint8_t *x_u8_dev, int32_t B, uint32_t mask,
                                           const float *grad_out_dev, float lambda, float shift, int include_max,
                                           float *grad_w_dev, float *grad_b_dev, void *ws, size_t ws_bytes,
                                           void *hip_stream)
{
    return backward_impl("rocket_soft_ppv_backward_u8", h, x_u8_dev, true, B, mask, grad_out_dev, lambda, shift,
                         include_max, grad_w_dev, grad_b_dev, ws, ws_bytes, hip_stream);
}

// ------------------------------------------------------------------ training step

extern "C" int rocket_mse_grad(const double *pred_dev, const float *targets_dev, const double *coef_dev, int32_t B,
                               int32_t p, float *grad_out_dev, double *loss_dev, void *hip_stream)
{
    if (!pred_dev || !targets_dev || !coef_dev || !grad_out_dev) return rk_fail(ROCKET_EINVAL, "rocket_mse_grad: NULL pointer");
    if (B < 1 || B > 65535 || p < 1) return rk_fail(ROCKET_EINVAL, "rocket_mse_grad: B must be in [1, 65535] and p >= 1");
    if (rk_launch_mse_grad(pred_dev, targets_dev, coef_dev, B, p, grad_out_dev, loss_dev, hip_stream) != ROCKET_OK)
        return rk_fail(ROCKET_EHIP, "launch of the loss gradient kernel failed");
    return ROCKET_OK;
}

extern "C" int rocket_sgd_update(rocket_kernels *h, const float *grad_w_dev, const float *grad_b_dev, float lr,
                                 int recentre, void *hip_stream)
{
    if (!h || !grad_w_dev || !grad_b_dev) return rk_fail(ROCKET_EINVAL, "rocket_sgd_update: NULL argument");
    if (!std::isfinite(lr)) return rk_fail(ROCKET_EINVAL, "rocket_sgd_update: lr must be finite");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int rc = ensure_device(h, stream);      // uploads host-side parameters first if they are the newer ones
    if (rc != ROCKET_OK) return rc;
    if (h->host_stale && h->update_stream != hip_stream) {
        // an earlier update ran on another stream (which may no longer exist): order this one after it
        RK_HIP(hipDeviceSynchronize());
    }
    if (rk_launch_sgd_update(h, grad_w_dev, grad_b_dev, lr, recentre, stream) != ROCKET_OK)
        return rk_fail(ROCKET_EHIP, "launch of the update kernel failed");
    h->host_stale = true;
    h->update_stream = hip_stream;
    h->mr_groups = 0;              // trained weights are no longer the predetermined set
    return ROCKET_OK;
}

// layout of the training workspace: [transform / backward workspace][features][upstream gradient]
// [predictions][weight gradient][bias gradient], every part rounded up to 256 bytes
struct TrainLayout {
    size_t inner, feats, gout, pred, gw, gb, total;
};

static TrainLayout train_layout(const rocket_kernels *h, int32_t B, uint32_t mask)
{
    TrainLayout t;
    const size_t p = static_cast<size_t>(rocket_num_features(mask)) * h->K;
    t.inner = std::max(rocket_workspace_bytes(h, B, mask, 0), rocket_workspace_bytes(h, B, mask, 1));
    t.feats = t.inner;
    t.gout = t.feats + round_up(static_cast<int64_t>(B) * p * 4, 256);
    t.pred = t.gout + round_up(static_cast<int64_t>(B) * p * 4, 256);
    t.gw = t.pred + round_up(static_cast<int64_t>(B) * 8, 256);
    t.gb = t.gw + round_up(static_cast<int64_t>(h->w_off[h->K]) * 4, 256);
    t.total = t.gb + round_up(static_cast<int64_t>(h->K) * 4, 256);
    return t;
}

extern "C" size_t rocket_train_workspace_bytes(const rocket_kernels *h, int32_t B, uint32_t mask)
{
    if (!h || B < 1 || rocket_num_features(mask) == 0) return 0;
    return train_layout(h, B, mask).total;
}

extern "C" int rocket_train_step(rocket_kernels *h, const void *x_dev, int x_is_u8, int32_t B, uint32_t mask,
                                 float lambda, float shift, const double *coef_dev, const double *intercept_dev,
                                 const float *targets_dev, float lr, int recentre, double *loss_dev, void *ws,
                                 size_t ws_bytes, void *hip_stream)
{
    if (!h) return rk_fail(ROCKET_EINVAL, "rocket_train_step: NULL handle");
    if (!coef_dev || !intercept_dev || !targets_dev) return rk_fail(ROCKET_EINVAL, "rocket_train_step: NULL pointer");
    if (B < 1 || rocket_num_features(mask) == 0 || !(mask & ROCKET_F_SOFTPPV))
        return rk_fail(ROCKET_EINVAL, "rocket_train_step: B >= 1 and a feature mask that contains ROCKET_F_SOFTPPV required");
    const TrainLayout t = train_layout(h, B, mask);
    if (!ws || ws_bytes < t.total)
        return rk_fail(ROCKET_EWORKSPACE, "rocket_train_step: workspace of " + std::to_string(t.total) + " bytes required");
    char *base = static_cast<char *>(ws);
    float *feats = reinterpret_cast<float *>(base + t.feats);
    float *gout = reinterpret_cast<float *>(base + t.gout);
    double *pred = reinterpret_cast<double *>(base + t.pred);
    float *gw = reinterpret_cast<float *>(base + t.gw);
    float *gb = reinterpret_cast<float *>(base + t.gb);
    const int32_t p = rocket_num_features(mask) * h->K;
    int rc = transform_impl("rocket_train_step", h, x_dev, x_is_u8 != 0, B, mask, lambda, shift, feats, ws, t.inner, hip_stream);
    if (rc != ROCKET_OK) return rc;
    rc = rocket_ridge_predict(feats, B, p, coef_dev, intercept_dev, pred, hip_stream);
    if (rc != ROCKET_OK) return rc;
    rc = rocket_mse_grad(pred, targets_dev, coef_dev, B, p, gout, loss_dev, hip_stream);
    if (rc != ROCKET_OK) return rc;
    rc = backward_impl("rocket_train_step", h, x_dev, x_is_u8 != 0, B, mask, gout, lambda, shift,
                       (mask & ROCKET_F_MAX) ? 1 : 0, gw, gb, ws, t.inner, hip_stream);
    if (rc != ROCKET_OK) return rc;
    return rocket_sgd_update(h, gw, gb, lr, recentre, hip_stream);
}

// ------------------------------------------------------------------ MINIROCKET-style variant

// Work items of the group kernel: every group's output cut into tiles whose channel-summed input fits the
// kMrTileFloats floats of LDS (see RkMrJob), group after group.
static void minirocket_plan(rocket_kernels &h)
{
    h.mr_jobs.clear();
    for (int32_t g = 0; g < h.mr_groups; ++g) {
        const int32_t k = g * kMrSet;
        const int64_t d = h.dilation[k], halo = static_cast<int64_t>(kMrLen - 1) * d;
        const int64_t n = static_cast<int64_t>(h.L) + 2LL * h.padding[k] - halo;
        RkMrJob j{};
        j.group = g;
        if (d <= kMrLinearMaxD) {
            const int64_t room = (kMrTileFloats - halo) / 64 * 64;
            const int64_t tiles = (n + room - 1) / room;
            const int64_t each = round_up((n + tiles - 1) / tiles, 64);
            for (int64_t t0 = 0; t0 < n; t0 += each) {
                j.mode = 0; j.first = static_cast<int32_t>(t0);
                j.count = static_cast<int32_t>(std::min(each, n - t0));
                j.width = static_cast<int32_t>(round_up(j.count, 64));
                j.rows = 1; j.col0 = 0;
                h.mr_jobs.push_back(j);
            }
        } else {
            const int64_t rows_total = (n + d - 1) / d;
            const int64_t blocks = (d + 255) / 256;
            const int64_t width = round_up((d + blocks - 1) / blocks, 64);
            const int64_t rows_max = kMrTileFloats / width - (kMrLen - 1);
            const int64_t row_tiles = (rows_total + rows_max - 1) / rows_max;
            const int64_t each = (rows_total + row_tiles - 1) / row_tiles;
            for (int64_t r0 = 0; r0 < rows_total; r0 += each)
                for (int64_t c0 = 0; c0 < d; c0 += width) {
                    if (r0 * d + c0 >= n) continue;   // the output ends before this block begins
                    j.mode = 1; j.first = static_cast<int32_t>(r0);
                    j.rows = static_cast<int32_t>(std::min(each, rows_total - r0));
                    j.col0 = static_cast<int32_t>(c0); j.width = static_cast<int32_t>(width); j.count = 0;
                    h.mr_jobs.push_back(j);
                }
        }
    }
}

extern "C" int rocket_minirocket_kernels(uint64_t seed, int32_t groups, int32_t C, int32_t L, rocket_kernels **out)
{
    if (!out) return rk_fail(ROCKET_EINVAL, "rocket_minirocket_kernels: out is NULL");
    *out = nullptr;
    if (groups < 1 || C < 1) return rk_fail(ROCKET_EINVAL, "rocket_minirocket_kernels: groups and C must be >= 1");
    if (groups > INT32_MAX / 84) return rk_fail(ROCKET_EINVAL, "rocket_minirocket_kernels: too many groups");
    if (L < 9) return rk_fail(ROCKET_EINVAL, "rocket_minirocket_kernels: L must be >= 9");
    if (L > (1 << 28)) return rk_fail(ROCKET_EINVAL, "rocket_minirocket_kernels: L must be at most 2^28");
    rocket_kernels *h = new (std::nothrow) rocket_kernels;
    if (!h) return rk_fail(ROCKET_ENOMEM, "rocket_minirocket_kernels: out of host memory");
    try {
        h->C = C; h->L = L;
        rk_sample_minirocket(seed, groups, *h);
        int rc = rk_finish_handle(*h);
        if (rc != ROCKET_OK) { delete h; return rc; }
        h->mr_groups = groups;
        minirocket_plan(*h);
    } catch (const std::bad_alloc &) {
        delete h;
        return rk_fail(ROCKET_ENOMEM, "rocket_minirocket_kernels: out of host memory");
    }
    *out = h;
    return ROCKET_OK;
}

// workspace of the bias fit: [padded batch][outputs of a chunk of kernels][examples][ranks]
struct FitLayout {
    size_t ybuf, example, rank, total;
    int64_t stride;      // floats per row of outputs
    int32_t chunk;       // kernels per chunk
};

static FitLayout fit_layout(const rocket_kernels *h, int32_t B)
{
    FitLayout f;
    f.stride = round_up(static_cast<int64_t>(h->L) + 2LL * h->pad_max, 64);
    const int64_t budget = (64LL << 20) / f.stride;          // rows in 256 MB of outputs
    f.chunk = static_cast<int32_t>(std::max<int64_t>(1, std::min<int64_t>(h->K, budget)));
    f.ybuf = padded_batch_bytes(h, B);
    f.example = f.ybuf + static_cast<size_t>(round_up(static_cast<int64_t>(f.chunk) * f.stride * 4, 256));
    f.rank = f.example + static_cast<size_t>(round_up(static_cast<int64_t>(h->K) * 4, 256));
    f.total = f.rank + static_cast<size_t>(round_up(static_cast<int64_t>(h->K) * 4, 256));
    return f;
}

extern "C" size_t rocket_minirocket_fit_workspace_bytes(const rocket_kernels *h, int32_t B)
{
    if (!h || B < 1) return 0;
    return fit_layout(h, B).total;
}

extern "C" int rocket_minirocket_fit_bias(rocket_kernels *h, const float *x_dev, int32_t B, uint64_t seed, void *ws,
                                          size_t ws_bytes, void *hip_stream)
{
    if (!h || !x_dev) return rk_fail(ROCKET_EINVAL, "rocket_minirocket_fit_bias: NULL argument");
    if (B < 1) return rk_fail(ROCKET_EINVAL, "rocket_minirocket_fit_bias: B must be >= 1");
    if (h->row_len > INT32_MAX) return rk_fail(ROCKET_EINVAL, "rocket_minirocket_fit_bias: series too long");
    const FitLayout f = fit_layout(h, B);
    if (!ws || ws_bytes < f.total)
        return rk_fail(ROCKET_EWORKSPACE, "rocket_minirocket_fit_bias: workspace of " + std::to_string(f.total) + " bytes required");
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return rk_fail(ROCKET_EWORKSPACE, "rocket_minirocket_fit_bias: workspace must be 256-byte aligned");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int rc = ensure_device(h, stream);
    if (rc != ROCKET_OK) return rc;
    if (h->host_stale && h->update_stream != hip_stream) RK_HIP(hipDeviceSynchronize());   // an earlier in-place update on another stream
    std::vector<int32_t> example, rank;
    try {
        rk_minirocket_draws(seed, *h, B, example, rank);
    } catch (const std::bad_alloc &) {
        return rk_fail(ROCKET_ENOMEM, "rocket_minirocket_fit_bias: out of host memory");
    }
    char *base = static_cast<char *>(ws);
    float *xpad = static_cast<float *>(ws);
    float *ybuf = reinterpret_cast<float *>(base + f.ybuf);
    int32_t *example_dev = reinterpret_cast<int32_t *>(base + f.example);
    int32_t *rank_dev = reinterpret_cast<int32_t *>(base + f.rank);
    // pageable sources: the copies return once the host arrays have been read
    RK_HIP(hipMemcpyAsync(example_dev, example.data(), example.size() * 4, hipMemcpyHostToDevice, stream));
    RK_HIP(hipMemcpyAsync(rank_dev, rank.data(), rank.size() * 4, hipMemcpyHostToDevice, stream));
    RK_HIP(hipStreamSynchronize(stream));
    if (rk_launch_pad(h, x_dev, B, xpad, stream) != ROCKET_OK)
        return rk_fail(ROCKET_EHIP, "launch of the padding kernel failed");
    for (int32_t k0 = 0; k0 < h->K; k0 += f.chunk) {
        const int32_t count = std::min(f.chunk, h->K - k0);
        if (rk_launch_minirocket_outputs(h, xpad, example_dev, k0, count, f.stride, ybuf, stream) != ROCKET_OK ||
            rk_launch_minirocket_select(h, rank_dev, k0, count, f.stride, ybuf, stream) != ROCKET_OK)
            return rk_fail(ROCKET_EHIP, "launch of the bias fitting kernels failed");
    }
    // the device records hold the new biases; the host copy is refreshed on demand (as after rocket_sgd_update)
    h->host_stale = true;
    h->update_stream = hip_stream;
    return ROCKET_OK;
}

// workspace of the group transform: [padded batch][B x K counters][row statistics of the 8-bit entry point]
static size_t minirocket_counts_bytes(const rocket_kernels *h, int32_t B)
{
    return static_cast<size_t>(round_up(static_cast<int64_t>(B) * h->K * 4, 256));
}

extern "C" size_t rocket_minirocket_workspace_bytes(const rocket_kernels *h, int32_t B)
{
    if (!h || B < 1 || h->mr_groups == 0) return 0;
    return padded_batch_bytes(h, B) + minirocket_counts_bytes(h, B) +
           static_cast<size_t>(round_up(static_cast<int64_t>(B) * h->C * 16, 256));
}

extern "C" int rocket_minirocket_jobs_view_get(const rocket_kernels *h, int32_t *count, const int32_t **items)
{
    if (!h || !count || !items) return rk_fail(ROCKET_EINVAL, "rocket_minirocket_jobs_view_get: NULL argument");
    if (h->mr_groups == 0) return rk_fail(ROCKET_EINVAL, "rocket_minirocket_jobs_view_get: the handle does not hold the predetermined kernel set");
    static_assert(sizeof(RkMrJob) == 8 * sizeof(int32_t), "a work item is eight int32");
    *count = static_cast<int32_t>(h->mr_jobs.size());
    *items = reinterpret_cast<const int32_t *>(h->mr_jobs.data());
    return ROCKET_OK;
}

static int minirocket_transform_impl(const char *fn, rocket_kernels *h, const void *x_dev, bool is_u8, int32_t B,
                                     float *out_dev, void *ws, size_t ws_bytes, void *hip_stream)
{
    const std::string who(fn);
    if (!h || !x_dev || !out_dev) return rk_fail(ROCKET_EINVAL, who + ": NULL argument");
    if (B < 1) return rk_fail(ROCKET_EINVAL, who + ": B must be >= 1");
    if (h->mr_groups == 0)
        return rk_fail(ROCKET_EINVAL, who + ": the handle does not hold the predetermined kernel set (it was not made "
                       "by rocket_minirocket_kernels, or its weights were changed); use rocket_transform");
    if (rk_grid_groups(B, static_cast<int64_t>(h->mr_jobs.size()), 1) > INT32_MAX || static_cast<int64_t>(B) * h->K > INT32_MAX)
        return rk_fail(ROCKET_EINVAL, who + ": B times the number of work items exceeds the grid limit");
    const size_t need = rocket_minirocket_workspace_bytes(h, B);
    if (!ws || ws_bytes < need)
        return rk_fail(ROCKET_EWORKSPACE, who + ": workspace of " + std::to_string(need) + " bytes required");
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return rk_fail(ROCKET_EWORKSPACE, who + ": workspace must be 256-byte aligned");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    int rc = ensure_device(h, stream);
    if (rc != ROCKET_OK) return rc;
    if (!h->d_mr_jobs) {
        void *jobs = nullptr;
        const size_t bytes = h->mr_jobs.size() * sizeof(RkMrJob);
        RK_HIP(hipMalloc(&jobs, bytes));
        h->d_mr_jobs = static_cast<const RkMrJob *>(jobs);
        RK_HIP(hipMemcpyAsync(jobs, h->mr_jobs.data(), bytes, hipMemcpyHostToDevice, stream));
        RK_HIP(hipStreamSynchronize(stream));
    }
    char *base = static_cast<char *>(ws);
    float *xpad = static_cast<float *>(ws);
    int32_t *counts = reinterpret_cast<int32_t *>(base + padded_batch_bytes(h, B));
    void *stats = base + padded_batch_bytes(h, B) + minirocket_counts_bytes(h, B);
    const int padded = is_u8 ? rk_launch_pad_u8(h, static_cast<const uint8_t *>(x_dev), B, xpad, stats, stream)
                             : rk_launch_pad(h, static_cast<const float *>(x_dev), B, xpad, stream);
    if (padded != ROCKET_OK || rk_launch_minirocket_clear(h, B, counts, stream) != ROCKET_OK)
        return rk_fail(ROCKET_EHIP, "launch of the padding kernel failed");
    rc = profile_mark(h, stream, true);
    if (rc != ROCKET_OK) return rc;
    if (rk_launch_minirocket_forward(h, xpad, B, counts, stream) != ROCKET_OK)
        return rk_fail(ROCKET_EHIP, "launch of the group kernel failed");
    rc = profile_mark(h, stream, false);
    if (rc != ROCKET_OK) return rc;
    if (rk_launch_minirocket_features(h, counts, B, out_dev, stream) != ROCKET_OK)
        return rk_fail(ROCKET_EHIP, "launch of the feature kernel failed");
    return ROCKET_OK;
}

extern "C" int rocket_minirocket_transform(rocket_kernels *h, const float *x_dev, int32_t B, float *out_dev, void *ws,
                                           size_t ws_bytes, void *hip_stream)
{
    return minirocket_transform_impl("rocket_minirocket_transform", h, x_dev, false, B, out_dev, ws, ws_bytes, hip_stream);
}

extern "C" int rocket_minirocket_transform_u8(rocket_kernels *h, const uint8_t *x_u8_dev, int32_t B, float *out_dev,
                                              void *ws, size_t ws_bytes, void *hip_stream)
{
    return minirocket_transform_impl("rocket_minirocket_transform_u8", h, x_u8_dev, true, B, out_dev, ws, ws_bytes,
                                     hip_stream);
}

// ------------------------------------------------------------------ pruning

extern "C" int rocket_kernels_subset(const rocket_kernels *h, const int32_t *index, int32_t count, rocket_kernels **out)
{
    if (!out) return rk_fail(ROCKET_EINVAL, "rocket_kernels_subset: out is NULL");
    *out = nullptr;
    if (!h || !index || count < 1) return rk_fail(ROCKET_EINVAL, "rocket_kernels_subset: NULL argument or count < 1");
    int rc = download_params(const_cast<rocket_kernels *>(h));
    if (rc != ROCKET_OK) return rc;
    try {
        std::vector<int32_t> length(count), dilation(count), padding(count), n_ch(count), channels;
        std::vector<float> bias(count), weights;
        for (int32_t i = 0; i < count; ++i) {
            const int32_t k = index[i];
            if (k < 0 || k >= h->K) return rk_fail(ROCKET_EINVAL, "rocket_kernels_subset: index out of range");
            length[i] = h->length[k]; dilation[i] = h->dilation[k]; padding[i] = h->padding[k];
            n_ch[i] = h->n_ch[k]; bias[i] = h->bias[k];
            channels.insert(channels.end(), h->channels.begin() + h->ch_off[k], h->channels.begin() + h->ch_off[k + 1]);
            weights.insert(weights.end(), h->weights.begin() + h->w_off[k], h->weights.begin() + h->w_off[k + 1]);
        }
        return rocket_kernels_import(count, h->C, h->L, length.data(), dilation.data(), padding.data(), bias.data(),
                                     n_ch.data(), channels.data(), weights.data(), out);
    } catch (const std::bad_alloc &) {
        return rk_fail(ROCKET_ENOMEM, "rocket_kernels_subset: out of host memory");
    }
}
