// ROCKET transform for MI355X (gfx950): C-ABI entry points, launch logic and
// the HIP kernels.  See include/rocket.h for the contract of every entry point.
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
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
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
    h.ch_off.assign(K + 1, 0);
    h.w_off.assign(K + 1, 0);
    h.pad_max = 0;
    h.conv_fma = 0.0;
    h.outputs = 0.0;
    h.max_terms = 0;
    int32_t max_dil = 0;
    std::vector<double> cost(K);
    for (int32_t k = 0; k < K; ++k) {
        h.ch_off[k + 1] = h.ch_off[k] + h.n_ch[k];
        h.w_off[k + 1] = h.w_off[k] + static_cast<int64_t>(h.n_ch[k]) * h.length[k];
        const int64_t n = static_cast<int64_t>(h.L) + 2LL * h.padding[k] -
                          static_cast<int64_t>(h.length[k] - 1) * h.dilation[k];
        if (n < 1) return rk_fail(ROCKET_ESHAPE, "kernel " + std::to_string(k) + " has no output position");
        h.pad_max = std::max(h.pad_max, h.padding[k]);
        max_dil = std::max(max_dil, h.dilation[k]);
        h.max_terms = std::max(h.max_terms, h.n_ch[k] * h.length[k]);
        cost[k] = static_cast<double>(n) * h.n_ch[k] * h.length[k];
        h.conv_fma += cost[k];
        h.outputs += static_cast<double>(n);
    }
    if (h.w_off[K] > INT32_MAX || h.ch_off[K] > INT32_MAX)
        return rk_fail(ROCKET_EINVAL, "too many weights for 32-bit offsets");
    // launch order: most expensive kernels first, so the last workgroups to
    // start are the cheapest and the tail of the launch is short
    h.order.resize(K);
    for (int32_t k = 0; k < K; ++k) h.order[k] = k;
    std::stable_sort(h.order.begin(), h.order.end(),
                     [&](int32_t a, int32_t b) { return cost[a] > cost[b]; });
    // padded rows: `lead` zeros, the L samples, then zeros: at least the largest padding,
    // and at least the largest dilation (idle lanes of a partial last row read up to one
    // row of d floats past the series)
    h.lead = static_cast<int32_t>(round_up(h.pad_max, 64));
    h.row_len = round_up(static_cast<int64_t>(h.lead) + h.L + std::max(h.pad_max, max_dil), 64);
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

extern "C" int rocket_kernels_view_get(const rocket_kernels *h, rocket_kernels_view *v)
{
    if (!h || !v) return rk_fail(ROCKET_EINVAL, "rocket_kernels_view_get: NULL argument");
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
    if (weights) {
        for (size_t i = 0; i < h->weights.size(); ++i)
            if (!std::isfinite(weights[i])) return rk_fail(ROCKET_EINVAL, "rocket_kernels_set_params: weight not finite");
        std::copy(weights, weights + h->weights.size(), h->weights.begin());
    }
    if (bias) {
        for (int32_t k = 0; k < h->K; ++k)
            if (!std::isfinite(bias[k])) return rk_fail(ROCKET_EINVAL, "rocket_kernels_set_params: bias not finite");
        std::copy(bias, bias + h->K, h->bias.begin());
    }
    h->params_dirty = true;
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
        if (hipGetDevice(&cur) == hipSuccess && cur != h->device && hipSetDevice(h->device) == hipSuccess) {
            (void)hipFree(h->d_blob);
            (void)hipSetDevice(cur);
        } else {
            (void)hipFree(h->d_blob);
        }
    }
    delete h;
}

// workspace layout: [padded batch: B*C*row_len floats][backward: B*(total_w + 2K) floats]
static size_t padded_batch_bytes(const rocket_kernels *h, int32_t B)
{
    // 8 KB of slack: the LDS staging of the last row may read a few hundred floats past it
    return static_cast<size_t>(round_up(static_cast<int64_t>(B) * h->C * h->row_len * 4 + 8192, 256));
}

static size_t backward_partial_floats(const rocket_kernels *h) { return static_cast<size_t>(h->w_off[h->K]) + h->K; }

extern "C" size_t rocket_workspace_bytes(const rocket_kernels *h, int32_t B, uint32_t mask, int backward)
{
    if (!h || B < 1 || rocket_num_features(mask) == 0) return 0;
    size_t bytes = padded_batch_bytes(h, B);
    if (backward) bytes += static_cast<size_t>(B) * backward_partial_floats(h) * 4;
    return bytes;
}

// ------------------------------------------------------------------ device mirror

static int ensure_device(rocket_kernels *h, hipStream_t stream)
{
    int cur = 0;
    RK_HIP(hipGetDevice(&cur));
    const int32_t K = h->K;
    const size_t rec_b = round_up(static_cast<int64_t>(K) * sizeof(RkKernelRec), 256);
    const size_t ord_b = round_up(static_cast<int64_t>(K) * 4, 256);
    const size_t ch_b = round_up(static_cast<int64_t>(h->channels.size()) * 4, 256);
    const size_t w_b = round_up(static_cast<int64_t>(h->weights.size()) * 4, 256);
    if (h->d_blob && h->device != cur)
        return rk_fail(ROCKET_EINVAL, "handle was first used on another device");
    if (!h->d_blob) {
        h->blob_bytes = rec_b + ord_b + ch_b + w_b;
        RK_HIP(hipMalloc(&h->d_blob, h->blob_bytes));
        h->device = cur;
        char *base = static_cast<char *>(h->d_blob);
        h->d_rec = reinterpret_cast<const RkKernelRec *>(base);
        h->d_order = reinterpret_cast<const int32_t *>(base + rec_b);
        h->d_channels = reinterpret_cast<const int32_t *>(base + rec_b + ord_b);
        h->d_weights = reinterpret_cast<float *>(base + rec_b + ord_b + ch_b);
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
        RK_HIP(hipMemcpyAsync(const_cast<int32_t *>(h->d_order), h->order.data(), K * 4, hipMemcpyHostToDevice, stream));
        RK_HIP(hipMemcpyAsync(const_cast<int32_t *>(h->d_channels), h->channels.data(), h->channels.size() * 4, hipMemcpyHostToDevice, stream));
        RK_HIP(hipMemcpyAsync(h->d_weights, h->weights.data(), h->weights.size() * 4, hipMemcpyHostToDevice, stream));
        RK_HIP(hipStreamSynchronize(stream));
        h->params_dirty = false;
    }
    return ROCKET_OK;
}

// ------------------------------------------------------------------ kernels

#ifndef RK_RMAX
#define RK_RMAX 32
#endif
#ifndef RK_WPE
#define RK_WPE 6
#endif
constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr float kLog2e = 1.4426950408889634f;

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

struct PoolState {
    float vmax;   // per lane
    float ssum;   // per lane
    int cnt;      // wavefront-uniform: positives seen by this wavefront
};

// Raw buffer descriptor (stride 0, 32-bit data format) over `bytes` bytes at `base`.
// Buffer loads take the address as descriptor base + scalar offset + lane offset,
// so the walk along a strip costs scalar adds only; reads past `bytes` return 0.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t rk_row_buffer(const char *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(base), 0, static_cast<int>(bytes), 0x00020000);
}

__device__ __forceinline__ float rk_load(__amdgpu_buffer_rsrc_t row, uint32_t lane_bytes, uint32_t uniform_bytes)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(row, static_cast<int>(lane_bytes),
                                                                          static_cast<int>(uniform_bytes), 0));
}

// Advances a scalar byte offset by `step` and hides the result from the optimiser, so
// the offsets of a strip's loads form one running scalar add per load instead of
// dozens of precomputed multiples that would not fit the scalar register file
// (they were spilled to vector lanes and read back once per channel).
__device__ __forceinline__ uint32_t rk_advance(uint32_t off, uint32_t step)
{
    off += step;
    asm volatile("" : "+s"(off));
    return off;
}

// Compile-time loop: f(integral_constant<int, I>) for I in [I0, N).  Every index into
// the per-lane accumulator and weight arrays below comes from such a constant, so the
// arrays always live in named registers (a run-time index would make the compiler
// address the register file indirectly).
template <int I0, int N, class F>
__device__ __forceinline__ void rk_static_for(F &&f)
{
    if constexpr (I0 < N) {
        f(std::integral_constant<int, I0>{});
        rk_static_for<I0 + 1, N>(f);
    }
}

// Input value number I of a strip feeds every output it overlaps: acc[I-j] += w[j]*x_I.
template <int LEN, int R, int I>
__device__ __forceinline__ void rk_taps(const float (&w)[LEN], float xv, float (&acc)[R])
{
    rk_static_for<0, LEN>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        constexpr int o = I - j;
        if constexpr (o >= 0 && o < R) acc[o] = fmaf(w[j], xv, acc[o]);
    });
}

// Pooling of R finished sums z = y - bias (section 3.2).  The bias is folded into
// the pooling: max(y) = max(z) + bias (added once per kernel at the end),
// y > 0 <=> z > -bias, and lambda*y + shift = lambda*z + (shift + lambda*bias).
// `mask` is uniform; ns already contains the bias term.
template <int R>
__device__ __forceinline__ void rk_pool(const float (&acc)[R], uint32_t mask, float negbias, float nl, float ns,
                                        PoolState &st)
{
    if (mask & ROCKET_F_MAX) {
#pragma unroll
        for (int i = 0; i < R; ++i) st.vmax = fmaxf(st.vmax, acc[i]);
    }
    if (mask & ROCKET_F_PPV) {   // Eq. 1-2: strict y > 0, counted per wavefront in a scalar register
#pragma unroll
        for (int i = 0; i < R; ++i) st.cnt += __builtin_popcountll(__ballot(acc[i] > negbias));
    }
    if (mask & ROCKET_F_SOFTPPV) {
#pragma unroll
        for (int i = 0; i < R; ++i) {
            // Eq. 3: 1/(1+exp(-(lambda*y+shift))) with nl = -lambda*log2(e), ns = -(shift+lambda*bias)*log2(e)
            const float e = __builtin_amdgcn_exp2f(fmaf(acc[i], nl, ns));
            st.ssum += __builtin_amdgcn_rcpf(1.f + e);
        }
    }
}

struct KernelCtx {
    const char *xk;        // padded row of channel 0 of this series, shifted by -p (bytes)
    size_t row_bytes;      // bytes per padded row
    uint32_t span_bytes;   // bytes from xk to the end of its row
    const int32_t *chans;  // this kernel's channel list
    const float *wts;      // this kernel's weights, channel-major
    int nch, d;
    int pad, L;            // the kernel's padding and the series length
    float negbias;         // -bias
    uint32_t mask;
    float nl, ns;          // softPPV: exp2(z*nl + ns) = exp(-(lambda*y + shift))
};

// Register path.  All strips of `nbands` bands of R rows x `ncols` columns starting at
// row `row0`; every lane reads its R+LEN-1 inputs straight from global memory
// (consecutive lanes read consecutive floats once d >= 64).
template <int LEN, int R>
__device__ __forceinline__ void rk_segment(const KernelCtx &k, int row0, int nbands, int ncols, PoolState &st)
{
    const int nstrips = nbands * ncols;
    const uint32_t dbytes = static_cast<uint32_t>(k.d) * 4u;
    for (int base = 0; base < nstrips; base += kThreads) {
        const int s = base + static_cast<int>(threadIdx.x);
        if (s < nstrips) {
            const int band = (nbands == 1) ? 0 : s / ncols;
            const int r = s - band * ncols;
            const uint32_t voff = static_cast<uint32_t>((row0 + band * R) * k.d + r) * 4u;
            float acc[R];
            auto channel = [&](int c) {
                const __amdgpu_buffer_rsrc_t row =
                    rk_row_buffer(k.xk + static_cast<size_t>(k.chans[c]) * k.row_bytes, k.span_bytes);
                float w[LEN];
#pragma unroll
                for (int j = 0; j < LEN; ++j) w[j] = k.wts[c * LEN + j];
                uint32_t soff = 0;
                rk_static_for<0, R + LEN - 1>([&](auto ic) {
                    constexpr int i = decltype(ic)::value;
                    rk_taps<LEN, R, i>(w, rk_load(row, voff, soff), acc);
                    soff = rk_advance(soff, dbytes);
                });
            };
#pragma unroll
            for (int i = 0; i < R; ++i) acc[i] = 0.f;
            for (int c = 0; c < k.nch; ++c) channel(c);
            rk_pool<R>(acc, k.mask, k.negbias, k.nl, k.ns, st);
        }
    }
}

// LDS path for small dilations (d < kLdsMaxD).  With d < 64 the strips of a wavefront start
// kLdsRows*d floats apart, so direct loads would touch a different cache line per
// lane group.  Instead the workgroup copies the contiguous input range of a
// chunk of bands into LDS with coalesced loads and the lanes read their strips
// from there.  Bands have kLdsRows = 17 rows: an odd row count makes the stride
// between neighbouring bands odd (times d), which spreads the strided LDS reads
// over the banks without padding.  D is a template parameter so that the LDS
// read offsets i*D*4 are immediates.
#ifndef RK_LDS_ROWS
#define RK_LDS_ROWS 17
#endif
#ifndef RK_LDS_MAXD
#define RK_LDS_MAXD 16
#endif
constexpr int kFewMinD = 256;            // few-rows path needs at least a workgroup of columns
constexpr int kLdsRows = RK_LDS_ROWS;
constexpr int kLdsMaxD = RK_LDS_MAXD;                             // dilations below this take this path
constexpr int kLdsStage = 4;                                      // staged words per lane per round
constexpr int kLdsTileWords = ((kLdsRows * kThreads + 10 * (kLdsMaxD - 1)) / (kThreads * kLdsStage) + 1) * kThreads * kLdsStage;

// Copies `nin` floats starting `chunk_bytes` into a row to the LDS tile with coalesced
// loads (rounded up to whole rounds of kThreads*kLdsStage words: the tile and the
// workspace slack are sized for that).  Barriers on both sides: nobody still reads the
// previous contents, and the new contents are visible to all lanes afterwards.
__device__ __forceinline__ void rk_stage_tile(__amdgpu_buffer_rsrc_t row, uint32_t chunk_bytes, int nin, float *tile)
{
    const int tid = static_cast<int>(threadIdx.x);
    __syncthreads();
    for (int base = 0; base < nin; base += kThreads * kLdsStage) {
        float v[kLdsStage];
#pragma unroll
        for (int u = 0; u < kLdsStage; ++u)
            v[u] = rk_load(row, static_cast<uint32_t>(tid + u * kThreads) * 4u,
                           chunk_bytes + static_cast<uint32_t>(base) * 4u);
#pragma unroll
        for (int u = 0; u < kLdsStage; ++u) tile[base + tid + u * kThreads] = v[u];
    }
    __syncthreads();
}

template <int LEN, int D>
__device__ __forceinline__ int rk_lds_bands(const KernelCtx &k, int rows, float *tile, PoolState &st)
{
    constexpr int R = kLdsRows;
    const int nb = rows / R;
    if (nb == 0) return 0;
    constexpr int G = kThreads / D;                 // bands per chunk
    const int tid = static_cast<int>(threadIdx.x);
    const int bl = tid / D;                         // lane's band inside the chunk
    const int r = tid - bl * D;                     // lane's column
    const float *mine = tile + bl * R * D + r;
    for (int band0 = 0; band0 < nb; band0 += G) {
        const int gb = min(G, nb - band0);
        const bool active = bl < gb;
        const int nin = (gb * R + LEN - 1) * D;     // input floats of this chunk
        const uint32_t chunk_bytes = static_cast<uint32_t>(band0 * R * D) * 4u;
        float acc[R];
        auto channel = [&](int c) {
            const __amdgpu_buffer_rsrc_t row =
                rk_row_buffer(k.xk + static_cast<size_t>(k.chans[c]) * k.row_bytes, k.span_bytes);
            float w[LEN];
#pragma unroll
            for (int j = 0; j < LEN; ++j) w[j] = k.wts[c * LEN + j];
            rk_stage_tile(row, chunk_bytes, nin, tile);
            if (active) {
                rk_static_for<0, R + LEN - 1>([&](auto ic) {
                    constexpr int i = decltype(ic)::value;
                    rk_taps<LEN, R, i>(w, mine[i * D], acc);
                });
            }
        };
#pragma unroll
        for (int i = 0; i < R; ++i) acc[i] = 0.f;
        for (int c = 0; c < k.nch; ++c) channel(c);
        if (active) rk_pool<R>(acc, k.mask, k.negbias, k.nl, k.ns, st);
    }
    return nb * R;
}

// Pooling of one finished sum (see rk_pool).
__device__ __forceinline__ void rk_pool1(float z, uint32_t mask, float negbias, float nl, float ns, PoolState &st)
{
    const float one[1] = {z};
    rk_pool<1>(one, mask, negbias, nl, ns, st);
}

// Few-rows path for large dilations: when the whole output has at most RM rows of d
// positions (d >= n/RM), one strip per column covers every row, so each input is
// loaded exactly once per channel, whatever the row count (the binary band
// decomposition would cut such a kernel into short strips with little reuse).
// The row count is a run-time uniform: window rows past it are skipped with scalar
// branches.  Window rows that lie entirely in the zero padding ("same" padding
// with a large dilation puts (len-1)/2 such rows on either side) are skipped too,
// loads and multiply-adds alike.  The partial last row is handled in the same
// strip and masked per lane in the pooling.
template <int LEN, int RM>
__device__ __forceinline__ void rk_few_rows(const KernelCtx &k, int rows, int tail, PoolState &st)
{
    const int nrows = rows + (tail > 0 ? 1 : 0);            // rows with at least one output
    const int prow = k.pad / k.d;                           // padding in rows: 0 or (LEN-1)/2
    const int data_rows = (k.L + k.d - 1) / k.d;            // input rows that hold samples
    const uint32_t dbytes = static_cast<uint32_t>(k.d) * 4u;
    // bit i: window row i is needed (i < nrows+LEN-1) and holds samples (0 <= i-prow < data_rows)
    uint32_t live_lo = 0, live_hi = 0;
    for (int i = 0; i < nrows + LEN - 1; ++i) {
        if (i >= prow && i - prow < data_rows) {
            if (i < 32) live_lo |= 1u << i;
            else live_hi |= 1u << (i - 32);
        }
    }
    // Tests bit i of the mask.  The mask is re-read through an opaque copy so that the
    // 30-odd tests stay single scalar bit tests instead of that many precomputed
    // (and spilled) lane masks.
    auto is_live = [&](int i) {
        uint32_t word = i < 32 ? live_lo : live_hi;
        asm volatile("" : "+s"(word));
        return ((word >> (i & 31)) & 1u) != 0;
    };
    for (int base = 0; base < k.d; base += kThreads) {      // uniform trip count
        const int r_raw = base + static_cast<int>(threadIdx.x);
        const bool lane_ok = r_raw < k.d;
        const int r = lane_ok ? r_raw : k.d - 1;            // idle lanes shadow the last column
        const uint32_t voff = static_cast<uint32_t>(r) * 4u;
        float acc[RM];
#pragma unroll
        for (int i = 0; i < RM; ++i) acc[i] = 0.f;
        for (int c = 0; c < k.nch; ++c) {
            const __amdgpu_buffer_rsrc_t row =
                rk_row_buffer(k.xk + static_cast<size_t>(k.chans[c]) * k.row_bytes, k.span_bytes);
            float w[LEN];
#pragma unroll
            for (int j = 0; j < LEN; ++j) w[j] = k.wts[c * LEN + j];
            // all loads first (so they are in flight together), then the multiply-adds
            float xv[RM + LEN - 1];
            uint32_t soff = 0;
            rk_static_for<0, RM + LEN - 1>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                if (is_live(i)) xv[i] = rk_load(row, voff, soff);
                soff = rk_advance(soff, dbytes);
            });
            rk_static_for<0, RM + LEN - 1>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                if (is_live(i)) rk_taps<LEN, RM, i>(w, xv[i], acc);
            });
        }
        // rows below `rows` are complete; row `rows` exists only in the first `tail` columns
        const int own_rows = lane_ok ? (rows + (r < tail ? 1 : 0)) : 0;
        rk_static_for<0, RM>([&](auto oc) {
            constexpr int o = decltype(oc)::value;
            int lim = nrows;
            asm volatile("" : "+s"(lim));
            if (o < lim) {                                  // uniform
                if (o < own_rows) rk_pool1(acc[o], k.mask, k.negbias, k.nl, k.ns, st);
            }
        });
    }
}

// Calls rk_lds_bands<LEN, D> for the D that equals the kernel's dilation (D < kLdsMaxD).
template <int LEN, int D>
__device__ __forceinline__ int rk_lds_dispatch(const KernelCtx &k, int rows, float *tile, PoolState &st)
{
    if constexpr (D < kLdsMaxD) {
        if (k.d == D) return rk_lds_bands<LEN, D>(k, rows, tile, st);
        return rk_lds_dispatch<LEN, D + 1>(k, rows, tile, st);
    } else {
        return 0;
    }
}

template <int LEN>
__device__ __forceinline__ void rk_forward_body(const KernelCtx &k, int nout, float *tile, PoolState &st)
{
    const int d = k.d;
    const int rows = nout / d;            // full rows of d outputs
    const int tail = nout - rows * d;     // outputs of the partial last row
    int row0 = 0;
    // every branch below is uniform per workgroup
    if (d >= kFewMinD) {
        const int nrows = rows + (tail > 0 ? 1 : 0);
        if (nrows <= 8) { rk_few_rows<LEN, 8>(k, rows, tail, st); return; }
        if (nrows <= 16) { rk_few_rows<LEN, 16>(k, rows, tail, st); return; }
        if (nrows <= 24) { rk_few_rows<LEN, 24>(k, rows, tail, st); return; }
    }
    if (d < kLdsMaxD) row0 = rk_lds_dispatch<LEN, 1>(k, rows, tile, st);
    const int left = rows - row0;         // rows for the register path
#if RK_RMAX == 32
    const int nb32 = left >> 5;
    if (nb32) { rk_segment<LEN, 32>(k, row0, nb32, d, st); row0 += nb32 << 5; }
    if (left & 16) { rk_segment<LEN, 16>(k, row0, 1, d, st); row0 += 16; }
#else
    const int nb16 = left >> 4;
    if (nb16) { rk_segment<LEN, 16>(k, row0, nb16, d, st); row0 += nb16 << 4; }
#endif
    if (left & 8) { rk_segment<LEN, 8>(k, row0, 1, d, st); row0 += 8; }
    if (left & 4) { rk_segment<LEN, 4>(k, row0, 1, d, st); row0 += 4; }
    if (left & 2) { rk_segment<LEN, 2>(k, row0, 1, d, st); row0 += 2; }
    if (left & 1) { rk_segment<LEN, 1>(k, row0, 1, d, st); row0 += 1; }
    if (tail) rk_segment<LEN, 1>(k, row0, 1, tail, st);
}

// grid: B*K workgroups; workgroup g handles series g / K and kernel order[g % K].
#if RK_WPE
__attribute__((amdgpu_waves_per_eu(RK_WPE)))
#endif
__global__ __launch_bounds__(kThreads) void rk_forward(const float *__restrict__ xpad, int row_len, int lead, int L, int C, int K,
                                                       const RkKernelRec *__restrict__ recs,
                                                       const int32_t *__restrict__ order,
                                                       const int32_t *__restrict__ channels,
                                                       const float *__restrict__ weights, uint32_t mask, float nl,
                                                       float ns, float *__restrict__ out)
{
    __shared__ float tile[kLdsTileWords];
    const int b = blockIdx.x / K;
    const int kid = order[blockIdx.x - b * K];
    const RkKernelRec rec = recs[kid];
    KernelCtx k;
    k.row_bytes = static_cast<size_t>(row_len) * 4;
    k.xk = reinterpret_cast<const char *>(xpad) + static_cast<size_t>(b) * C * k.row_bytes +
           static_cast<size_t>(lead - rec.pad) * 4;
    k.span_bytes = static_cast<uint32_t>(row_len - (lead - rec.pad)) * 4u;
    k.chans = channels + rec.ch_off;
    k.wts = weights + rec.w_off;
    k.nch = rec.nch;
    k.d = rec.dil;
    k.pad = rec.pad;
    k.L = L;
    k.negbias = -rec.bias;
    k.mask = mask;
    k.nl = nl;
    k.ns = fmaf(rec.bias, nl, ns);

    PoolState st;
    st.vmax = -INFINITY;
    st.ssum = 0.f;
    st.cnt = 0;
    if (rec.len == 7) rk_forward_body<7>(k, rec.nout, tile, st);
    else if (rec.len == 9) rk_forward_body<9>(k, rec.nout, tile, st);
    else rk_forward_body<11>(k, rec.nout, tile, st);

    // close the reductions: lanes -> wavefront (shuffles) -> workgroup (LDS)
    float vmax = st.vmax, ssum = st.ssum;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        vmax = fmaxf(vmax, __shfl_xor(vmax, off));
        ssum += __shfl_xor(ssum, off);
    }
    __shared__ float s_max[kWaves];
    __shared__ float s_sum[kWaves];
    __shared__ int s_cnt[kWaves];
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { s_max[wave] = vmax; s_sum[wave] = ssum; s_cnt[wave] = st.cnt; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float m = s_max[0], sm = s_sum[0];
        int cn = s_cnt[0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) { m = fmaxf(m, s_max[w]); sm += s_sum[w]; cn += s_cnt[w]; }
        const int F = __builtin_popcount(mask);
        float *o = out + static_cast<size_t>(b) * F * K + kid;
        int f = 0;
        if (mask & ROCKET_F_MAX) { o[static_cast<size_t>(f) * K] = m + rec.bias; ++f; }
        if (mask & ROCKET_F_PPV) { o[static_cast<size_t>(f) * K] = static_cast<float>(static_cast<double>(cn) / static_cast<double>(rec.nout)); ++f; }
        if (mask & ROCKET_F_SOFTPPV) { o[static_cast<size_t>(f) * K] = sm / static_cast<float>(rec.nout); ++f; }
    }
}

// ------------------------------------------------------------------ backward kernels
//
// Backward pass through softPPV (and, optionally, the max): one workgroup per
// (series, kernel), the same strip decomposition as the forward pass.  Per strip:
//   1. recompute the R conv outputs,
//   2. turn them into q_i = g_soft * (lambda/n) * s_i (1 - s_i),
//   3. per channel, re-read the strip's inputs and form the lane's share of
//      d/dw[c][j] = sum_i q_i * x[c][t_i + j*d - p]  (R*LEN multiply-adds), sum it over
//      each row of 16 lanes with four DPP adds, and let one lane per row add the row
//      sum to that row's own slot in LDS (16 slots per weight: 4 wavefronts x 4 rows;
//      plain read-modify-write, no atomics, nobody else touches the slot).
// Lanes without a strip recompute the last strip with a zero coefficient, so control
// flow stays wavefront-uniform around the cross-lane adds.  At the end the slots are
// summed and the workgroup writes its partial gradient row partial[b][...]; a second
// kernel sums the rows over the batch in a fixed order, so results are deterministic.

constexpr int kBwdMaxTerms = 9 * 11;     // n_ch <= 9 channels x len <= 11 weights
constexpr int kBwdSlots = 16;            // LDS slots per weight: 4 wavefronts x 4 rows of 16 lanes

struct BwdState {
    float qsum;     // per lane: sum of q (bias gradient)
    float vmax;     // per lane: running max of z = y - bias
    int targ;       // per lane: first position attaining vmax
};

// softPPV derivative factor: given z = y - bias returns s(1-s) with
// s = 1/(1+e), e = exp(-(lambda*y+shift)) = exp2(z*nl + ns).  The exponent is capped so
// that e stays finite; 1-s is formed as e*s, which keeps its relative accuracy
// when s is close to 1.
__device__ __forceinline__ float rk_dsigmoid(float z, float nl, float ns)
{
    const float e = __builtin_amdgcn_exp2f(fminf(fmaf(z, nl, ns), 80.f));
    const float sg = __builtin_amdgcn_rcpf(1.f + e);
    return sg * (e * sg);
}

// Sum over each row of 16 lanes (all 16 lanes end up with the row sum).
__device__ __forceinline__ float rk_row16_sum(float v)
{
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x124, 0xF, 0xF, true));  // row_ror:4
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x128, 0xF, 0xF, true));  // row_ror:8
    return v;
}

// Adds the lane shares g[0..LEN) of channel c's weight gradient to the LDS slots.
// Must be called by all 64 lanes of the wavefront.
template <int LEN>
__device__ __forceinline__ void rk_bwd_deposit(float (&g)[LEN], int c, float *slots)
{
#pragma unroll
    for (int j = 0; j < LEN; ++j) g[j] = rk_row16_sum(g[j]);
    const int tid = static_cast<int>(threadIdx.x);
    if ((tid & 15) == 0) {
        float *slot = slots + (c * LEN) * kBwdSlots + (tid >> 4);   // (wavefront, row) = tid / 16
#pragma unroll
        for (int j = 0; j < LEN; ++j) slot[j * kBwdSlots] += g[j];
    }
}

template <int LEN, int R>
__device__ __forceinline__ void rk_bwd_segment(const KernelCtx &k, int row0, int nbands, int ncols, float coef,
                                               bool want_max, float *slots, BwdState &st)
{
    const int nstrips = nbands * ncols;
    const uint32_t dbytes = static_cast<uint32_t>(k.d) * 4u;
    const int step_band = kThreads / ncols, step_r = kThreads - step_band * ncols;   // uniform
    int band_run = (nbands == 1) ? 0 : static_cast<int>(threadIdx.x) / ncols;
    int r_run = static_cast<int>(threadIdx.x) - band_run * ncols;
    for (int base = 0; base < nstrips; base += kThreads, band_run += step_band, r_run += step_r) {   // uniform trip count
        if (r_run >= ncols) { r_run -= ncols; ++band_run; }
        const int s_raw = base + static_cast<int>(threadIdx.x);
        const bool valid = s_raw < nstrips;
        const float lane_coef = valid ? coef : 0.f;
        // idle lanes redo the segment's last strip with weight 0
        const int band = valid ? band_run : nbands - 1;
        const int r = valid ? r_run : ncols - 1;
        const int t0 = (row0 + band * R) * k.d + r;
        const uint32_t voff = static_cast<uint32_t>(t0) * 4u;
        float acc[R];
#pragma unroll
        for (int i = 0; i < R; ++i) acc[i] = 0.f;
        for (int c = 0; c < k.nch; ++c) {
            const __amdgpu_buffer_rsrc_t row =
                rk_row_buffer(k.xk + static_cast<size_t>(k.chans[c]) * k.row_bytes, k.span_bytes);
            float w[LEN];
#pragma unroll
            for (int j = 0; j < LEN; ++j) w[j] = k.wts[c * LEN + j];
            uint32_t soff = 0;
            rk_static_for<0, R + LEN - 1>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                rk_taps<LEN, R, i>(w, rk_load(row, voff, soff), acc);
                soff = rk_advance(soff, dbytes);
            });
        }
        if (want_max) {
#pragma unroll
            for (int i = 0; i < R; ++i) {
                if (acc[i] > st.vmax) { st.vmax = acc[i]; st.targ = t0 + i * k.d; }
            }
        }
#pragma unroll
        for (int i = 0; i < R; ++i) {
            acc[i] = lane_coef * rk_dsigmoid(acc[i], k.nl, k.ns);   // acc now holds q
            st.qsum += acc[i];
        }
        for (int c = 0; c < k.nch; ++c) {
            const __amdgpu_buffer_rsrc_t row =
                rk_row_buffer(k.xk + static_cast<size_t>(k.chans[c]) * k.row_bytes, k.span_bytes);
            float g[LEN];
#pragma unroll
            for (int j = 0; j < LEN; ++j) g[j] = 0.f;
            uint32_t soff = 0;
            rk_static_for<0, R + LEN - 1>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                const float xv = rk_load(row, voff, soff);
                soff = rk_advance(soff, dbytes);
                rk_static_for<0, LEN>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
                    constexpr int o = i - j;
                    if constexpr (o >= 0 && o < R) g[j] = fmaf(acc[o], xv, g[j]);
                });
            });
            rk_bwd_deposit<LEN>(g, c, slots);
        }
    }
}

// LDS path of the backward pass (d < 8): the chunk's input range is staged once per
// channel for the conv and once more for the weight gradient.
template <int LEN, int D>
__device__ __forceinline__ int rk_bwd_lds_bands(const KernelCtx &k, int rows, float coef, bool want_max, float *tile,
                                                float *slots, BwdState &st)
{
    constexpr int R = kLdsRows;
    const int nb = rows / R;
    if (nb == 0) return 0;
    constexpr int G = kThreads / D;
    const int tid = static_cast<int>(threadIdx.x);
    const int lane = tid & 63;
    const int bl_raw = tid / D;
    const int r = tid - bl_raw * D;
    for (int band0 = 0; band0 < nb; band0 += G) {
        const int gb = min(G, nb - band0);
        const bool active = bl_raw < gb;
        const int bl = active ? bl_raw : gb - 1;        // idle lanes redo the chunk's last band with weight 0
        const float lane_coef = active ? coef : 0.f;
        const float *mine = tile + bl * R * D + r;
        const int nin = (gb * R + LEN - 1) * D;
        const uint32_t chunk_bytes = static_cast<uint32_t>(band0 * R * D) * 4u;
        float acc[R];
#pragma unroll
        for (int i = 0; i < R; ++i) acc[i] = 0.f;
        for (int c = 0; c < k.nch; ++c) {
            const __amdgpu_buffer_rsrc_t row =
                rk_row_buffer(k.xk + static_cast<size_t>(k.chans[c]) * k.row_bytes, k.span_bytes);
            float w[LEN];
#pragma unroll
            for (int j = 0; j < LEN; ++j) w[j] = k.wts[c * LEN + j];
            rk_stage_tile(row, chunk_bytes, nin, tile);
            rk_static_for<0, R + LEN - 1>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                rk_taps<LEN, R, i>(w, mine[i * D], acc);
            });
        }
        {
            const int t0 = ((band0 + bl) * R) * D + r;
            if (want_max) {
#pragma unroll
                for (int i = 0; i < R; ++i) {
                    if (acc[i] > st.vmax) { st.vmax = acc[i]; st.targ = t0 + i * D; }
                }
            }
#pragma unroll
            for (int i = 0; i < R; ++i) {
                acc[i] = lane_coef * rk_dsigmoid(acc[i], k.nl, k.ns);
                st.qsum += acc[i];
            }
        }
        for (int c = 0; c < k.nch; ++c) {
            const __amdgpu_buffer_rsrc_t row =
                rk_row_buffer(k.xk + static_cast<size_t>(k.chans[c]) * k.row_bytes, k.span_bytes);
            rk_stage_tile(row, chunk_bytes, nin, tile);
            float g[LEN];
#pragma unroll
            for (int j = 0; j < LEN; ++j) g[j] = 0.f;
            rk_static_for<0, R + LEN - 1>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                const float xv = mine[i * D];
                rk_static_for<0, LEN>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
                    constexpr int o = i - j;
                    if constexpr (o >= 0 && o < R) g[j] = fmaf(acc[o], xv, g[j]);
                });
            });
            rk_bwd_deposit<LEN>(g, c, slots);
        }
    }
    return nb * R;
}

template <int LEN, int D>
__device__ __forceinline__ int rk_bwd_lds_dispatch(const KernelCtx &k, int rows, float coef, bool want_max,
                                                   float *tile, float *slots, BwdState &st)
{
    if constexpr (D < kLdsMaxD) {
        if (k.d == D) return rk_bwd_lds_bands<LEN, D>(k, rows, coef, want_max, tile, slots, st);
        return rk_bwd_lds_dispatch<LEN, D + 1>(k, rows, coef, want_max, tile, slots, st);
    } else {
        return 0;
    }
}

template <int LEN>
__device__ __forceinline__ void rk_backward_body(const KernelCtx &k, int nout, float coef, bool want_max,
                                                 float *tile, float *slots, BwdState &st)
{
    const int d = k.d;
    const int total_rows = nout / d;
    const int tail = nout - total_rows * d;
    int row0 = 0;
    if (d < kLdsMaxD) row0 = rk_bwd_lds_dispatch<LEN, 1>(k, total_rows, coef, want_max, tile, slots, st);
    const int rows = total_rows - row0;   // rows left for the register path
    const int nb32 = rows >> 5;
    if (nb32) { rk_bwd_segment<LEN, 32>(k, row0, nb32, d, coef, want_max, slots, st); row0 += nb32 << 5; }
    if (rows & 16) { rk_bwd_segment<LEN, 16>(k, row0, 1, d, coef, want_max, slots, st); row0 += 16; }
    if (rows & 8) { rk_bwd_segment<LEN, 8>(k, row0, 1, d, coef, want_max, slots, st); row0 += 8; }
    if (rows & 4) { rk_bwd_segment<LEN, 4>(k, row0, 1, d, coef, want_max, slots, st); row0 += 4; }
    if (rows & 2) { rk_bwd_segment<LEN, 2>(k, row0, 1, d, coef, want_max, slots, st); row0 += 2; }
    if (rows & 1) { rk_bwd_segment<LEN, 1>(k, row0, 1, d, coef, want_max, slots, st); row0 += 1; }
    if (tail) rk_bwd_segment<LEN, 1>(k, row0, 1, tail, coef, want_max, slots, st);
}

// grid: B*K workgroups.  grad_out is B x (F*K); plane_soft / plane_max are the plane
// indices of the softPPV and max features in it (plane_max < 0: max not included).
// partial is B rows of (total_w + K) floats: weight gradients in the layout of
// `weights`, then the K bias gradients.
__global__ __launch_bounds__(kThreads) void rk_backward(const float *__restrict__ xpad, int row_len, int lead, int L, int C, int K,
                                                        const RkKernelRec *__restrict__ recs,
                                                        const int32_t *__restrict__ order,
                                                        const int32_t *__restrict__ channels,
                                                        const float *__restrict__ weights,
                                                        const float *__restrict__ grad_out, int F, int plane_soft,
                                                        int plane_max, float lambda, float nl, float ns,
                                                        float *__restrict__ partial, int total_w)
{
    __shared__ float tile[kLdsTileWords];
    __shared__ float slots[kBwdMaxTerms * kBwdSlots];
    __shared__ float s_q[kWaves];
    __shared__ float s_max[kWaves];
    __shared__ int s_arg[kWaves];
    const int b = blockIdx.x / K;
    const int kid = order[blockIdx.x - b * K];
    const RkKernelRec rec = recs[kid];
    KernelCtx k;
    k.row_bytes = static_cast<size_t>(row_len) * 4;
    k.xk = reinterpret_cast<const char *>(xpad) + static_cast<size_t>(b) * C * k.row_bytes +
           static_cast<size_t>(lead - rec.pad) * 4;
    k.span_bytes = static_cast<uint32_t>(row_len - (lead - rec.pad)) * 4u;
    k.chans = channels + rec.ch_off;
    k.wts = weights + rec.w_off;
    k.nch = rec.nch;
    k.d = rec.dil;
    k.pad = rec.pad;
    k.L = L;
    k.negbias = -rec.bias;
    k.mask = 0;
    k.nl = nl;
    k.ns = fmaf(rec.bias, nl, ns);

    const int nterms = rec.nch * rec.len;
    for (int i = threadIdx.x; i < nterms * kBwdSlots; i += kThreads) slots[i] = 0.f;
    __syncthreads();

    const float *g_row = grad_out + static_cast<size_t>(b) * F * K;
    const float g_soft = g_row[static_cast<size_t>(plane_soft) * K + kid];
    const float coef = g_soft * lambda / static_cast<float>(rec.nout);
    const bool want_max = plane_max >= 0;

    BwdState st;
    st.qsum = 0.f;
    st.vmax = -INFINITY;
    st.targ = 0;
    if (rec.len == 7) rk_backward_body<7>(k, rec.nout, coef, want_max, tile, slots, st);
    else if (rec.len == 9) rk_backward_body<9>(k, rec.nout, coef, want_max, tile, slots, st);
    else rk_backward_body<11>(k, rec.nout, coef, want_max, tile, slots, st);

    // close the lane reductions: sum of q, and (max, first position) pairs
    float qsum = st.qsum, vmax = st.vmax;
    int targ = st.targ;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        qsum += __shfl_xor(qsum, off);
        const float om = __shfl_xor(vmax, off);
        const int ot = __shfl_xor(targ, off);
        if (om > vmax || (om == vmax && ot < targ)) { vmax = om; targ = ot; }
    }
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { s_q[wave] = qsum; s_max[wave] = vmax; s_arg[wave] = targ; }
    __syncthreads();   // also orders the slot updates before the slot sums below
    float gq = s_q[0], gm = s_max[0];
    int ga = s_arg[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {
        gq += s_q[w];
        if (s_max[w] > gm || (s_max[w] == gm && s_arg[w] < ga)) { gm = s_max[w]; ga = s_arg[w]; }
    }
    const float g_max = want_max ? g_row[static_cast<size_t>(plane_max) * K + kid] : 0.f;

    float *prow = partial + static_cast<size_t>(b) * (static_cast<size_t>(total_w) + K);
    const int t = static_cast<int>(threadIdx.x);
    if (t < nterms) {
        float sum = 0.f;
#pragma unroll
        for (int l = 0; l < kBwdSlots; ++l) sum += slots[t * kBwdSlots + l];
        if (want_max) {
            const int c = t / rec.len, j = t - c * rec.len;
            const float *xrow = reinterpret_cast<const float *>(k.xk + static_cast<size_t>(k.chans[c]) * k.row_bytes);
            sum = fmaf(g_max, xrow[ga + j * rec.dil], sum);
        }
        prow[rec.w_off + t] = sum;
    }
    if (t == 0) prow[total_w + kid] = gq + g_max;
}

// out[i] = sum_b partial[b][i] for i < width, in ascending b; the first total_w
// entries go to grad_w, the remaining K to grad_b.
__global__ __launch_bounds__(256) void rk_reduce_batch(const float *__restrict__ partial, int B, int width, int total_w,
                                                       float *__restrict__ grad_w, float *__restrict__ grad_b)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= width) return;
    float sum = 0.f;
    for (int b = 0; b < B; ++b) sum += partial[static_cast<size_t>(b) * width + i];
    if (i < total_w) grad_w[i] = sum;
    else grad_b[i - total_w] = sum;
}

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
    if (static_cast<int64_t>(B) * h->K > INT32_MAX) return rk_fail(ROCKET_EINVAL, who + ": B*K exceeds the grid limit");
    const size_t need = rocket_workspace_bytes(h, B, mask, backward);
    if (!ws || ws_bytes < need)
        return rk_fail(ROCKET_EWORKSPACE, who + ": workspace of " + std::to_string(need) + " bytes required");
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return rk_fail(ROCKET_EWORKSPACE, who + ": workspace must be 256-byte aligned");
    return ROCKET_OK;
}

static int launch_pad(const rocket_kernels *h, const float *x, int32_t B, float *xpad, hipStream_t stream)
{
    const int nrows = B * h->C;
    dim3 grid(static_cast<unsigned>((h->row_len / 4 + 255) / 256), static_cast<unsigned>(std::min(nrows, 32768)));
    hipLaunchKernelGGL(rk_pad_rows, grid, dim3(256), 0, stream, x, xpad, h->L, h->lead,
                       static_cast<int>(h->row_len), nrows);
    RK_HIP(hipGetLastError());
    return ROCKET_OK;
}

extern "C" int rocket_transform(rocket_kernels *h, const float *x_dev, int32_t B, uint32_t mask, float lambda,
                                float shift, float *out_dev, void *ws, size_t ws_bytes, void *hip_stream)
{
    int rc = check_common("rocket_transform", h, x_dev, B, mask, lambda, shift, ws, ws_bytes, 0);
    if (rc != ROCKET_OK) return rc;
    if (!out_dev) return rk_fail(ROCKET_EINVAL, "rocket_transform: out_dev is NULL");
    if (h->row_len > INT32_MAX) return rk_fail(ROCKET_EINVAL, "rocket_transform: series too long");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    rc = ensure_device(h, stream);
    if (rc != ROCKET_OK) return rc;
    float *xpad = static_cast<float *>(ws);
    rc = launch_pad(h, x_dev, B, xpad, stream);
    if (rc != ROCKET_OK) return rc;
    const float nl = -lambda * kLog2e, ns = -shift * kLog2e;
    rc = profile_mark(h, stream, true);
    if (rc != ROCKET_OK) return rc;
    hipLaunchKernelGGL(rk_forward, dim3(static_cast<unsigned>(B) * h->K), dim3(kThreads), 0, stream, xpad,
                       static_cast<int>(h->row_len), h->lead, h->L, h->C, h->K, h->d_rec, h->d_order, h->d_channels,
                       h->d_weights, mask, nl, ns, out_dev);
    RK_HIP(hipGetLastError());
    return profile_mark(h, stream, false);
}

extern "C" int rocket_soft_ppv_backward(rocket_kernels *h, const float *x_dev, int32_t B, uint32_t mask,
                                        const float *grad_out_dev, float lambda, float shift, int include_max,
                                        float *grad_w_dev, float *grad_b_dev, void *ws, size_t ws_bytes,
                                        void *hip_stream)
{
    int rc = check_common("rocket_soft_ppv_backward", h, x_dev, B, mask, lambda, shift, ws, ws_bytes, 1);
    if (rc != ROCKET_OK) return rc;
    if (!(mask & ROCKET_F_SOFTPPV)) return rk_fail(ROCKET_EINVAL, "rocket_soft_ppv_backward: mask must contain ROCKET_F_SOFTPPV");
    if (include_max && !(mask & ROCKET_F_MAX)) return rk_fail(ROCKET_EINVAL, "rocket_soft_ppv_backward: include_max needs ROCKET_F_MAX in the mask");
    if (!grad_out_dev || !grad_w_dev || !grad_b_dev) return rk_fail(ROCKET_EINVAL, "rocket_soft_ppv_backward: NULL gradient pointer");
    if (h->row_len > INT32_MAX) return rk_fail(ROCKET_EINVAL, "rocket_soft_ppv_backward: series too long");
    if (h->max_terms > kBwdMaxTerms)
        return rk_fail(ROCKET_ESHAPE, "rocket_soft_ppv_backward: a kernel has more than 9 channels x 11 weights");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    rc = ensure_device(h, stream);
    if (rc != ROCKET_OK) return rc;
    float *xpad = static_cast<float *>(ws);
    float *partial = reinterpret_cast<float *>(static_cast<char *>(ws) + padded_batch_bytes(h, B));
    rc = launch_pad(h, x_dev, B, xpad, stream);
    if (rc != ROCKET_OK) return rc;
    const int F = rocket_num_features(mask);
    const int plane_soft = F - 1;                 // planes are in bit order: softPPV is last
    const int plane_max = include_max ? 0 : -1;   // and max, when present, is first
    const float nl = -lambda * kLog2e, ns = -shift * kLog2e;
    const int total_w = static_cast<int>(h->w_off[h->K]);
    rc = profile_mark(h, stream, true);
    if (rc != ROCKET_OK) return rc;
    hipLaunchKernelGGL(rk_backward, dim3(static_cast<unsigned>(B) * h->K), dim3(kThreads), 0, stream, xpad,
                       static_cast<int>(h->row_len), h->lead, h->L, h->C, h->K, h->d_rec, h->d_order, h->d_channels,
                       h->d_weights, grad_out_dev, F, plane_soft, plane_max, lambda, nl, ns, partial, total_w);
    RK_HIP(hipGetLastError());
    rc = profile_mark(h, stream, false);
    if (rc != ROCKET_OK) return rc;
    const int width = total_w + h->K;
    hipLaunchKernelGGL(rk_reduce_batch, dim3((width + 255) / 256), dim3(256), 0, stream, partial, B, width, total_w,
                       grad_w_dev, grad_b_dev);
    RK_HIP(hipGetLastError());
    return ROCKET_OK;
}
