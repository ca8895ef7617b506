// ROCKET transform for MI355X (gfx950): forward kernels (zero-padding copy, conv +
// pooling) and their launchers.  See include/rocket.h for the contract of the entry points.
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
#include "rocket_device.hpp"

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
    KernelCtx k = rk_make_ctx(rec, xpad, row_len, lead, L, C, b, channels, weights);
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

// ------------------------------------------------------------------ launchers

int rk_launch_pad(const rocket_kernels *h, const float *x, int32_t B, float *xpad, void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    const int nrows = B * h->C;
    dim3 grid(static_cast<unsigned>((h->row_len / 4 + 255) / 256), static_cast<unsigned>(nrows < 32768 ? nrows : 32768));
    hipLaunchKernelGGL(rk_pad_rows, grid, dim3(256), 0, stream, x, xpad, h->L, h->lead,
                       static_cast<int>(h->row_len), nrows);
    return hipGetLastError() == hipSuccess ? ROCKET_OK : ROCKET_EHIP;
}

int rk_launch_forward(const rocket_kernels *h, const float *xpad, int32_t B, uint32_t mask, float nl, float ns,
                      float *out, void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    hipLaunchKernelGGL(rk_forward, dim3(static_cast<unsigned>(B) * h->K), dim3(kThreads), 0, stream, xpad,
                       static_cast<int>(h->row_len), h->lead, h->L, h->C, h->K, h->d_rec, h->d_order, h->d_channels,
                       h->d_weights, mask, nl, ns, out);
    return hipGetLastError() == hipSuccess ? ROCKET_OK : ROCKET_EHIP;
}
