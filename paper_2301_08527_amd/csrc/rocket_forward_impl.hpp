// Forward kernel of the ROCKET transform, templated on the workgroup size NT
// (256 lanes for long series, one 64-lane wavefront per (series, kernel) for short
// ones).  Included by rocket_forward.hip and rocket_forward_short.hip.
#pragma once
#include "rocket_device.hpp"

// Register path.  All strips of `nbands` bands of R rows x `ncols` columns starting at
// row `row0`; every lane reads its R+LEN-1 inputs straight from global memory
// (consecutive lanes read consecutive floats once d >= 64).
template <int LEN, int R, int NT>
__device__ __forceinline__ void rk_segment(const KernelCtx &k, int row0, int nbands, int ncols, PoolState &st)
{
    const int nstrips = nbands * ncols;
    const uint32_t dbytes = static_cast<uint32_t>(k.d) * 4u;
    for (int base = 0; base < nstrips; base += NT) {
        const int s = base + static_cast<int>(threadIdx.x);
        if (s < nstrips) {
            const int band = (nbands == 1) ? 0 : s / ncols;
            const int r = s - band * ncols;
            const uint32_t voff = static_cast<uint32_t>((row0 + band * R) * k.d + r) * 4u;
            float acc[R];
            auto channel = [&](int c, auto first) {
                const __amdgpu_buffer_rsrc_t row =
                    rk_row_buffer(k.xk + static_cast<size_t>(k.chans[c]) * k.row_bytes, k.span_bytes);
                float w[LEN];
#pragma unroll
                for (int j = 0; j < LEN; ++j) w[j] = k.wts[c * LEN + j];
                uint32_t soff = 0;
                rk_static_for<0, R + LEN - 1>([&](auto ic) {
                    constexpr int i = decltype(ic)::value;
                    rk_taps<LEN, R, i, decltype(first)::value>(w, rk_load(row, voff, soff), acc);
                    soff = rk_advance(soff, dbytes);
                });
            };
            channel(0, std::true_type{});       // starts the sums: no zeroing of the accumulators
            for (int c = 1; c < k.nch; ++c) channel(c, std::false_type{});
            rk_pool<R>(acc, k.mask, k.negbias, k.nl, k.ns, st);
        }
    }
}

template <int LEN, int D, int NT>
__device__ __forceinline__ int rk_lds_bands(const KernelCtx &k, int first_row, int end_row, float *tile, PoolState &st)
{
    constexpr int R = kLdsRows;
    const int nb = (end_row - first_row) / R;    // whole bands in [first_row, end_row)
    if (nb == 0) return first_row;
    constexpr int G = NT / D;                 // bands per chunk
    const int tid = static_cast<int>(threadIdx.x);
    const int bl = tid / D;                         // lane's band inside the chunk
    const int r = tid - bl * D;                     // lane's column
    const float *mine = tile + bl * R * D + r;
    for (int band0 = 0; band0 < nb; band0 += G) {
        const int gb = min(G, nb - band0);
        const bool active = bl < gb;
        const int nin = (gb * R + LEN - 1) * D;     // input floats of this chunk
        const uint32_t chunk_bytes = static_cast<uint32_t>((first_row + band0 * R) * D) * 4u;
        float acc[R];
        auto channel = [&](int c, auto first) {
            const __amdgpu_buffer_rsrc_t row =
                rk_row_buffer(k.xk + static_cast<size_t>(k.chans[c]) * k.row_bytes, k.span_bytes);
            float w[LEN];
#pragma unroll
            for (int j = 0; j < LEN; ++j) w[j] = k.wts[c * LEN + j];
            rk_stage_tile<NT>(row, chunk_bytes, nin, tile);
            if (active) {
                rk_static_for<0, R + LEN - 1>([&](auto ic) {
                    constexpr int i = decltype(ic)::value;
                    rk_taps<LEN, R, i, decltype(first)::value>(w, mine[i * D], acc);
                });
            }
        };
        channel(0, std::true_type{});                  // starts the sums (lanes without a strip neither sum nor pool)
        for (int c = 1; c < k.nch; ++c) channel(c, std::false_type{});
        if (active) rk_pool<R>(acc, k.mask, k.negbias, k.nl, k.ns, st);
    }
    return first_row + nb * R;
}

// Pooling of one finished sum (see rk_pool).
__device__ __forceinline__ void rk_pool1(float z, uint32_t mask, float negbias, float nl, float ns, PoolState &st)
{
    const float one[1] = {z};
    rk_pool<1>(one, mask, negbias, nl, ns, st);
}

// Few-rows path for large dilations: rows [row0, row0 + rows) and the partial row after them
// (`tail` outputs, 0 if none), at most RM rows in all -- a whole kernel when its output has few
// rows of d positions, otherwise what a job has left after its bands of 32.  One strip per
// column covers every row, so each input is loaded exactly once per channel, whatever the row
// count (the binary band decomposition would cut them into short strips with little reuse).
// The row count is a run-time uniform: window rows past it are skipped with scalar
// branches.  Window rows that lie entirely in the zero padding ("same" padding
// with a large dilation puts (len-1)/2 such rows on either side) are skipped too,
// loads and multiply-adds alike.  The partial last row is handled in the same
// strip and masked per lane in the pooling.
template <int LEN, int RM, int NT>
__device__ __forceinline__ void rk_few_rows(const KernelCtx &k, int row0, int rows, int tail, PoolState &st)
{
    const int nrows = rows + (tail > 0 ? 1 : 0);            // rows with at least one output
    const int prow = k.pad / k.d;                           // padding in rows: 0 or (LEN-1)/2
    const int data_rows = (k.L + k.d - 1) / k.d;            // input rows that hold samples
    const uint32_t dbytes = static_cast<uint32_t>(k.d) * 4u;
    // bit i: window row row0 + i is needed (i < nrows+LEN-1) and holds samples (0 <= row0+i-prow < data_rows)
    uint32_t live_lo = 0, live_hi = 0;
    for (int i = 0; i < nrows + LEN - 1; ++i) {
        if (row0 + i >= prow && row0 + i - prow < data_rows) {
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
    const int wave0 = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x) & ~63);   // first lane of this wavefront
    for (int base = 0; base < k.d; base += NT) {      // uniform trip count
        if (base + wave0 >= k.d) continue;            // no column left for this wavefront in this pass
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
            uint32_t soff = static_cast<uint32_t>(row0) * dbytes;
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
template <int LEN, int D, int NT>
__device__ __forceinline__ int rk_lds_dispatch(const KernelCtx &k, int first_row, int end_row, float *tile, PoolState &st)
{
    if constexpr (D < kLdsMaxD) {
        if (k.d == D) return rk_lds_bands<LEN, D, NT>(k, first_row, end_row, tile, st);
        return rk_lds_dispatch<LEN, D + 1, NT>(k, first_row, end_row, tile, st);
    } else {
        return first_row;
    }
}

template <int LEN, int NT>
__device__ __forceinline__ void rk_forward_body(const KernelCtx &k, int nout, const RkJob job, float *tile, PoolState &st)
{
    const int d = k.d;
    const int rows = nout / d;            // full rows of d outputs
    const int tail = nout - rows * d;     // outputs of the partial last row
    // every branch below is uniform per workgroup
    int row0 = job.row0;
    if (d < kLdsMaxD) row0 = rk_lds_dispatch<LEN, 1, NT>(k, row0, job.row1, tile, st);
    // Register path for the remaining rows: bands of 32 rows first.  A band height is used when its
    // strips fill the workgroup (bands x d >= NT).
    int left = job.row1 - row0;
    auto bands_of = [&](auto rc, bool force) {
        constexpr int R = decltype(rc)::value;
        const int nb = left / R;
        if (nb > 0 && (force || nb * d >= NT)) {
            rk_segment<LEN, R, NT>(k, row0, nb, d, st);
            row0 += nb * R;
            left -= nb * R;
        }
    };
#if RK_RMAX >= 64
    bands_of(std::integral_constant<int, 64>{}, false);
#endif
#if RK_RMAX >= 32
    bands_of(std::integral_constant<int, 32>{}, false);
#endif
    const int own_tail = (job.flags & 1) ? tail : 0;
    if (d >= kFewMinD) {
        // With a row of at least kFewMinD columns the rows that are left (fewer than 32, and the partial last
        // row) go through one strip per column with a run-time row count instead of a cascade of bands of 16, 8,
        // 4, 2, 1 rows, each of which would load its own window: a whole kernel when it has few rows.
        if (left + (own_tail > 0 ? 1 : 0) > kFewRowsMax) bands_of(std::integral_constant<int, 16>{}, true);
        const int nrows = left + (own_tail > 0 ? 1 : 0);
        if (nrows == 0) return;
        if (nrows <= 8) { rk_few_rows<LEN, 8, NT>(k, row0, left, own_tail, st); return; }
        if (nrows <= 16) { rk_few_rows<LEN, 16, NT>(k, row0, left, own_tail, st); return; }
        rk_few_rows<LEN, 24, NT>(k, row0, left, own_tail, st);
        return;
    }
    // smaller dilations: bands of 16, 8, 4, 2 rows, tallest first; rows that are left go to the next
    // smaller height, and single rows take the rest
    bands_of(std::integral_constant<int, 16>{}, false);
    bands_of(std::integral_constant<int, 8>{}, false);
    bands_of(std::integral_constant<int, 4>{}, false);
    bands_of(std::integral_constant<int, 2>{}, false);
    bands_of(std::integral_constant<int, 1>{}, true);
    if (own_tail) rk_segment<LEN, 1, NT>(k, rows, 1, own_tail, st);
}

// grid: one workgroup per (series, job), a job being a row range of one kernel; the index
// mapping is rk_block_to_pair's.  It writes the job's partial pooling results: partials holds three planes
// of B*J words (max of y - bias, count of y > 0, sum of sigmoids).
template <int NT>
#if RK_WPE
__attribute__((amdgpu_waves_per_eu(RK_WPE)))
#endif
__global__ __launch_bounds__(NT) void rk_forward(const float *__restrict__ xpad, int row_len, int lead, int L, int C, int J,
                                                       const RkKernelRec *__restrict__ recs,
                                                       const RkJob *__restrict__ jobs,
                                                       const int32_t *__restrict__ channels,
                                                       const float *__restrict__ weights, uint32_t mask, float nl,
                                                       float ns, float *__restrict__ partials, int B, int spread)
{
    __shared__ __attribute__((aligned(16))) float tile[rk_tile_words(NT)];   // 16-byte pieces are written straight into it
    int b, jid;
    if (!rk_block_to_pair(J, B, spread, b, jid)) return;
    const RkJob job = jobs[jid];
    const RkKernelRec rec = recs[job.kernel];
    KernelCtx k = rk_make_ctx(rec, xpad, row_len, lead, L, C, b, channels, weights);
    k.mask = mask;
    k.nl = nl;
    k.ns = fmaf(rec.bias, nl, ns);

    PoolState st;
    st.vmax = -INFINITY;
    st.ssum = 0.f;
    st.cnt = 0;
    if (rec.len == 7) rk_forward_body<7, NT>(k, rec.nout, job, tile, st);
    else if (rec.len == 9) rk_forward_body<9, NT>(k, rec.nout, job, tile, st);
    else rk_forward_body<11, NT>(k, rec.nout, job, tile, st);

    // close the reductions: lanes -> wavefront (shuffles) -> workgroup (LDS)
    float vmax = st.vmax, ssum = st.ssum;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        vmax = fmaxf(vmax, __shfl_xor(vmax, off));
        ssum += __shfl_xor(ssum, off);
    }
    __shared__ float s_max[(NT / 64)];
    __shared__ float s_sum[(NT / 64)];
    __shared__ int s_cnt[(NT / 64)];
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { s_max[wave] = vmax; s_sum[wave] = ssum; s_cnt[wave] = st.cnt; }
    __syncthreads();
    if (threadIdx.x == 0) {
        float m = s_max[0], sm = s_sum[0];
        int cn = s_cnt[0];
#pragma unroll
        for (int w = 1; w < (NT / 64); ++w) { m = fmaxf(m, s_max[w]); sm += s_sum[w]; cn += s_cnt[w]; }
        const size_t plane = static_cast<size_t>(B) * J;
        const size_t slot = static_cast<size_t>(b) * J + jid;
        partials[slot] = m;
        reinterpret_cast<int *>(partials)[plane + slot] = cn;
        partials[2 * plane + slot] = sm;
    }
}
