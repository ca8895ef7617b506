// ROCKET transform for MI355X (gfx950): soft-PPV backward kernels and their launcher.
// See include/rocket.h for the contract of rocket_soft_ppv_backward.
#include "rocket_device.hpp"

// ------------------------------------------------------------------ backward kernels
//
// Backward pass through softPPV (and, optionally, the max): one workgroup per
// (series, job), the same time tiles and strip decomposition as the forward pass.  Per strip:
//   1. recompute the R conv outputs,
//   2. turn them into q_i = g_soft * (lambda/n) * s_i (1 - s_i),
//   3. per channel, re-read the strip's inputs and form the lane's share of
//      d/dw[c][j] = sum_i q_i * x[c][t_i + j*d - p]  (R*LEN multiply-adds), sum it over
//      each row of 16 lanes with four DPP adds, and let one lane per row add the row
//      sum to that row's own slot in LDS (16 slots per weight: 4 wavefronts x 4 rows;
//      plain read-modify-write, no atomics, nobody else touches the slot).
// Lanes without a strip recompute the last strip with a zero coefficient, so control
// flow stays wavefront-uniform around the cross-lane adds.  At the end the slots are
// summed and the workgroup writes its job's partial sums; a second kernel sums the jobs
// of every kernel over the batch in a fixed order, so results are deterministic.

constexpr int kBwdMaxTerms = 9 * 11;     // n_ch <= 9 channels x len <= 11 weights
constexpr int kReduceThreads = 128;      // >= kBwdMaxTerms + 1: one thread per gradient term of a kernel
constexpr int kBwdFewRowsMax = 20;       // most rows of a kernel that takes the few-rows path (register budget)
constexpr int kBwdSlots = 16;            // LDS slots per weight: 4 wavefronts x 4 rows of 16 lanes

struct BwdState {
    float qsum;     // per lane: sum of q (bias gradient)
    float vmax;     // per lane: running max of z = y - bias
    int targ;       // per lane: first position attaining vmax
};

// q = coef * s(1-s) for z = y - bias, with s = 1/(1+e), e = exp(-(lambda*y+shift)) = exp2(t),
// t = z*nl + ns.  s(1-s) is even in t, so it is evaluated at -|t|: e <= 1 never overflows (no cap
// on the exponent is needed, and the sign flip is a free source modifier), and 1-s is formed as
// e*s, which keeps its relative accuracy in the saturated tails where s - s*s would cancel.
__device__ __forceinline__ float rk_q(float z, float coef, float nl, float ns)
{
    const float e = __builtin_amdgcn_exp2f(-fabsf(fmaf(z, nl, ns)));
    const float sg = __builtin_amdgcn_rcpf(1.f + e);
    return coef * sg * (e * sg);
}

// Running (largest z, first position that attains it) of a lane.  A lane does not always meet
// its positions in increasing order (with d > 256 its next column block, 256 positions on, comes
// after its next row, d positions on), so an exact tie keeps the smaller position.
__device__ __forceinline__ void rk_track_max(float z, int t, BwdState &st)
{
    if (z > st.vmax || (z == st.vmax && t < st.targ)) { st.vmax = z; st.targ = t; }
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
    const int wave0 = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x) & ~63);   // first lane of this wavefront
    for (int base = 0; base < nstrips; base += kThreads, band_run += step_band, r_run += step_r) {   // uniform trip count
        if (r_run >= ncols) { r_run -= ncols; ++band_run; }
        if (base + wave0 >= nstrips) continue;      // no strip left for this wavefront in this pass
        const int s_raw = base + static_cast<int>(threadIdx.x);
        const bool valid = s_raw < nstrips;
        const float lane_coef = valid ? coef : 0.f;
        // idle lanes of a wavefront that still has strips redo the segment's last strip with weight 0
        const int band = valid ? band_run : nbands - 1;
        const int r = valid ? r_run : ncols - 1;
        const int t0 = (row0 + band * R) * k.d + r;
        const uint32_t voff = static_cast<uint32_t>(t0) * 4u;
        float acc[R];
#pragma unroll
        for (int i = 0; i < R; ++i) acc[i] = 0.f;
        const int last = k.nch - 1;
        for (int c = 0; c < last; ++c) {
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
        // the last channel's inputs stay in registers: its weight gradient below needs no second read
        float xlast[R + LEN - 1];
        {
            const __amdgpu_buffer_rsrc_t row =
                rk_row_buffer(k.xk + static_cast<size_t>(k.chans[last]) * k.row_bytes, k.span_bytes);
            float w[LEN];
#pragma unroll
            for (int j = 0; j < LEN; ++j) w[j] = k.wts[last * LEN + j];
            uint32_t soff = 0;
            rk_static_for<0, R + LEN - 1>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                xlast[i] = rk_load(row, voff, soff);
                soff = rk_advance(soff, dbytes);
            });
            rk_static_for<0, R + LEN - 1>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                rk_taps<LEN, R, i>(w, xlast[i], acc);
            });
        }
        if (want_max) {
#pragma unroll
            for (int i = 0; i < R; ++i) {
                rk_track_max(acc[i], t0 + i * k.d, st);
            }
        }
#pragma unroll
        for (int i = 0; i < R; ++i) {
            acc[i] = rk_q(acc[i], lane_coef, k.nl, k.ns);   // acc now holds q
            st.qsum += acc[i];
        }
        {
            float g[LEN];
#pragma unroll
            for (int j = 0; j < LEN; ++j) g[j] = 0.f;
            rk_static_for<0, R + LEN - 1>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                rk_static_for<0, LEN>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
                    constexpr int o = i - j;
                    if constexpr (o >= 0 && o < R) g[j] = fmaf(acc[o], xlast[i], g[j]);
                });
            });
            rk_bwd_deposit<LEN>(g, last, slots);
        }
        for (int c = 0; c < last; ++c) {
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

// One band of R < 32 rows.  A lane takes S column blocks (columns tid, tid + 256, ...) per pass,
// so that R*S outputs share one cross-lane reduction per weight: with few rows per band the
// reduction, not the multiply-adds, would otherwise dominate (a kernel with dilation in the
// thousands has a dozen rows in all).  Column blocks that lie wholly beyond the band for this
// wavefront are skipped by wavefront-uniform branches.
template <int LEN, int R, int S>
__device__ __forceinline__ void rk_bwd_band(const KernelCtx &k, int row0, int ncols, float coef, bool want_max,
                                            float *slots, BwdState &st)
{
    const uint32_t dbytes = static_cast<uint32_t>(k.d) * 4u;
    const int tid = static_cast<int>(threadIdx.x);
    const int wave0 = __builtin_amdgcn_readfirstlane(tid & ~63);    // first lane of this wavefront
    for (int base = 0; base < ncols; base += S * kThreads) {        // uniform trip count
        if (base + wave0 >= ncols) continue;                        // nothing for this wavefront in this pass
        float acc[S][R];
        uint32_t voff[S];
        int t0[S];
        float lane_coef[S];
        bool live[S];
        rk_static_for<0, S>([&](auto sc) {
            constexpr int s = decltype(sc)::value;
            const int col = base + s * kThreads + tid;
            const bool valid = col < ncols;
            live[s] = base + s * kThreads + wave0 < ncols;          // wavefront-uniform
            lane_coef[s] = valid ? coef : 0.f;
            t0[s] = row0 * k.d + (valid ? col : ncols - 1);         // idle lanes redo the last column with weight 0
            voff[s] = static_cast<uint32_t>(t0[s]) * 4u;
#pragma unroll
            for (int i = 0; i < R; ++i) acc[s][i] = 0.f;
        });
        for (int c = 0; c < k.nch; ++c) {
            const __amdgpu_buffer_rsrc_t row =
                rk_row_buffer(k.xk + static_cast<size_t>(k.chans[c]) * k.row_bytes, k.span_bytes);
            float w[LEN];
#pragma unroll
            for (int j = 0; j < LEN; ++j) w[j] = k.wts[c * LEN + j];
            rk_static_for<0, S>([&](auto sc) {
                constexpr int s = decltype(sc)::value;
                if (live[s]) {
                    uint32_t soff = 0;
                    rk_static_for<0, R + LEN - 1>([&](auto ic) {
                        constexpr int i = decltype(ic)::value;
                        rk_taps<LEN, R, i>(w, rk_load(row, voff[s], soff), acc[s]);
                        soff = rk_advance(soff, dbytes);
                    });
                }
            });
        }
        rk_static_for<0, S>([&](auto sc) {
            constexpr int s = decltype(sc)::value;
            if (live[s]) {
                if (want_max) {
#pragma unroll
                    for (int i = 0; i < R; ++i) {
                        rk_track_max(acc[s][i], t0[s] + i * k.d, st);
                    }
                }
#pragma unroll
                for (int i = 0; i < R; ++i) {
                    acc[s][i] = rk_q(acc[s][i], lane_coef[s], k.nl, k.ns);   // acc now holds q
                    st.qsum += acc[s][i];
                }
            }
        });
        for (int c = 0; c < k.nch; ++c) {
            const __amdgpu_buffer_rsrc_t row =
                rk_row_buffer(k.xk + static_cast<size_t>(k.chans[c]) * k.row_bytes, k.span_bytes);
            float g[LEN];
#pragma unroll
            for (int j = 0; j < LEN; ++j) g[j] = 0.f;
            rk_static_for<0, S>([&](auto sc) {
                constexpr int s = decltype(sc)::value;
                if (live[s]) {
                    uint32_t soff = 0;
                    rk_static_for<0, R + LEN - 1>([&](auto ic) {
                        constexpr int i = decltype(ic)::value;
                        const float xv = rk_load(row, voff[s], soff);
                        soff = rk_advance(soff, dbytes);
                        rk_static_for<0, LEN>([&](auto jc) {
                            constexpr int j = decltype(jc)::value;
                            constexpr int o = i - j;
                            if constexpr (o >= 0 && o < R) g[j] = fmaf(acc[s][o], xv, g[j]);
                        });
                    });
                }
            });
            rk_bwd_deposit<LEN>(g, c, slots);
        }
    }
}

// Rows [row0, row0 + rows) of a kernel with a large dilation, and the partial row after them (`tail`
// outputs, 0 if none): a whole kernel when it has few rows (n / d), otherwise what a job has left
// after its bands of 32.  They form one strip per lane, so every input value is loaded once per
// pass instead of once per band of a 16/8/4/2/1 cascade.  As in the forward pass the row count is a run-time
// uniform: window rows past it, and window rows that lie wholly in the zero padding, are
// skipped (loads and multiply-adds) with scalar branches.  The conv's last channel is the
// weight gradient's first, with its inputs still in registers.
template <int LEN, int RM>
__device__ __forceinline__ void rk_bwd_few_rows(const KernelCtx &k, int row0, int rows, int tail, float coef,
                                                bool want_max, float *slots, BwdState &st)
{
    const int nrows = rows + (tail > 0 ? 1 : 0);            // rows with at least one output
    const int prow = k.pad / k.d;                           // padding in rows: 0 or (LEN-1)/2
    const int data_rows = (k.L + k.d - 1) / k.d;            // input rows that hold samples
    const uint32_t dbytes = static_cast<uint32_t>(k.d) * 4u;
    // bit i: window row row0 + i is needed (i < nrows+LEN-1) and holds samples (0 <= row0+i-prow < data_rows)
    uint32_t live = 0;
    for (int i = 0; i < nrows + LEN - 1; ++i) {
        if (row0 + i >= prow && row0 + i - prow < data_rows) live |= 1u << i;
    }
    const uint32_t soff0 = static_cast<uint32_t>(row0) * dbytes;
    // single scalar bit tests on an opaque copy, instead of twenty-odd precomputed lane masks
    auto is_live = [&](int i) {
        uint32_t word = live;
        asm volatile("" : "+s"(word));
        return ((word >> i) & 1u) != 0;
    };
    const int tid = static_cast<int>(threadIdx.x);
    const int wave0 = __builtin_amdgcn_readfirstlane(tid & ~63);
    const int last = k.nch - 1;
    for (int base = 0; base < k.d; base += kThreads) {      // uniform trip count
        if (base + wave0 >= k.d) continue;                  // no column for this wavefront in this pass
        const int r_raw = base + tid;
        const bool lane_ok = r_raw < k.d;
        const int r = lane_ok ? r_raw : k.d - 1;            // idle lanes shadow the last column with weight 0
        const uint32_t voff = static_cast<uint32_t>(r) * 4u;
        float acc[RM];
#pragma unroll
        for (int i = 0; i < RM; ++i) acc[i] = 0.f;
        float xv[RM + LEN - 1];
        for (int c = 0; c <= last; ++c) {                   // xv keeps the inputs of channel `last`
            const __amdgpu_buffer_rsrc_t row =
                rk_row_buffer(k.xk + static_cast<size_t>(k.chans[c]) * k.row_bytes, k.span_bytes);
            float w[LEN];
#pragma unroll
            for (int j = 0; j < LEN; ++j) w[j] = k.wts[c * LEN + j];
            uint32_t soff = soff0;
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
            float q = 0.f;
            if (o < lim) {                                  // uniform
                const bool own = o < own_rows;
                if (want_max && own) rk_track_max(acc[o], (row0 + o) * k.d + r, st);
                q = rk_q(acc[o], own ? coef : 0.f, k.nl, k.ns);
                st.qsum += q;
            }
            acc[o] = q;                                     // acc now holds q (0 for rows that do not exist)
        });
        for (int cc = 0; cc <= last; ++cc) {
            const int c = cc == 0 ? last : cc - 1;
            float g[LEN];
#pragma unroll
            for (int j = 0; j < LEN; ++j) g[j] = 0.f;
            if (cc > 0) {
                const __amdgpu_buffer_rsrc_t row =
                    rk_row_buffer(k.xk + static_cast<size_t>(k.chans[c]) * k.row_bytes, k.span_bytes);
                uint32_t soff = soff0;
                rk_static_for<0, RM + LEN - 1>([&](auto ic) {
                    constexpr int i = decltype(ic)::value;
                    if (is_live(i)) xv[i] = rk_load(row, voff, soff);
                    soff = rk_advance(soff, dbytes);
                });
            }
            rk_static_for<0, RM + LEN - 1>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                if (is_live(i)) {
                    rk_static_for<0, LEN>([&](auto jc) {
                        constexpr int j = decltype(jc)::value;
                        constexpr int o = i - j;
                        if constexpr (o >= 0 && o < RM) g[j] = fmaf(acc[o], xv[i], g[j]);
                    });
                }
            });
            rk_bwd_deposit<LEN>(g, c, slots);
        }
    }
}

// LDS path of the backward pass (d < kLdsMaxD): the chunk's input range is staged once per
// channel for the conv and once more for the weight gradient.
template <int LEN, int D>
__device__ __forceinline__ int rk_bwd_lds_bands(const KernelCtx &k, int first_row, int end_row, float coef,
                                                bool want_max, float *tile, float *slots, BwdState &st)
{
    constexpr int R = kLdsRows;
    const int nb = (end_row - first_row) / R;    // whole bands in [first_row, end_row)
    if (nb == 0) return first_row;
    constexpr int G = kThreads / D;
    const int tid = static_cast<int>(threadIdx.x);
    const int bl_raw = tid / D;
    const int r = tid - bl_raw * D;
    for (int band0 = 0; band0 < nb; band0 += G) {
        const int gb = min(G, nb - band0);
        const bool active = bl_raw < gb;
        const int bl = active ? bl_raw : gb - 1;        // idle lanes redo the chunk's last band with weight 0
        const float lane_coef = active ? coef : 0.f;
        const float *mine = tile + bl * R * D + r;
        const int nin = (gb * R + LEN - 1) * D;
        const uint32_t chunk_bytes = static_cast<uint32_t>((first_row + band0 * R) * D) * 4u;
        float acc[R];
#pragma unroll
        for (int i = 0; i < R; ++i) acc[i] = 0.f;
        for (int c = 0; c < k.nch; ++c) {
            const __amdgpu_buffer_rsrc_t row =
                rk_row_buffer(k.xk + static_cast<size_t>(k.chans[c]) * k.row_bytes, k.span_bytes);
            float w[LEN];
#pragma unroll
            for (int j = 0; j < LEN; ++j) w[j] = k.wts[c * LEN + j];
            rk_stage_tile<kThreads>(row, chunk_bytes, nin, tile);
            rk_static_for<0, R + LEN - 1>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                rk_taps<LEN, R, i>(w, mine[i * D], acc);
            });
        }
        {
            const int t0 = (first_row + (band0 + bl) * R) * D + r;
            if (want_max) {
#pragma unroll
                for (int i = 0; i < R; ++i) {
                    rk_track_max(acc[i], t0 + i * D, st);
                }
            }
#pragma unroll
            for (int i = 0; i < R; ++i) {
                acc[i] = rk_q(acc[i], lane_coef, k.nl, k.ns);
                st.qsum += acc[i];
            }
        }
        // the tile still holds the last channel of the conv: its weight gradient goes first and
        // needs no second staging; the other channels are staged again
        for (int cc = 0; cc < k.nch; ++cc) {
            const int c = cc == 0 ? k.nch - 1 : cc - 1;
            if (cc > 0) {
                const __amdgpu_buffer_rsrc_t row =
                    rk_row_buffer(k.xk + static_cast<size_t>(k.chans[c]) * k.row_bytes, k.span_bytes);
                rk_stage_tile<kThreads>(row, chunk_bytes, nin, tile);
            }
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
    return first_row + nb * R;
}

template <int LEN, int D>
__device__ __forceinline__ int rk_bwd_lds_dispatch(const KernelCtx &k, int first_row, int end_row, float coef,
                                                   bool want_max, float *tile, float *slots, BwdState &st)
{
    if constexpr (D < kLdsMaxD) {
        if (k.d == D) return rk_bwd_lds_bands<LEN, D>(k, first_row, end_row, coef, want_max, tile, slots, st);
        return rk_bwd_lds_dispatch<LEN, D + 1>(k, first_row, end_row, coef, want_max, tile, slots, st);
    } else {
        return first_row;
    }
}

template <int LEN>
__device__ __forceinline__ void rk_backward_body(const KernelCtx &k, int nout, const RkJob job, float coef,
                                                 bool want_max, float *tile, float *slots, BwdState &st)
{
    const int d = k.d;
    const int total_rows = nout / d;
    const int tail = nout - total_rows * d;
    // the job's rows: whole LDS chunks first (small dilations), then bands of 32 rows, then what is left
    int row0 = job.row0;
    if (d < kLdsMaxD) row0 = rk_bwd_lds_dispatch<LEN, 1>(k, row0, job.row1, coef, want_max, tile, slots, st);
    int rows = job.row1 - row0;   // rows left for the register path
    const int nb32 = rows >> 5;
    if (nb32) { rk_bwd_segment<LEN, 32>(k, row0, nb32, d, coef, want_max, slots, st); row0 += nb32 << 5; rows &= 31; }
    const int own_tail = (job.flags & 1) ? tail : 0;
    if (d >= kFewMinD) {          // uniform
        // With at least kFewMinD columns to a row the rows that are left (fewer than 32, and the partial last
        // row) form one strip per column with a run-time row count: a whole kernel when it has few rows.
        if (rows + (own_tail > 0 ? 1 : 0) > kBwdFewRowsMax) {
            rk_bwd_band<LEN, 16, 2>(k, row0, d, coef, want_max, slots, st);
            row0 += 16; rows -= 16;
        }
        const int nrows = rows + (own_tail > 0 ? 1 : 0);
        if (nrows == 0) return;
        if (nrows <= 8) { rk_bwd_few_rows<LEN, 8>(k, row0, rows, own_tail, coef, want_max, slots, st); return; }
        rk_bwd_few_rows<LEN, kBwdFewRowsMax>(k, row0, rows, own_tail, coef, want_max, slots, st);
        return;
    }
    // smaller dilations: the binary remainder; the job that owns the partial last row does it last
    if (rows & 16) { rk_bwd_band<LEN, 16, 2>(k, row0, d, coef, want_max, slots, st); row0 += 16; }
    if (rows & 8) { rk_bwd_band<LEN, 8, 4>(k, row0, d, coef, want_max, slots, st); row0 += 8; }
    if (rows & 4) { rk_bwd_band<LEN, 4, 8>(k, row0, d, coef, want_max, slots, st); row0 += 4; }
    if (rows & 2) { rk_bwd_band<LEN, 2, 8>(k, row0, d, coef, want_max, slots, st); row0 += 2; }
    if (rows & 1) { rk_bwd_band<LEN, 1, 8>(k, row0, d, coef, want_max, slots, st); row0 += 1; }
    if (own_tail) rk_bwd_band<LEN, 1, 8>(k, total_rows, own_tail, coef, want_max, slots, st);
}

// grid: one workgroup per (series, job), mapped by rk_block_to_pair; a job is a time tile of one
// kernel's outputs, the same ones the forward pass uses, in the same order (by the window of the
// series they read), so that workgroups running together share one stretch of one series in L2.
// grad_out is B x (F*K); plane_soft / plane_max are the plane indices of the softPPV and max
// features in it (plane_max < 0: max not included).  partial is B rows of `stride` floats; job j
// owns the words [bjob_off[j], bjob_off[j+1]) of its series' row: the n_ch*len weight-gradient
// sums of its positions, then the sum of q, the largest z = y - bias, and the first position
// that attains it.
__global__ __launch_bounds__(kThreads) void rk_backward(const float *__restrict__ xpad, int row_len, int lead, int L, int C, int K,
                                                        int J, const RkKernelRec *__restrict__ recs,
                                                        const RkJob *__restrict__ jobs,
                                                        const int32_t *__restrict__ bjob_off,
                                                        const int32_t *__restrict__ channels,
                                                        const float *__restrict__ weights,
                                                        const float *__restrict__ grad_out, int F, int plane_soft,
                                                        int plane_max, float lambda, float nl, float ns,
                                                        float *__restrict__ partial, int stride, int B, int spread)
{
    __shared__ __attribute__((aligned(16))) float tile[kLdsTileWords];   // 16-byte pieces are written straight into it
    __shared__ float slots[kBwdMaxTerms * kBwdSlots];
    __shared__ float s_q[kWaves];
    __shared__ float s_max[kWaves];
    __shared__ int s_arg[kWaves];
    int b, jid;
    if (!rk_block_to_pair(J, B, spread, b, jid)) return;
    const RkJob job = jobs[jid];
    const int kid = job.kernel;
    const RkKernelRec rec = recs[kid];
    KernelCtx k = rk_make_ctx(rec, xpad, row_len, lead, L, C, b, channels, weights);
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
    if (rec.len == 7) rk_backward_body<7>(k, rec.nout, job, coef, want_max, tile, slots, st);
    else if (rec.len == 9) rk_backward_body<9>(k, rec.nout, job, coef, want_max, tile, slots, st);
    else rk_backward_body<11>(k, rec.nout, job, coef, want_max, tile, slots, st);

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

    float *prow = partial + static_cast<size_t>(b) * stride + bjob_off[jid];
    const int t = static_cast<int>(threadIdx.x);
    if (t < nterms) {
        float sum = 0.f;
#pragma unroll
        for (int l = 0; l < kBwdSlots; ++l) sum += slots[t * kBwdSlots + l];
        prow[t] = sum;
    }
    if (t == 0) {
        prow[nterms] = gq;
        prow[nterms + 1] = gm;
        reinterpret_cast<int *>(prow)[nterms + 2] = ga;
    }
}

// One workgroup per kernel; thread t < n_ch*len owns weight-gradient term t, thread n_ch*len the
// bias gradient.  Sums the kernel's job partials over the series in ascending b and over the
// jobs in tile order (a fixed order: results repeat bit for bit), finds per series the first
// position of the largest output across the jobs, and adds the max plane's sub-gradient there.
__global__ __launch_bounds__(kReduceThreads) void rk_reduce_jobs(const float *__restrict__ partial, int B, int stride,
                                                                 const float *__restrict__ xpad, int row_len, int lead, int C,
                                                                 int K, const RkKernelRec *__restrict__ recs,
                                                                 const int32_t *__restrict__ kjob_off,
                                                                 const int32_t *__restrict__ kjob_idx,
                                                                 const int32_t *__restrict__ bjob_off,
                                                                 const int32_t *__restrict__ channels,
                                                                 const float *__restrict__ grad_out, int F, int plane_max,
                                                                 float *__restrict__ grad_w, float *__restrict__ grad_b)
{
    const int kid = blockIdx.x;
    const RkKernelRec rec = recs[kid];
    const int nterms = rec.nch * rec.len;
    const int t = static_cast<int>(threadIdx.x);
    if (t > nterms) return;
    const bool want_max = plane_max >= 0;
    const int q0 = kjob_off[kid], q1 = kjob_off[kid + 1];
    int chan = 0, tap = 0;
    if (t < nterms) {
        const int c = t / rec.len;
        tap = (t - c * rec.len) * rec.dil;
        chan = channels[rec.ch_off + c];
    }
    float sum = 0.f;
    for (int b = 0; b < B; ++b) {
        const float *prow = partial + static_cast<size_t>(b) * stride;
        float vmax = -INFINITY;
        int targ = 0;
        for (int q = q0; q < q1; ++q) {
            const float *job = prow + bjob_off[kjob_idx[q]];
            sum += job[t];                                    // term t, or the sum of q at t == nterms
            if (want_max) {
                const float m = job[nterms + 1];
                const int a = reinterpret_cast<const int *>(job)[nterms + 2];
                if (m > vmax || (m == vmax && a < targ)) { vmax = m; targ = a; }
            }
        }
        if (want_max) {
            const float g_max = grad_out[static_cast<size_t>(b) * F * K + static_cast<size_t>(plane_max) * K + kid];
            if (t < nterms) {
                const float *xrow = xpad + (static_cast<size_t>(b) * C + chan) * row_len + (lead - rec.pad);
                sum = fmaf(g_max, xrow[targ + tap], sum);
            } else {
                sum += g_max;
            }
        }
    }
    if (t < nterms) grad_w[rec.w_off + t] = sum;
    else grad_b[kid] = sum;
}

// ------------------------------------------------------------------ launchers

int rk_launch_backward(const rocket_kernels *h, const float *xpad, int32_t B, const float *grad_out, int F,
                       int plane_soft, int plane_max, float lambda, float nl, float ns, float *partial,
                       void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    const int J = static_cast<int>(h->jobs.size());
    const int spread = rk_spread(h, B);
    hipLaunchKernelGGL(rk_backward, dim3(static_cast<unsigned>(rk_grid_groups(B, J, spread))), dim3(kThreads), 0, stream, xpad,
                       static_cast<int>(h->row_len), h->lead, h->L, h->C, h->K, J, h->d_rec, h->d_jobs, h->d_bjob_off,
                       h->d_channels, h->d_weights, grad_out, F, plane_soft, plane_max, lambda, nl, ns, partial,
                       static_cast<int>(h->bjob_off.back()), B, spread);
    return hipGetLastError() == hipSuccess ? ROCKET_OK : ROCKET_EHIP;
}

int rk_launch_reduce_jobs(const rocket_kernels *h, const float *partial, const float *xpad, int32_t B,
                          const float *grad_out, int F, int plane_max, float *grad_w, float *grad_b, void *stream_ptr)
{
    hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
    hipLaunchKernelGGL(rk_reduce_jobs, dim3(static_cast<unsigned>(h->K)), dim3(kReduceThreads), 0, stream, partial, B,
                       static_cast<int>(h->bjob_off.back()), xpad, static_cast<int>(h->row_len), h->lead, h->C, h->K,
                       h->d_rec, h->d_kjob_off, h->d_kjob_idx, h->d_bjob_off, h->d_channels, grad_out, F, plane_max,
                       grad_w, grad_b);
    return hipGetLastError() == hipSuccess ? ROCKET_OK : ROCKET_EHIP;
}
