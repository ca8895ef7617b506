// Device-side helpers shared by the forward and backward translation units of the
// ROCKET transform library (gfx950).  Strip decomposition, notation and the contract
// of every entry point: include/rocket.h and the head of rocket_forward.hip.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "rocket_internal.hpp"

#ifndef RK_RMAX
#define RK_RMAX 32
#endif
#ifndef RK_WPE
#define RK_WPE 6
#endif
constexpr int kWaves = kThreads / 64;
constexpr float kLog2e = 1.4426950408889634f;


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
// With FIRST set (the first channel of a strip) an output's first tap, j = 0, starts its sum with a plain
// product instead of a multiply-add onto a zero that would have to be written first: one vector instruction
// less per output, the same value (the sign of a zero sum aside, which no feature can see).
template <int LEN, int R, int I, bool FIRST = false>
__device__ __forceinline__ void rk_taps(const float (&w)[LEN], float xv, float (&acc)[R])
{
    rk_static_for<0, LEN>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        constexpr int o = I - j;
        if constexpr (o >= 0 && o < R) {
            if constexpr (FIRST && j == 0) acc[o] = w[0] * xv;
            else acc[o] = fmaf(w[j], xv, acc[o]);
        }
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

// Workgroup index -> (series b, work item).  The hardware deals consecutive workgroups out to
// the chip's XCDs (kXcds of them, each with its own L2) in turn.  In the plain mapping all XCDs
// work on the same series at the same time and every L2 fetches the same rows.  With `spread`
// set (the launcher does so when B is a multiple of kXcds) XCD x takes the series with
// b mod kXcds == x, so each L2 holds rows of its own series only.  (The mapping itself works for
// any B: the grid then has kXcds*ceil(B/kXcds)*items workgroups and the ones whose series does
// not exist return false.)
__device__ __forceinline__ bool rk_block_to_pair(int items, int B, int spread, int &b, int &item)
{
    const int g = static_cast<int>(blockIdx.x);
    if (spread) {
        const int x = g % kXcds;
        const int slot = g / kXcds;
        const int bl = slot / items;
        item = slot - bl * items;
        b = bl * kXcds + x;
        return b < B;
    }
    b = g / items;
    item = g - b * items;
    return true;
}

struct KernelCtx {
    const char *xk;        // padded row of channel 0 of this series, shifted by -p (bytes)
    size_t row_bytes;      // bytes per padded row
    uint32_t span_bytes;   // bytes from xk to the end of the zero gap that follows its row
    const int32_t *chans;  // this kernel's channel list
    const float *wts;      // this kernel's weights, channel-major
    int nch, d;
    int pad, L;            // the kernel's padding and the series length
    float negbias;         // -bias
    uint32_t mask;
    float nl, ns;          // softPPV: exp2(z*nl + ns) = exp(-(lambda*y + shift))
};

// LDS path for small dilations (d < kLdsMaxD).  With d < 64 the strips of a wavefront start
// kLdsRows*d floats apart, so direct loads would touch a different cache line per
// lane group.  Instead the workgroup copies the contiguous input range of a
// chunk of bands into LDS with coalesced loads and the lanes read their strips
// from there.  Bands have kLdsRows = 17 rows: an odd row count makes the stride
// between neighbouring bands odd (times d), which spreads the strided LDS reads
// over the banks without padding.  D is a template parameter so that the LDS
// read offsets i*D*4 are immediates.
constexpr int kLdsStage = 4;                                      // staged words per lane per round
// words of the LDS tile of a workgroup of NT lanes: the largest chunk (NT strips of kLdsRows rows
// plus the halo of the widest kernel at the largest LDS-path dilation), rounded up to whole staging rounds
constexpr int rk_tile_words(int nt) { return ((kLdsRows * nt + 10 * (kLdsMaxD - 1)) / (nt * kLdsStage) + 1) * nt * kLdsStage; }
constexpr int kLdsTileWords = rk_tile_words(kThreads);

// Copies `nin` floats starting `chunk_bytes` into a row to the LDS tile (rounded up to whole rounds of
// NT*kLdsStage words: the tile and the workspace slack are sized for that).  The data go from memory straight
// into LDS (buffer_load_dwordx4 ... lds: a wavefront moves 1 KB per instruction, lane l's 16 bytes to the
// wavefront's LDS base + 16 l), not through the vector registers, whose return path is what bounds the
// register paths of these kernels; the source only has to be 4-byte aligned.  Barriers on both sides: nobody
// still reads the previous contents, and the new contents are visible to all lanes afterwards.
template <int NT>
__device__ __forceinline__ void rk_stage_tile(__amdgpu_buffer_rsrc_t row, uint32_t chunk_bytes, int nin, float *tile)
{
    typedef __attribute__((address_space(3))) void *lds_ptr;
    const int tid = static_cast<int>(threadIdx.x);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    __syncthreads();
    for (int base = 0; base < nin; base += NT * kLdsStage) {
        __builtin_amdgcn_raw_ptr_buffer_load_lds(row, (lds_ptr)(tile + base + wave * (64 * kLdsStage)), 16,
                                                 static_cast<int>(static_cast<uint32_t>(tid) * 16u),
                                                 static_cast<int>(chunk_bytes + static_cast<uint32_t>(base) * 4u), 0, 0);
    }
    // vmcnt(0): the copies have landed (gfx9 encoding: vmcnt[3:0] and [15:14], expcnt[6:4] = 7 and lgkmcnt[11:8] = 15 not waited for)
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
}


// Fills the per-workgroup kernel context from the packed record of kernel `rec` and series b.
__device__ __forceinline__ KernelCtx rk_make_ctx(const RkKernelRec &rec, const float *xpad, int row_len, int lead, int L,
                                                 int C, int b, const int32_t *channels, const float *weights)
{
    KernelCtx k;
    k.row_bytes = static_cast<size_t>(row_len) * 4;
    k.xk = reinterpret_cast<const char *>(xpad) + static_cast<size_t>(b) * C * k.row_bytes +
           static_cast<size_t>(lead - rec.pad) * 4;
    k.span_bytes = static_cast<uint32_t>(row_len + rec.pad) * 4u;   // to the end of the next row's gap
    k.chans = channels + rec.ch_off;
    k.wts = weights + rec.w_off;
    k.nch = rec.nch;
    k.d = rec.dil;
    k.pad = rec.pad;
    k.L = L;
    k.negbias = -rec.bias;
    k.mask = 0;
    k.nl = 0.f;
    k.ns = 0.f;
    return k;
}
