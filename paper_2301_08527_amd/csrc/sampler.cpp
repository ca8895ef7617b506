// Random kernel initialisation (paper section 3.1), host side of the library.
//
// Compiled with -ffp-contract=off and without fast-math: every kernel must come
// out bit-identical on any host.  The draws of one kernel come from its own
// SplitMix64 stream keyed by (seed, kernel index); each draw uses one 64-bit
// output.  Order of draws: length, channel count, channel subset, weights
// (channel by channel), bias, dilation, padding.
//
// The accept test of the normal draws and the floors that give the channel count and
// the dilation depend on a logarithm and on a power of two.  A math library's last-bit
// rounding differs between machines and could turn such a decision, so the three
// functions are spelt out here (natural_log, two_to_the) as short series of IEEE
// additions, multiplications and divisions in a fixed order; anyone who repeats the
// same operations gets the same kernels.
#include <cmath>
#include <numeric>

#include "rocket_internal.hpp"

namespace {

constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;

inline uint64_t scramble(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

constexpr double kLn2 = 0.6931471805599453;        // ln 2, nearest double
constexpr double kSqrtHalf = 0.7071067811865476;   // sqrt(1/2), nearest double
constexpr int kLogTerms = 12;                      // atanh series: z^(2i+1)/(2i+1), i = 0..12
constexpr int kExpTerms = 19;                      // Taylor polynomial of exp on [0, ln 2)

// ln x for positive finite x: x = m*2^e with m in [sqrt(1/2), sqrt(2)), ln m = 2 atanh((m-1)/(m+1))
// by its odd series, summed from the smallest term.  Truncation error below 1e-19.
double natural_log(double x)
{
    int e = 0;
    double m = std::frexp(x, &e);   // exact
    if (m < kSqrtHalf) { m = m * 2.0; e -= 1; }
    const double z = (m - 1.0) / (m + 1.0);
    const double z2 = z * z;
    double s = 1.0 / static_cast<double>(2 * kLogTerms + 1);
    for (int i = kLogTerms - 1; i >= 0; --i) s = s * z2 + 1.0 / static_cast<double>(2 * i + 1);
    return static_cast<double>(e) * kLn2 + (2.0 * z) * s;
}

double log_base2(double x) { return natural_log(x) / kLn2; }

// 2^y for 0 <= y < 1000: the integer part is an exact scaling, the fraction goes through
// exp(t), t in [0, ln 2), as a nested Taylor polynomial.  Truncation error below 1e-19.
double two_to_the(double y)
{
    const double n = std::floor(y);
    const double t = (y - n) * kLn2;
    double s = 1.0;
    for (int i = kExpTerms; i >= 1; --i) s = 1.0 + (s * t) / static_cast<double>(i);
    return std::ldexp(s, static_cast<int>(n));
}

class KernelStream {
public:
    KernelStream(uint64_t seed, uint64_t k)
        : state_(scramble(scramble(seed + kGolden) + (k + 1) * kGolden)) {}
    uint64_t bits() { state_ += kGolden; return scramble(state_); }
    uint32_t word() { return static_cast<uint32_t>(bits() >> 32); }
    // uniform on [0,1) and on (0,1], 53 bits
    double unit() { return static_cast<double>(bits() >> 11) * 0x1.0p-53; }
    double unit_open() { return static_cast<double>((bits() >> 11) + 1) * 0x1.0p-53; }
    // integer uniform on [0, range) by the multiply-shift map
    uint32_t below(uint32_t range) { return static_cast<uint32_t>((static_cast<uint64_t>(word()) * range) >> 32); }

    // N(0,1) by the ratio of uniforms: the point (u, v) is uniform on
    // (0,1] x [-sqrt(2/e), sqrt(2/e)); v/u is kept when (v/u)^2 <= -4 ln u.
    double gauss()
    {
        for (;;) {
            const double u = unit_open();
            const double v = 0.8577638849607068 * (2.0 * unit() - 1.0);
            const double ratio = v / u;
            if (ratio * ratio <= -4.0 * natural_log(u)) return ratio;
        }
    }

private:
    uint64_t state_;
};

}  // namespace

void rk_sample_kernels(uint64_t seed, rocket_kernels &h)
{
    const int32_t K = h.K, C = h.C, L = h.L;
    h.length.resize(K); h.dilation.resize(K); h.padding.resize(K);
    h.n_ch.resize(K); h.bias.resize(K);
    h.channels.clear(); h.weights.clear();
    const int32_t max_ch = C < 9 ? C : 9;
    const double ch_span = log_base2(static_cast<double>(max_ch + 1));
    std::vector<int32_t> pool(C);
    std::vector<double> row(11);

    for (int32_t k = 0; k < K; ++k) {
        KernelStream rng(seed, static_cast<uint64_t>(k));
        const int32_t len = 7 + 2 * static_cast<int32_t>(rng.below(3));

        int32_t nch = static_cast<int32_t>(std::floor(two_to_the(rng.unit() * ch_span)));
        if (nch < 1) nch = 1;
        if (nch > max_ch) nch = max_ch;

        std::iota(pool.begin(), pool.end(), 0);
        for (int32_t i = 0; i < nch; ++i) {
            const int32_t j = i + static_cast<int32_t>(rng.below(static_cast<uint32_t>(C - i)));
            std::swap(pool[i], pool[j]);
            h.channels.push_back(pool[i]);
        }

        for (int32_t c = 0; c < nch; ++c) {
            double total = 0.0;
            for (int32_t j = 0; j < len; ++j) { row[j] = rng.gauss(); total += row[j]; }
            const double mean = total / static_cast<double>(len);
            for (int32_t j = 0; j < len; ++j) h.weights.push_back(static_cast<float>(row[j] - mean));
        }

        h.bias[k] = static_cast<float>(static_cast<double>(rng.word() >> 8) * 0x1.0p-23 - 1.0);

        const double span = log_base2(static_cast<double>(L - 1) / static_cast<double>(len - 1));
        int32_t dil = static_cast<int32_t>(std::floor(two_to_the(rng.unit() * span)));
        const int32_t dil_max = (L - 1) / (len - 1);
        if (dil < 1) dil = 1;
        if (dil > dil_max) dil = dil_max;

        const bool same = (rng.word() & 1u) != 0;
        h.length[k] = len;
        h.n_ch[k] = nch;
        h.dilation[k] = dil;
        h.padding[k] = same ? ((len - 1) * dil) / 2 : 0;
    }
}

// ------------------------------------------------------------------ MINIROCKET-style kernels
//
// The paper's related-work section describes MINIROCKET as: two-valued ("binary") kernels, so that the
// convolution can be done by additions; weights from a predetermined set; biases sampled from the input
// data; PPV as the only pooled feature.  This build's reading of the rest: length 9, weights -1 and 2 with
// three 2s (zero sum, like the mean-centred weights of section 3.1), the predetermined set being all
// C(9,3) = 84 such kernels in lexicographic order of the positions of the 2s; kernels come in groups of 84
// that share dilation, padding and channel subset, drawn per group by the laws of section 3.1 from the
// stream of (seed, group): channel count, channels, dilation, padding.

void rk_sample_minirocket(uint64_t seed, int32_t groups, rocket_kernels &h)
{
    const int32_t C = h.C, L = h.L;
    constexpr int32_t kLen = 9, kSet = 84;
    const int32_t K = groups * kSet;
    h.K = K;
    h.length.assign(K, kLen); h.dilation.resize(K); h.padding.resize(K);
    h.n_ch.resize(K); h.bias.assign(K, 0.f);
    h.channels.clear(); h.weights.clear();
    const int32_t max_ch = C < 9 ? C : 9;
    const double ch_span = log_base2(static_cast<double>(max_ch + 1));
    std::vector<int32_t> pool(C);
    for (int32_t g = 0; g < groups; ++g) {
        KernelStream rng(seed, static_cast<uint64_t>(g));
        int32_t nch = static_cast<int32_t>(std::floor(two_to_the(rng.unit() * ch_span)));
        if (nch < 1) nch = 1;
        if (nch > max_ch) nch = max_ch;
        std::iota(pool.begin(), pool.end(), 0);
        for (int32_t i = 0; i < nch; ++i) {
            const int32_t j = i + static_cast<int32_t>(rng.below(static_cast<uint32_t>(C - i)));
            std::swap(pool[i], pool[j]);
        }
        const double span = log_base2(static_cast<double>(L - 1) / static_cast<double>(kLen - 1));
        int32_t dil = static_cast<int32_t>(std::floor(two_to_the(rng.unit() * span)));
        const int32_t dil_max = (L - 1) / (kLen - 1);
        if (dil < 1) dil = 1;
        if (dil > dil_max) dil = dil_max;
        const bool same = (rng.word() & 1u) != 0;
        int32_t k = g * kSet;
        for (int32_t a = 0; a < kLen; ++a)
            for (int32_t b = a + 1; b < kLen; ++b)
                for (int32_t c = b + 1; c < kLen; ++c, ++k) {     // lexicographic triples (a, b, c)
                    h.dilation[k] = dil;
                    h.padding[k] = same ? ((kLen - 1) * dil) / 2 : 0;
                    h.n_ch[k] = nch;
                    for (int32_t q = 0; q < nch; ++q) {
                        h.channels.push_back(pool[q]);
                        for (int32_t j = 0; j < kLen; ++j) h.weights.push_back(j == a || j == b || j == c ? 2.f : -1.f);
                    }
                }
    }
}

// Bias draws of kernel k, from the stream of (seed + 1, k): a training example, uniform on [0, n_train), and a
// level q, uniform on [0, 1); the bias will be minus the order statistic of rank floor(q (n_k - 1)) of the
// kernel's bias-free output on that example.
void rk_minirocket_draws(uint64_t seed, const rocket_kernels &h, int32_t n_train, std::vector<int32_t> &example,
                         std::vector<int32_t> &rank)
{
    example.resize(h.K);
    rank.resize(h.K);
    for (int32_t k = 0; k < h.K; ++k) {
        KernelStream rng(seed + 1, static_cast<uint64_t>(k));
        example[k] = static_cast<int32_t>(rng.below(static_cast<uint32_t>(n_train)));
        const double q = rng.unit();
        const int64_t n = static_cast<int64_t>(h.L) + 2LL * h.padding[k] - static_cast<int64_t>(h.length[k] - 1) * h.dilation[k];
        rank[k] = static_cast<int32_t>(std::floor(q * static_cast<double>(n - 1)));
    }
}
