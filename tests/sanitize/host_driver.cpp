// Drives the host-only code of the library (kernel sampler, import validation, job planner, parameter
// updates, pruning, the MINIROCKET-style kernel set) so that it can run under AddressSanitizer and
// UndefinedBehaviorSanitizer without a GPU.  Linked with sampler.cpp and rocket_api.hip compiled for the host
// only; the kernel launchers that rocket_api.hip refers to are replaced by stubs that must never be reached.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "rocket_internal.hpp"

#define STUB(name) { std::fprintf(stderr, "stub reached: %s\n", name); std::abort(); }
int rk_launch_pad(const rocket_kernels *, const float *, int32_t, float *, void *) STUB("pad")
int rk_launch_mse_grad(const double *, const float *, const double *, int32_t, int32_t, float *, double *, void *) STUB("mse")
int rk_launch_sgd_update(const rocket_kernels *, const float *, const float *, float, int, void *) STUB("sgd")
int rk_launch_pad_u8(const rocket_kernels *, const uint8_t *, int32_t, float *, void *, void *) STUB("pad_u8")
int rk_launch_forward(const rocket_kernels *, const float *, int32_t, uint32_t, float, float, float *, void *) STUB("forward")
int rk_launch_forward_short(const rocket_kernels *, const float *, int32_t, uint32_t, float, float, float *, void *) STUB("short")
int rk_launch_finalize(const rocket_kernels *, const float *, int32_t, uint32_t, float *, void *) STUB("finalize")
int rk_launch_backward(const rocket_kernels *, const float *, int32_t, const float *, int, int, int, float, float, float,
                       float *, void *) STUB("backward")
int rk_launch_reduce_jobs(const rocket_kernels *, const float *, const float *, int32_t, const float *, int, int, float *,
                          float *, void *) STUB("reduce")
int rk_launch_minirocket_outputs(const rocket_kernels *, const float *, const int32_t *, int32_t, int32_t, int64_t, float *,
                                 void *) STUB("mr_outputs")
int rk_launch_minirocket_select(const rocket_kernels *, const int32_t *, int32_t, int32_t, int64_t, const float *, void *)
    STUB("mr_select")
int rk_launch_minirocket_clear(const rocket_kernels *, int32_t, int32_t *, void *) STUB("mr_clear")
int rk_launch_minirocket_forward(const rocket_kernels *, const float *, int32_t, int32_t *, void *) STUB("mr_forward")
int rk_launch_minirocket_features(const rocket_kernels *, const int32_t *, int32_t, float *, void *) STUB("mr_features")
extern "C" int rocket_ridge_predict(const float *, int32_t, int32_t, const double *, const double *, double *, void *)
    STUB("ridge_predict")

#define CHECK(cond) do { if (!(cond)) { std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

static int exercise(uint64_t seed, int K, int C, int L)
{
    rocket_kernels *h = nullptr;
    CHECK(rocket_make_kernels(seed, K, C, L, &h) == ROCKET_OK);
    rocket_kernels_view v;
    CHECK(rocket_kernels_view_get(h, &v) == ROCKET_OK);
    CHECK(v.K == K && v.total_weights == v.w_off[K] && v.total_channels == v.ch_off[K]);
    // the jobs partition every kernel's rows
    int32_t count = 0, stride = 0;
    const int32_t *kernel, *row0, *row1, *flags;
    CHECK(rocket_jobs_view_get(h, &count, &kernel, &row0, &row1, &flags, &stride) == ROCKET_OK);
    std::vector<long long> covered(K, 0);
    for (int32_t j = 0; j < count; ++j) {
        const char *base = reinterpret_cast<const char *>(kernel) + static_cast<size_t>(j) * stride;
        const int32_t *rec = reinterpret_cast<const int32_t *>(base);      // kernel, row0, row1, flags
        CHECK(rec[0] >= 0 && rec[0] < K && rec[2] >= rec[1]);
        covered[rec[0]] += rec[2] - rec[1];
    }
    for (int k = 0; k < K; ++k) {
        const long long n = static_cast<long long>(L) + 2LL * v.padding[k] - static_cast<long long>(v.length[k] - 1) * v.dilation[k];
        CHECK(n >= 1 && covered[k] == n / v.dilation[k]);
    }
    CHECK(rocket_workspace_bytes(h, 3, 7, 0) > 0 && rocket_workspace_bytes(h, 3, 5, 1) > 0);
    CHECK(rocket_train_workspace_bytes(h, 3, 5) > 0);
    double fma = 0, outs = 0;
    CHECK(rocket_work_per_series(h, &fma, &outs) == ROCKET_OK && fma > 0 && outs > 0);
    // round trip through import, parameter replacement (one rejected), pruning
    rocket_kernels *h2 = nullptr;
    CHECK(rocket_kernels_import(K, C, L, v.length, v.dilation, v.padding, v.bias, v.n_ch, v.channels, v.weights, &h2) == ROCKET_OK);
    std::vector<float> w(v.weights, v.weights + v.total_weights), b(v.bias, v.bias + K);
    for (auto &x : w) x *= 0.5f;
    CHECK(rocket_kernels_set_params(h2, w.data(), nullptr) == ROCKET_OK);
    b[K / 2] = NAN;
    CHECK(rocket_kernels_set_params(h2, w.data(), b.data()) == ROCKET_EINVAL);
    std::vector<int32_t> bad_len(v.length, v.length + K);
    bad_len[0] = 8;
    rocket_kernels *h3 = nullptr;
    CHECK(rocket_kernels_import(K, C, L, bad_len.data(), v.dilation, v.padding, v.bias, v.n_ch, v.channels, v.weights, &h3) == ROCKET_ESHAPE);
    std::vector<int32_t> keep = {K - 1, 0, K / 2, K - 1};
    CHECK(rocket_kernels_subset(h2, keep.data(), static_cast<int32_t>(keep.size()), &h3) == ROCKET_OK);
    keep[1] = K;
    rocket_kernels *h4 = nullptr;
    CHECK(rocket_kernels_subset(h2, keep.data(), static_cast<int32_t>(keep.size()), &h4) == ROCKET_EINVAL);
    // compute entry points reject bad arguments before touching a GPU
    float dummy;
    CHECK(rocket_transform(h, &dummy, 0, 3, 10.f, -3.f, &dummy, &dummy, 1u << 30, nullptr) == ROCKET_EINVAL);
    CHECK(rocket_transform(h, &dummy, 1, 3, 10.f, -3.f, &dummy, &dummy, 16, nullptr) == ROCKET_EWORKSPACE);
    CHECK(rocket_transform_noalloc(h, &dummy, 1, 3, 10.f, -3.f, &dummy, nullptr) == ROCKET_EINVAL);
    rocket_free_kernels(h);
    rocket_free_kernels(h2);
    rocket_free_kernels(h3);
    return 0;
}

int main()
{
    if (exercise(2000, 300, 1, 512)) return 1;
    if (exercise(2002, 400, 20, 50000)) return 1;
    if (exercise(7, 120, 40, 333)) return 1;
    if (exercise(0, 64, 3, 11)) return 1;
    if (exercise(5, 100, 5, 200001)) return 1;
    rocket_kernels *m = nullptr;
    if (rocket_minirocket_kernels(3, 7, 20, 50000, &m) != ROCKET_OK) return 1;
    rocket_kernels_view v;
    if (rocket_kernels_view_get(m, &v) != ROCKET_OK || v.K != 7 * 84) return 1;
    if (rocket_minirocket_fit_workspace_bytes(m, 2) == 0) return 1;
    if (rocket_minirocket_workspace_bytes(m, 2) == 0) return 1;
    rocket_free_kernels(m);
    // the plan of the group kernel at sizes around its tile limits (short series, one position, long series)
    const int shapes[][3] = {{1, 1, 9}, {3, 2, 10}, {5, 3, 73}, {9, 1, 4105}, {4, 20, 8193}, {2, 9, 200001}};
    for (const auto &sh : shapes) {
        if (rocket_minirocket_kernels(11, sh[0], sh[1], sh[2], &m) != ROCKET_OK) return 1;
        if (rocket_minirocket_workspace_bytes(m, 3) == 0) return 1;
        rocket_free_kernels(m);
    }
    if (rocket_minirocket_kernels(3, 0, 20, 50000, &m) != ROCKET_EINVAL) return 1;
    std::puts("host driver: ok");
    return 0;
}
