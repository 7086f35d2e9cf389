// The C ABI used from a plain HIP program: no Python, no PyTorch, device memory from hipMalloc,
// the default stream and a stream of its own.  Runs pack -> K-way weighted reduce -> unpack-scale,
// the fused single pass, the entry point that allocates nothing, SGD on unpack and the one-pass
// reduce + SGD (by value, then with resident weights and scalars) on a small ragged gradient set and compares every element with the CPU checker's C functions (strict
// binary32 mode: bit-identical).  Test infrastructure: links libkt.so and libkt_oracle.so.
// Prints "ok ..." and exits 0, or names the first mismatch and exits 1.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "kt.h"

extern "C" {
void kto_reduce_f32_S(const float *const *x, const float *w, int K, int64_t n, float *out);
void kto_scale_f32(const float *in, int64_t n, float scale, float *out);
void kto_sgd_f32_S(const float *x, int64_t n, float scale, float *p, float *v, float lr, float mu, float wd, int first);
}

#define HIP_OK(call)                                                                         \
    do {                                                                                     \
        hipError_t e_ = (call);                                                              \
        if (e_ != hipSuccess) { printf("%s: %s\n", #call, hipGetErrorString(e_)); return 1; } \
    } while (0)
#define KT_OKAY(call)                                                                  \
    do {                                                                               \
        kt_status s_ = (call);                                                         \
        if (s_ != KT_OK) { printf("%s: %s: %s\n", #call, kt_status_string(s_), kt_last_error()); return 1; } \
    } while (0)

static uint64_t g_state = 0x243F6A8885A308D3ull;
static float next_value()
{
    g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
    return (float)((int64_t)(g_state >> 40) - (1 << 23)) * (1.0f / (1 << 23)) * 1e-2f;   // uniform in [-0.01, 0.01)
}

static bool same(const std::vector<float> &a, const std::vector<float> &b, const char *what, int t)
{
    if (a.size() != b.size() || memcmp(a.data(), b.data(), a.size() * 4) != 0) {
        for (size_t i = 0; i < a.size() && i < b.size(); ++i)
            if (memcmp(&a[i], &b[i], 4) != 0) { printf("%s, tensor %d, element %zu: got %a want %a\n", what, t, i, a[i], b[i]); break; }
        return false;
    }
    return true;
}

int main()
{
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) { printf("skip: no GPU\n"); return 77; }
    HIP_OK(hipSetDevice(0));

    const int K = 3;
    const std::vector<int64_t> numel = {5, 70001, 3, 4096, 1, 12345, 8193, 7, 40000};
    const int T = (int)numel.size();
    const double thr[K] = {1.0, 0.6, 0.4};
    int64_t shares[K];
    float w[K];
    KT_OKAY(kt_plan_shares(thr, K, 96, shares, w));
    if (shares[0] + shares[1] + shares[2] != 96) { printf("shares do not sum to B\n"); return 1; }

    kt_plan *plan = nullptr;
    KT_OKAY(kt_plan_create(numel.data(), T, KT_F32, 96 * 1024, 16, &plan));
    const int nb = kt_plan_num_buckets(plan);
    std::vector<int64_t> belems(nb);
    for (int b = 0; b < nb; ++b) KT_OKAY(kt_plan_bucket_info(plan, b, &belems[b], nullptr, nullptr));

    // host copies of the K gradient sets and their device tensors
    std::vector<std::vector<std::vector<float>>> hg(K, std::vector<std::vector<float>>(T));
    std::vector<std::vector<void *>> dg(K, std::vector<void *>(T, nullptr));
    for (int k = 0; k < K; ++k)
        for (int t = 0; t < T; ++t) {
            hg[k][t].resize((size_t)numel[t]);
            for (float &x : hg[k][t]) x = next_value();
            HIP_OK(hipMalloc(&dg[k][t], (size_t)numel[t] * 4));
            HIP_OK(hipMemcpy(dg[k][t], hg[k][t].data(), (size_t)numel[t] * 4, hipMemcpyHostToDevice));
        }
    // K peer copies of every bucket, one output bucket, result tensors (three sets)
    std::vector<std::vector<void *>> slot(K, std::vector<void *>(nb, nullptr));
    std::vector<void *> red(nb, nullptr);
    for (int b = 0; b < nb; ++b) {
        for (int k = 0; k < K; ++k) HIP_OK(hipMalloc(&slot[k][b], (size_t)belems[b] * 4));
        HIP_OK(hipMalloc(&red[b], (size_t)belems[b] * 4));
    }
    std::vector<void *> res(T), res_fused(T), res_na(T), par(T), mom(T);
    for (int t = 0; t < T; ++t) {
        for (std::vector<void *> *v : {&res, &res_fused, &res_na, &par, &mom}) HIP_OK(hipMalloc(&(*v)[t], (size_t)numel[t] * 4));
    }

    hipStream_t side;
    HIP_OK(hipStreamCreate(&side));
    const float scale = 0.37f;

    // chained path on the default stream (NULL)
    for (int k = 0; k < K; ++k) KT_OKAY(kt_bucket_pack(plan, KT_ALL_BUCKETS, dg[k].data(), slot[k].data(), nullptr));
    std::vector<const void *> peers((size_t)nb * K);
    for (int b = 0; b < nb; ++b)
        for (int k = 0; k < K; ++k) peers[(size_t)b * K + k] = slot[k][b];
    KT_OKAY(kt_weighted_reduce(plan, KT_ALL_BUCKETS, peers.data(), K, w, red.data(), nullptr));
    KT_OKAY(kt_bucket_unpack_scale(plan, KT_ALL_BUCKETS, red.data(), scale, res.data(), nullptr));
    HIP_OK(hipDeviceSynchronize());
    // fused pass and the entry point that allocates nothing, on a stream of their own
    std::vector<const void *> others((size_t)nb * (K - 1));
    for (int b = 0; b < nb; ++b)
        for (int k = 1; k < K; ++k) others[(size_t)b * (K - 1) + (k - 1)] = slot[k][b];
    KT_OKAY(kt_fused_step(plan, KT_ALL_BUCKETS, dg[0].data(), others.data(), K, w, scale, res_fused.data(), side));
    KT_OKAY(kt_fused_step_noalloc(plan, KT_ALL_BUCKETS, dg[0].data(), others.data(), K, w, scale, res_na.data(), side));
    HIP_OK(hipStreamSynchronize(side));

    // expected values: the checker's strict functions on the un-bucketed tensors
    int bad = 0;
    std::vector<std::vector<float>> want(T);
    for (int t = 0; t < T; ++t) {
        const size_t n = (size_t)numel[t];
        const float *xs[K] = {hg[0][t].data(), hg[1][t].data(), hg[2][t].data()};
        std::vector<float> sum(n);
        want[t].resize(n);
        kto_reduce_f32_S(xs, w, K, (int64_t)n, sum.data());
        kto_scale_f32(sum.data(), (int64_t)n, scale, want[t].data());
        std::vector<float> got(n);
        for (auto pr : {std::make_pair(res[t], "pack/reduce/unpack"), std::make_pair(res_fused[t], "fused pass"),
                        std::make_pair(res_na[t], "fused pass without allocation")}) {
            HIP_OK(hipMemcpy(got.data(), pr.first, n * 4, hipMemcpyDeviceToHost));
            if (!same(got, want[t], pr.second, t)) ++bad;
        }
    }

    // SGD on unpack, two steps off the reduced buckets
    std::vector<std::vector<float>> hp(T), hv(T);
    for (int t = 0; t < T; ++t) {
        hp[t].resize((size_t)numel[t]);
        hv[t].assign((size_t)numel[t], 0.0f);
        for (float &x : hp[t]) x = next_value() * 100.0f;
        HIP_OK(hipMemcpy(par[t], hp[t].data(), (size_t)numel[t] * 4, hipMemcpyHostToDevice));
        HIP_OK(hipMemset(mom[t], 0xFF, (size_t)numel[t] * 4));     // NaN: not to be read on the first step
    }
    for (int step = 0; step < 2; ++step) {
        KT_OKAY(kt_bucket_unpack_sgd(plan, KT_ALL_BUCKETS, red.data(), scale, par.data(), mom.data(), 0.1f, 0.9f, 5e-4f,
                                     step == 0, side));
        HIP_OK(hipStreamSynchronize(side));
        for (int t = 0; t < T; ++t) {
            const size_t n = (size_t)numel[t];
            // the reduced bucket values of this tensor are want[t] / scale before scaling: recompute the sum
            const float *xs[K] = {hg[0][t].data(), hg[1][t].data(), hg[2][t].data()};
            std::vector<float> sum(n), got(n);
            kto_reduce_f32_S(xs, w, K, (int64_t)n, sum.data());
            kto_sgd_f32_S(sum.data(), (int64_t)n, scale, hp[t].data(), hv[t].data(), 0.1f, 0.9f, 5e-4f, step == 0);
            HIP_OK(hipMemcpy(got.data(), par[t], n * 4, hipMemcpyDeviceToHost));
            if (!same(got, hp[t], "SGD parameters", t)) ++bad;
            HIP_OK(hipMemcpy(got.data(), mom[t], n * 4, hipMemcpyDeviceToHost));
            if (!same(got, hv[t], "SGD momentum", t)) ++bad;
        }
    }

    // the same two steps in one pass from the local tensors and the peer buckets, with the weights and the
    // optimizer scalars resident on the device for the second step
    std::vector<void *> par2(T), mom2(T);
    std::vector<std::vector<float>> hp2(T), hv2(T);
    g_state = 0x13198A2E03707344ull;
    for (int t = 0; t < T; ++t) {
        HIP_OK(hipMalloc(&par2[t], (size_t)numel[t] * 4));
        HIP_OK(hipMalloc(&mom2[t], (size_t)numel[t] * 4));
        hp2[t].resize((size_t)numel[t]);
        hv2[t].assign((size_t)numel[t], 0.0f);
        for (float &x : hp2[t]) x = next_value() * 100.0f;
        HIP_OK(hipMemcpy(par2[t], hp2[t].data(), (size_t)numel[t] * 4, hipMemcpyHostToDevice));
        HIP_OK(hipMemset(mom2[t], 0xFF, (size_t)numel[t] * 4));
    }
    for (int step = 0; step < 2; ++step) {
        const float lr = step == 0 ? 0.1f : 0.01f;
        if (step == 0) {
            KT_OKAY(kt_fused_step_sgd(plan, KT_ALL_BUCKETS, dg[0].data(), others.data(), K, w, scale, par2.data(), mom2.data(),
                                      nullptr, lr, 0.9f, 5e-4f, 1, side));
        } else {
            KT_OKAY(kt_plan_set_weights(plan, w, K, side));
            KT_OKAY(kt_plan_set_sgd(plan, scale, lr, 0.9f, 5e-4f, side));
            KT_OKAY(kt_fused_step_sgd_resident(plan, KT_ALL_BUCKETS, dg[0].data(), others.data(), K, par2.data(), mom2.data(),
                                               nullptr, 0, side));
        }
        HIP_OK(hipStreamSynchronize(side));
        for (int t = 0; t < T; ++t) {
            const size_t n = (size_t)numel[t];
            const float *xs[K] = {hg[0][t].data(), hg[1][t].data(), hg[2][t].data()};
            std::vector<float> sum(n), got(n);
            kto_reduce_f32_S(xs, w, K, (int64_t)n, sum.data());
            kto_sgd_f32_S(sum.data(), (int64_t)n, scale, hp2[t].data(), hv2[t].data(), lr, 0.9f, 5e-4f, step == 0);
            HIP_OK(hipMemcpy(got.data(), par2[t], n * 4, hipMemcpyDeviceToHost));
            if (!same(got, hp2[t], "one-pass SGD parameters", t)) ++bad;
            HIP_OK(hipMemcpy(got.data(), mom2[t], n * 4, hipMemcpyDeviceToHost));
            if (!same(got, hv2[t], "one-pass SGD momentum", t)) ++bad;
        }
    }

    // errors come back as codes, with a message, and leave the plan usable
    if (kt_weighted_reduce(plan, nb, peers.data(), K, w, red.data(), nullptr) != KT_EINVAL || !*kt_last_error()) { printf("bad bucket not refused\n"); ++bad; }
    KT_OKAY(kt_weighted_reduce(plan, 0, peers.data(), K, w, red.data(), nullptr));
    HIP_OK(hipDeviceSynchronize());
    KT_OKAY(kt_plan_destroy(plan));
    HIP_OK(hipStreamDestroy(side));
    if (bad) { printf("%d mismatches\n", bad); return 1; }
    printf("ok %s: %d tensors, %d buckets, K=%d; chained, fused, no-allocation, SGD and one-pass SGD paths equal the checker\n",
           kt_version(), T, nb, K);
    return 0;
}
