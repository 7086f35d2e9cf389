// Load-adaptive sampler partition (KAITIAN Sec. III-C, phase 2: each device
// receives a portion of every global mini-batch in proportion to its score;
// Sec. IV-A: the DistributedSampler override).  Host only: the index lists are
// consumed by the host-side data loader.
#include <cstddef>
#include <cstdint>
#include <numeric>
#include <vector>

#include "kt.h"

extern void kt_set_error(const char *fmt, ...);

namespace {

// SplitMix64 (Steele, Lea, Flood 2014).
struct Mix64 {
    uint64_t s;
    uint64_t next()
    {
        s += 0x9E3779B97F4A7C15ull;
        uint64_t z = s;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
        z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
        return z ^ (z >> 31);
    }
    // uniform in [0, n), n >= 1: high word of a 64x64 product with the biased
    // low words rejected (Lemire 2019)
    uint64_t below(uint64_t n)
    {
        unsigned __int128 m = (unsigned __int128)next() * n;
        uint64_t low = (uint64_t)m;
        if (low < n) {
            const uint64_t t = (0 - n) % n;
            while (low < t) {
                m = (unsigned __int128)next() * n;
                low = (uint64_t)m;
            }
        }
        return (uint64_t)(m >> 64);
    }
};

kt_status check(int64_t N, int64_t B, const int64_t *shares, int K, int rank, int64_t *start)
{
    if (!shares || K < 1 || K > KT_MAX_PEERS || rank < 0 || rank >= K || N < 0 || B < 1) {
        kt_set_error("kt_sampler: bad N, B, K, rank or NULL shares");
        return KT_EINVAL;
    }
    int64_t sum = 0, before = 0;
    for (int k = 0; k < K; ++k) {
        if (shares[k] < 0 || shares[k] > B) { kt_set_error("kt_sampler: share %d out of range", k); return KT_EINVAL; }
        if (k < rank) before += shares[k];
        sum += shares[k];
    }
    if (sum != B) { kt_set_error("kt_sampler: shares sum to %lld, not B", (long long)sum); return KT_EINVAL; }
    *start = before;
    return KT_OK;
}

}  // namespace

extern "C" kt_status kt_sampler_epoch_size(int64_t N, int64_t B, const int64_t *shares, int K, int rank,
                                           int drop_last, int64_t *count)
{
    int64_t start;
    kt_status st = check(N, B, shares, K, rank, &start);
    if (st != KT_OK) return st;
    if (!count) { kt_set_error("kt_sampler_epoch_size: NULL count"); return KT_EINVAL; }
    const int64_t steps = drop_last ? N / B : (N + B - 1) / B;
    *count = steps * shares[rank];
    return KT_OK;
}

extern "C" kt_status kt_sampler_epoch(int64_t N, int64_t B, const int64_t *shares, int K, uint64_t seed,
                                      uint64_t epoch, int shuffle, int rank, int drop_last, int64_t *out,
                                      int64_t capacity, int64_t *count)
{
    int64_t start;
    kt_status st = check(N, B, shares, K, rank, &start);
    if (st != KT_OK) return st;
    const int64_t steps = drop_last ? N / B : (N + B - 1) / B;
    const int64_t mine = shares[rank];
    const int64_t total = steps * mine;
    if (total > 0 && (!out || capacity < total)) {
        kt_set_error("kt_sampler_epoch: output capacity %lld < %lld", (long long)capacity, (long long)total);
        return KT_EINVAL;
    }
    std::vector<int64_t> order;
    try {
        order.resize((size_t)N);
    } catch (...) {
        kt_set_error("kt_sampler_epoch: out of host memory");
        return KT_ENOMEM;
    }
    std::iota(order.begin(), order.end(), (int64_t)0);
    if (shuffle) {
        Mix64 g{seed + epoch * 0x9E3779B97F4A7C15ull};
        for (int64_t i = N - 1; i >= 1; --i) {
            const int64_t j = (int64_t)g.below((uint64_t)i + 1);
            const int64_t tmp = order[(size_t)i];
            order[(size_t)i] = order[(size_t)j];
            order[(size_t)j] = tmp;
        }
    }
    int64_t w = 0;
    for (int64_t s = 0; s < steps; ++s) {
        const int64_t base = s * B + start;
        for (int64_t i = 0; i < mine; ++i) out[w++] = order[(size_t)((base + i) % N)];
    }
    if (count) *count = total;
    return KT_OK;
}
