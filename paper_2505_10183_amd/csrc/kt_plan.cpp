// Host-only planning: batch shares (KAITIAN Sec. III-C) and the bucket layout
// with its tile table.  No GPU is touched here.  Compile with
// -ffp-contract=off: the share quotas must be plain IEEE double operations.
#include <algorithm>
#include <cmath>
#include <numeric>

#include "kt_internal.h"

extern void kt_set_error(const char *fmt, ...);

extern "C" kt_status kt_plan_shares(const double *thr, int K, int64_t B, int64_t *shares, float *weights)
{
    if (!thr || !shares) { kt_set_error("kt_plan_shares: NULL thr or shares"); return KT_EINVAL; }
    if (K < 1 || K > KT_MAX_PEERS) { kt_set_error("kt_plan_shares: K=%d outside [1,%d]", K, KT_MAX_PEERS); return KT_EINVAL; }
    if (B < 0 || B > ((int64_t)1 << 40)) { kt_set_error("kt_plan_shares: B outside [0, 2^40]"); return KT_EINVAL; }
    if (weights && B == 0) { kt_set_error("kt_plan_shares: weights need B > 0"); return KT_EINVAL; }
    double total = 0.0;
    for (int k = 0; k < K; ++k) {
        if (!(std::isfinite(thr[k]) && thr[k] > 0.0)) {
            kt_set_error("kt_plan_shares: throughput %d is not finite and positive", k);
            return KT_EINVAL;
        }
        total += thr[k];
    }
    if (!std::isfinite(total)) { kt_set_error("kt_plan_shares: throughput sum overflows"); return KT_EINVAL; }

    // Sec. III-C display equation: quota_i = score_i / sum_j score_j * B.
    // Integer part first; the leftover units go to the largest remainders.
    int64_t base[KT_MAX_PEERS];
    double rem[KT_MAX_PEERS];
    int order[KT_MAX_PEERS];
    int64_t given = 0;
    for (int k = 0; k < K; ++k) {
        const double quota = (thr[k] / total) * (double)B;
        const double whole = std::floor(quota);
        base[k] = (int64_t)whole;
        rem[k] = quota - whole;
        given += base[k];
        order[k] = k;
    }
    const int64_t left = B - given;
    if (left < 0 || left > K) { kt_set_error("kt_plan_shares: remainder %lld out of range", (long long)left); return KT_EINVAL; }
    std::stable_sort(order, order + K, [&](int a, int b) { return rem[a] > rem[b]; });
    for (int64_t i = 0; i < left; ++i) base[order[i]] += 1;

    for (int k = 0; k < K; ++k) shares[k] = base[k];
    if (weights)
        for (int k = 0; k < K; ++k) weights[k] = (float)base[k] / (float)B;
    return KT_OK;
}

// Online adaptation (Sec. III-C phase 1): exponential moving average of the
// measured time per sample of every device, then the shares for speeds 1/ema.
extern "C" kt_status kt_replan_shares(const double *step_time, const int64_t *shares_used, double *ema, double alpha,
                                      int K, int64_t B, int64_t *shares, float *weights)
{
    if (!step_time || !shares_used || !ema || !shares) { kt_set_error("kt_replan_shares: NULL argument"); return KT_EINVAL; }
    if (K < 1 || K > KT_MAX_PEERS) { kt_set_error("kt_replan_shares: K=%d outside [1,%d]", K, KT_MAX_PEERS); return KT_EINVAL; }
    if (!(alpha > 0.0 && alpha <= 1.0)) { kt_set_error("kt_replan_shares: alpha outside (0,1]"); return KT_EINVAL; }
    double next[KT_MAX_PEERS], speed[KT_MAX_PEERS];
    for (int k = 0; k < K; ++k) {
        double e = ema[k];
        if (shares_used[k] < 0) { kt_set_error("kt_replan_shares: negative sample count for device %d", k); return KT_EINVAL; }
        if (shares_used[k] > 0) {
            if (!(std::isfinite(step_time[k]) && step_time[k] > 0.0)) {
                kt_set_error("kt_replan_shares: step time of device %d is not finite and positive", k);
                return KT_EINVAL;
            }
            const double tau = step_time[k] / (double)shares_used[k];
            e = !(e > 0.0) ? tau : alpha * tau + (1.0 - alpha) * e;
        }
        if (!(e > 0.0 && std::isfinite(e))) { kt_set_error("kt_replan_shares: no speed estimate for device %d", k); return KT_EINVAL; }
        next[k] = e;
        speed[k] = 1.0 / e;
    }
    int64_t b[KT_MAX_PEERS];
    float w[KT_MAX_PEERS];
    kt_status st = kt_plan_shares(speed, K, B, b, weights ? w : nullptr);
    if (st != KT_OK) return st;
    for (int k = 0; k < K; ++k) { ema[k] = next[k]; shares[k] = b[k]; }
    if (weights)
        for (int k = 0; k < K; ++k) weights[k] = w[k];
    return KT_OK;
}

// Two-level weights (Sec. III-A): inside group g device k weighs b_k / B_g,
// across groups group g weighs B_g / B.
extern "C" kt_status kt_plan_group_weights(const int64_t *shares, int K, const int *group_of, int G,
                                           float *w_intra, float *w_inter, int64_t *group_batch)
{
    if (!shares || !group_of || !w_intra || !w_inter) { kt_set_error("kt_plan_group_weights: NULL argument"); return KT_EINVAL; }
    if (K < 1 || K > KT_MAX_PEERS || G < 1 || G > K) { kt_set_error("kt_plan_group_weights: need 1 <= G <= K <= %d", KT_MAX_PEERS); return KT_EINVAL; }
    int64_t per_group[KT_MAX_PEERS] = {0};
    int64_t total = 0;
    for (int k = 0; k < K; ++k) {
        if (group_of[k] < 0 || group_of[k] >= G) { kt_set_error("kt_plan_group_weights: group of device %d outside [0,%d)", k, G); return KT_EINVAL; }
        if (shares[k] < 0 || shares[k] > ((int64_t)1 << 40)) { kt_set_error("kt_plan_group_weights: share %d out of range", k); return KT_EINVAL; }
        per_group[group_of[k]] += shares[k];
        total += shares[k];
    }
    for (int g = 0; g < G; ++g)
        if (per_group[g] <= 0) { kt_set_error("kt_plan_group_weights: group %d has no samples", g); return KT_EINVAL; }
    for (int k = 0; k < K; ++k) w_intra[k] = (float)shares[k] / (float)per_group[group_of[k]];
    for (int g = 0; g < G; ++g) w_inter[g] = (float)per_group[g] / (float)total;
    if (group_batch)
        for (int g = 0; g < G; ++g) group_batch[g] = per_group[g];
    return KT_OK;
}

static inline int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

kt_status kt_build_host_plan(const int64_t *numel, int T, kt_dtype dt, int64_t cap_bytes, int align_bytes,
                             KtHostPlan &hp, const char **msg)
{
    const int es = dt == KT_F32 ? 4 : 2;
    if (dt != KT_F32 && dt != KT_BF16) { *msg = "unknown dtype"; return KT_EINVAL; }
    if (T < 0 || (T > 0 && !numel)) { *msg = "bad tensor list"; return KT_EINVAL; }
    if (cap_bytes < 0) { *msg = "negative cap_bytes"; return KT_EINVAL; }
    if (align_bytes < es || align_bytes > KT_TILE_BYTES || (align_bytes & (align_bytes - 1)) || align_bytes % es) {
        *msg = "align_bytes must be a power of two in [element size, 16384]";
        return KT_EINVAL;
    }
    const int64_t A = align_bytes / es;
    const int64_t limit = INT64_MAX / 64;
    hp.dt = dt;
    hp.elem_size = es;
    hp.cap_bytes = cap_bytes;
    hp.align_bytes = align_bytes;
    hp.tile_elems = KT_TILE_BYTES / es;

    hp.t_numel.assign(numel, numel + T);
    hp.t_off.resize(T);
    hp.t_bucket.resize(T);
    int64_t fill = 0;      // end of the last tensor placed in the open bucket
    int placed = 0;        // tensors in the open bucket
    for (int t = 0; t < T; ++t) {
        const int64_t n = numel[t];
        if (n < 0 || n > limit) { *msg = "tensor element count out of range"; return KT_EINVAL; }
        int64_t at = round_up(fill, A);
        if (at > limit) { *msg = "bucket too large"; return KT_EUNSUPPORTED; }
        const bool overflow = cap_bytes > 0 && placed > 0 && round_up(at + n, A) * es > cap_bytes;
        if (overflow) {
            hp.b_count.push_back(placed);
            hp.b_elems.push_back(round_up(fill, A));
            fill = 0; placed = 0; at = 0;
        }
        if (placed == 0) hp.b_first.push_back(t);
        hp.t_bucket[t] = (int32_t)hp.b_first.size() - 1;
        hp.t_off[t] = at;
        fill = at + n;
        ++placed;
    }
    if (placed > 0) {
        hp.b_count.push_back(placed);
        hp.b_elems.push_back(round_up(fill, A));
    }

    // Tile table.  For each tile: the first tensor whose data reaches past the
    // tile start, and how many tensors begin before the tile end.
    const int nb = (int)hp.b_elems.size();
    hp.b_tile0.assign(nb + 1, 0);
    for (int b = 0; b < nb; ++b) {
        const int64_t ntile = (hp.b_elems[b] + hp.tile_elems - 1) / hp.tile_elems;
        hp.b_tile0[b + 1] = hp.b_tile0[b] + ntile;
    }
    // one workgroup of KT_BLOCK lanes per tile; a dispatch holds fewer than 2^32 work-items
    if (hp.b_tile0[nb] * KT_BLOCK >= ((int64_t)1 << 32)) { *msg = "plan too large: 2^24 or more tiles"; return KT_EUNSUPPORTED; }
    hp.tiles.resize((size_t)hp.b_tile0[nb]);
    const int VE = KT_VEC_BYTES / es;
    for (int b = 0; b < nb; ++b) {
        const int tb = hp.b_first[b], te = tb + hp.b_count[b];
        int t = tb;
        const int64_t ntile = hp.b_tile0[b + 1] - hp.b_tile0[b];
        for (int64_t k = 0; k < ntile; ++k) {
            const int64_t s = k * hp.tile_elems;
            const int64_t e = std::min(s + hp.tile_elems, hp.b_elems[b]);
            while (t < te - 1 && hp.t_off[t] + hp.t_numel[t] <= s) ++t;
            int last = t;
            while (last + 1 < te && hp.t_off[last + 1] < e) ++last;
            KtTile &tl = hp.tiles[(size_t)(hp.b_tile0[b] + k)];
            tl.bucket = b;
            tl.tile_in_bucket = (uint32_t)k;
            tl.t0 = t;
            const bool solid = last == t && hp.t_off[t] <= s && hp.t_off[t] + hp.t_numel[t] >= e && (e - s) % VE == 0;
            tl.nt = solid ? 0 : last - t + 1;
        }
    }
    return KT_OK;
}
