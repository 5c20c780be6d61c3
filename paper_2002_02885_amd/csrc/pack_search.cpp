// Host logic of the pack-aware hyper-parameter search (paper Section 5): which configurations of a
// Hyperband rung train together in one pack.  No GPU work happens here; the caller trains the groups
// with the packed step.
//
//   pack_opt_knn        Section 5.2: a random configuration among those not yet grouped becomes the
//                       centroid; the others join it nearest first while they are within the
//                       similarity threshold and the device memory has room.
//   pack_opt_random     Section 5.3, "Random Pack": m randomly chosen configurations per group.
//   pack_opt_batchsize  Section 5.3, "Batch-size Pack": only equal batch sizes share a group.
//   pack_hyperband_plan the rungs (n_i, r_i) of every bracket (Section 5.1, Algorithm 1; sizes as in
//                       the Hyperband paper it cites), pack_halving_keep the survivors of a rung.
//
// The distance between two configurations follows the worked example of Section 5.2 (value 5 for
// four index steps of batch size plus a different optimiser): numeric dimensions contribute the
// absolute difference of their table indices, categorical ones 0 or 1, and the contributions add.
#include "../../include/pack.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <numeric>
#include <string>
#include <vector>

namespace packk {
pack_status set_error(pack_status s, const std::string& msg);
}
using packk::set_error;

namespace {

int dist(const int32_t* a, const int32_t* b, const uint8_t* categorical, int D) {
    int d = 0;
    for (int j = 0; j < D; ++j) d += categorical[j] ? (a[j] != b[j]) : std::abs(a[j] - b[j]);
    return d;
}

}  // namespace

extern "C" {

int32_t pack_config_distance(const int32_t* a, const int32_t* b, const uint8_t* categorical, int32_t n_dims) {
    if (!a || !b || !categorical || n_dims < 1) return -1;
    return dist(a, b, categorical, n_dims);
}

pack_status pack_opt_knn(const int32_t* feats, const uint8_t* categorical, int32_t T, int32_t D, const uint64_t* need,
                         uint64_t capacity, int32_t threshold, const double* draws, int32_t* group_out, int32_t* n_groups) {
    if (!feats || !categorical || !need || !draws || !group_out || !n_groups) return set_error(PACK_EINVAL, "null argument");
    if (T < 1 || D < 1 || threshold < 0) return set_error(PACK_EINVAL, "need T >= 1, D >= 1, threshold >= 0");
    std::vector<int> remaining(T);
    std::iota(remaining.begin(), remaining.end(), 0);
    std::vector<std::pair<int, int>> cand;   // (distance, position in `remaining`)
    int groups = 0;
    while (!remaining.empty()) {
        const double u = draws[groups];
        if (!(u >= 0.0 && u < 1.0)) return set_error(PACK_EINVAL, "draws must lie in [0, 1)");
        const size_t at = (size_t)std::floor(u * (double)remaining.size());
        const int c = remaining[at];
        remaining.erase(remaining.begin() + (long)at);
        group_out[c] = groups;
        uint64_t used = need[c];
        cand.clear();
        for (size_t i = 0; i < remaining.size(); ++i) {
            const int d = dist(feats + (size_t)c * D, feats + (size_t)remaining[i] * D, categorical, D);
            if (d <= threshold) cand.push_back({d, (int)i});
        }
        std::stable_sort(cand.begin(), cand.end(), [](const std::pair<int, int>& x, const std::pair<int, int>& y) { return x.first < y.first; });
        std::vector<char> taken(remaining.size(), 0);
        for (const auto& cd : cand) {
            const int i = remaining[(size_t)cd.second];
            if (need[i] <= capacity && used <= capacity - need[i]) {
                used += need[i];
                group_out[i] = groups;
                taken[(size_t)cd.second] = 1;
            }
        }
        std::vector<int> rest;
        rest.reserve(remaining.size());
        for (size_t i = 0; i < remaining.size(); ++i)
            if (!taken[i]) rest.push_back(remaining[i]);
        remaining.swap(rest);
        ++groups;
    }
    *n_groups = groups;
    return PACK_OK;
}

pack_status pack_opt_random(int32_t T, int32_t m, const int32_t* perm, int32_t* group_out, int32_t* n_groups) {
    if (!perm || !group_out || !n_groups) return set_error(PACK_EINVAL, "null argument");
    if (T < 1 || m < 1) return set_error(PACK_EINVAL, "need T >= 1 and m >= 1");
    std::vector<char> seen((size_t)T, 0);
    for (int i = 0; i < T; ++i) {
        if (perm[i] < 0 || perm[i] >= T || seen[(size_t)perm[i]]) return set_error(PACK_EINVAL, "perm is not a permutation of 0 .. T-1");
        seen[(size_t)perm[i]] = 1;
    }
    for (int i = 0; i < T; ++i) group_out[perm[i]] = i / m;
    *n_groups = (T + m - 1) / m;
    return PACK_OK;
}

pack_status pack_opt_batchsize(const int32_t* batch, int32_t T, const uint64_t* need, uint64_t capacity,
                               int32_t* group_out, int32_t* n_groups) {
    if (!batch || !need || !group_out || !n_groups) return set_error(PACK_EINVAL, "null argument");
    if (T < 1) return set_error(PACK_EINVAL, "need T >= 1");
    std::vector<int32_t> sizes(batch, batch + T);
    std::sort(sizes.begin(), sizes.end());
    sizes.erase(std::unique(sizes.begin(), sizes.end()), sizes.end());
    int groups = 0;
    for (int32_t b : sizes) {
        uint64_t used = 0;
        bool open = false;
        for (int i = 0; i < T; ++i) {
            if (batch[i] != b) continue;
            if (open && (need[i] > capacity || used > capacity - need[i])) {
                ++groups;
                open = false;
                used = 0;
            }
            group_out[i] = groups;
            used += need[i];
            open = true;
        }
        if (open) ++groups;
    }
    *n_groups = groups;
    return PACK_OK;
}

pack_status pack_hyperband_plan(int32_t R, int32_t eta, int32_t* n_out, int32_t* r_out, int32_t* rungs_out,
                                int32_t capacity, int32_t* n_brackets) {
    if (!n_out || !r_out || !rungs_out || !n_brackets) return set_error(PACK_EINVAL, "null argument");
    if (R < 1 || eta < 2) return set_error(PACK_EINVAL, "need R >= 1 and eta >= 2");
    int s_max = 0;
    long long pw = eta;
    while (pw <= R) { ++s_max; pw *= eta; }
    const long long B = (long long)(s_max + 1) * R;
    int written = 0;
    for (int s = s_max; s >= 0; --s) {
        long long eta_s = 1;
        for (int j = 0; j < s; ++j) eta_s *= eta;
        const long long n = (B * eta_s + (long long)R * (s + 1) - 1) / ((long long)R * (s + 1));
        if (written + s + 1 > capacity) return set_error(PACK_EINVAL, "output arrays too small for the plan");
        long long eta_i = 1;
        for (int i = 0; i <= s; ++i) {
            n_out[written] = (int32_t)(n / eta_i);
            r_out[written] = (int32_t)((long long)R * eta_i / eta_s);
            ++written;
            eta_i *= eta;
        }
        rungs_out[s_max - s] = s + 1;
    }
    *n_brackets = s_max + 1;
    return PACK_OK;
}

pack_status pack_halving_keep(const float* loss, int32_t n, int32_t keep, int32_t* idx_out) {
    if (!loss || !idx_out) return set_error(PACK_EINVAL, "null argument");
    if (n < 1 || keep < 0 || keep > n) return set_error(PACK_EINVAL, "need n >= 1 and keep in [0, n]");
    std::vector<int32_t> order((size_t)n);
    std::iota(order.begin(), order.end(), 0);
    // A diverged configuration reports NaN (or +inf).  NaN compares false with everything, which is no
    // ordering at all, so it is ranked explicitly: after every number, +inf included, ties by position.
    auto before = [&](int32_t a, int32_t b) {
        const bool na = std::isnan(loss[a]), nb = std::isnan(loss[b]);
        if (na || nb) return !na && nb;
        return loss[a] < loss[b];
    };
    std::stable_sort(order.begin(), order.end(), before);
    std::sort(order.begin(), order.begin() + keep);
    for (int i = 0; i < keep; ++i) idx_out[i] = order[(size_t)i];
    return PACK_OK;
}

}  // extern "C"
