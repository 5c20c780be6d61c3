// Epoch schedule of a pack whose members use different batch sizes (paper Section 3.2, second
// half; step counts of Section 3.3).  Host logic only: which samples form the shared batch of each
// step and how many of its leading rows each member trains on, so that every member sees every
// sample exactly once although the members advance through the dataset at different rates.
//
// The shared batch of a phase has the size of the largest batch among the members still training
// and is cut from the samples THAT member has not used; a member with a smaller batch takes the
// leading rows.  Usage is recorded per member as one bit per sample.  When the leading member has
// used everything it leaves, and the next phase is led by the largest batch that remains.
#include "../../include/pack.h"

#include <algorithm>
#include <new>
#include <string>
#include <vector>

namespace packk {
pack_status set_error(pack_status s, const std::string& msg);   // pack_api.cpp: text for pack_last_error
}
using packk::set_error;

struct pack_schedule {
    int64_t n = 0;
    int K = 0;
    std::vector<int32_t> batch;
    std::vector<std::vector<uint64_t>> used;   // [K][ceil(n / 64)], bit i set: member has trained on sample i
    std::vector<int64_t> n_used;               // [K]
    int lead = -1;                             // member leading the current phase, -1 before the first
    std::vector<int64_t> pool;                 // samples of the current phase, in dataset order
    size_t pool_pos = 0;
};

namespace {

bool finished(const pack_schedule* s, int k) { return s->n_used[k] == s->n; }

// opens the next phase; false when every member has finished
bool next_phase(pack_schedule* s) {
    s->lead = -1;
    for (int k = 0; k < s->K; ++k)
        if (!finished(s, k) && (s->lead < 0 || s->batch[k] > s->batch[s->lead])) s->lead = k;
    if (s->lead < 0) return false;
    const std::vector<uint64_t>& bits = s->used[s->lead];
    s->pool.clear();
    s->pool.reserve((size_t)(s->n - s->n_used[s->lead]));
    for (size_t w = 0; w < bits.size(); ++w) {
        uint64_t free_bits = ~bits[w];
        while (free_bits) {
            const int b = __builtin_ctzll(free_bits);
            free_bits &= free_bits - 1;
            const int64_t i = (int64_t)w * 64 + b;
            if (i < s->n) s->pool.push_back(i);
        }
    }
    s->pool_pos = 0;
    return true;
}

}  // namespace

extern "C" {

pack_status pack_schedule_create(int64_t n_samples, const int32_t* batch, int32_t K, pack_schedule_t** out) {
    if (out) *out = nullptr;
    if (!batch || !out) return set_error(PACK_EINVAL, "null argument");
    if (n_samples < 1 || K < 1 || K > PACK_MAX_MODELS) return set_error(PACK_EINVAL, "need n_samples >= 1 and K in [1, PACK_MAX_MODELS]");
    for (int k = 0; k < K; ++k)
        if (batch[k] < 1) return set_error(PACK_EINVAL, "batch sizes must be >= 1");
    pack_schedule* s = new (std::nothrow) pack_schedule();
    if (!s) return set_error(PACK_ENOMEM, "host allocation failed");
    try {
        s->n = n_samples;
        s->K = K;
        s->batch.assign(batch, batch + K);
        s->used.assign(K, std::vector<uint64_t>((size_t)((n_samples + 63) / 64), 0));
        s->n_used.assign(K, 0);
    } catch (const std::bad_alloc&) {
        delete s;
        return set_error(PACK_ENOMEM, "host allocation failed");
    }
    *out = s;
    return PACK_OK;
}

pack_status pack_schedule_next(pack_schedule_t* s, int64_t* idx_host, int32_t* rows, int32_t* rows_k, int32_t* lead) {
    if (!s || !idx_host || !rows || !rows_k) return set_error(PACK_EINVAL, "null argument");
    if (s->lead < 0 || s->pool_pos == s->pool.size()) {
        if (!next_phase(s)) {
            *rows = 0;
            for (int k = 0; k < s->K; ++k) rows_k[k] = 0;
            if (lead) *lead = -1;
            return PACK_OK;
        }
    }
    const size_t take = std::min<size_t>((size_t)s->batch[s->lead], s->pool.size() - s->pool_pos);
    const int64_t* shared = s->pool.data() + s->pool_pos;
    for (size_t r = 0; r < take; ++r) idx_host[r] = shared[r];
    for (int k = 0; k < s->K; ++k) {
        rows_k[k] = 0;
        if (finished(s, k)) continue;
        const size_t mine = std::min<size_t>((size_t)s->batch[k], take);
        for (size_t r = 0; r < mine; ++r) {
            uint64_t& w = s->used[k][(size_t)(shared[r] >> 6)];
            const uint64_t bit = 1ull << (shared[r] & 63);
            if (w & bit) return set_error(PACK_EINVAL, "internal: a member would see a sample twice");
            w |= bit;
        }
        s->n_used[k] += (int64_t)mine;
        rows_k[k] = (int32_t)mine;
    }
    s->pool_pos += take;
    *rows = (int32_t)take;
    if (lead) *lead = s->lead;
    return PACK_OK;
}

pack_status pack_schedule_used(const pack_schedule_t* s, int64_t* used_host) {
    if (!s || !used_host) return set_error(PACK_EINVAL, "null argument");
    for (int k = 0; k < s->K; ++k) used_host[k] = s->n_used[k];
    return PACK_OK;
}

void pack_schedule_destroy(pack_schedule_t* s) { delete s; }

}  // extern "C"
