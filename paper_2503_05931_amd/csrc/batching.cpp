// Host-side 2D bucketing batch former (see include/aed_batching.h).  Plain C++, no GPU work.
#include "../../include/aed_batching.h"

#include <algorithm>
#include <numeric>
#include <vector>

struct aed_bucketing {
    int n_in = 0, n_out = 0;
    std::vector<int32_t> in_upper;   // [n_in], non-decreasing
    std::vector<int32_t> out_upper;  // [n_in * n_out], non-decreasing inside a bin
};

namespace {
uint64_t splitmix64(uint64_t x) {
    x += 0x9E3779B97F4A7C15ull;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}
}  // namespace

extern "C" {

int aed_bucketing_estimate(const int32_t* in_len, const int32_t* out_len, int64_t n, int32_t n_in_bins,
                           int32_t n_out_bins, aed_bucketing** out) {
    if (!in_len || !out_len || !out || n < 1 || n_in_bins < 1 || n_out_bins < 1) return AED_BATCHING_EINVAL;
    for (int64_t i = 0; i < n; ++i)
        if (in_len[i] < 1 || out_len[i] < 1) return AED_BATCHING_EINVAL;
    std::vector<int64_t> order(n);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int64_t a, int64_t b) { return in_len[a] < in_len[b]; });
    int64_t total = 0;  // exact integer arithmetic: edges do not depend on rounding
    for (int64_t i = 0; i < n; ++i) total += in_len[i];

    aed_bucketing* b = new aed_bucketing();
    b->n_in = n_in_bins;
    b->n_out = n_out_bins;
    b->in_upper.assign(n_in_bins, 0);
    b->out_upper.assign((size_t)n_in_bins * n_out_bins, 0);
    int64_t pos = 0;
    int64_t cum = 0;
    int32_t prev_in = 0;
    std::vector<int32_t> prev_out(n_out_bins, 0);
    for (int k = 0; k < n_in_bins; ++k) {
        const int64_t first = pos;
        if (k == n_in_bins - 1) {
            while (pos < n) cum += in_len[order[pos++]];
        } else {
            // a sample joins bin k while the cumulative length stays within (k + 1) / n_in_bins of the total
            while (pos < n && (cum + in_len[order[pos]]) * n_in_bins <= total * (k + 1)) cum += in_len[order[pos++]];
            // equal lengths stay together: pull in the rest of a run that the edge would split
            while (pos < n && pos > first && in_len[order[pos]] == in_len[order[pos - 1]]) cum += in_len[order[pos++]];
        }
        if (pos == first) {  // empty bin: repeat the previous bounds
            b->in_upper[k] = prev_in;
            for (int j = 0; j < n_out_bins; ++j) b->out_upper[(size_t)k * n_out_bins + j] = prev_out[j];
            continue;
        }
        b->in_upper[k] = prev_in = in_len[order[pos - 1]];
        std::vector<int32_t> outs;
        outs.reserve(pos - first);
        for (int64_t i = first; i < pos; ++i) outs.push_back(out_len[order[i]]);
        std::sort(outs.begin(), outs.end());
        const int64_t m = (int64_t)outs.size();
        int32_t last = 0;
        for (int j = 0; j < n_out_bins; ++j) {
            const int64_t hi = m * (j + 1) / n_out_bins;  // sub-bin j holds sorted positions [m j / n, hi)
            if (hi > m * j / n_out_bins) last = outs[hi - 1];
            b->out_upper[(size_t)k * n_out_bins + j] = prev_out[j] = last;
        }
    }
    *out = b;
    return AED_BATCHING_OK;
}

void aed_bucketing_free(aed_bucketing* b) { delete b; }

int aed_bucketing_bounds(const aed_bucketing* b, int32_t* in_upper, int32_t* out_upper) {
    if (!b || !in_upper || !out_upper) return AED_BATCHING_EINVAL;
    std::copy(b->in_upper.begin(), b->in_upper.end(), in_upper);
    std::copy(b->out_upper.begin(), b->out_upper.end(), out_upper);
    return AED_BATCHING_OK;
}

int32_t aed_bucketing_allocate(const aed_bucketing* b, int32_t in_len, int32_t out_len, int32_t mode) {
    if (!b || in_len < 1 || out_len < 1) return -1;
    for (int k = 0; k < b->n_in; ++k) {
        if (b->in_upper[k] < in_len) continue;
        for (int j = 0; j < b->n_out; ++j)
            if (b->out_upper[(size_t)k * b->n_out + j] >= out_len) return k * b->n_out + j;
        if (mode == AED_ALLOC_STRICT) return -1;  // the output is longer than this bin's last sub-bin
    }
    return -1;
}

int32_t aed_tps_keep(int32_t in_len, int32_t out_len, double frames_per_second, double max_tps) {
    if (in_len < 1 || out_len < 0 || !(frames_per_second > 0)) return 0;
    return (double)out_len * frames_per_second <= max_tps * (double)in_len ? 1 : 0;
}

int aed_bucketing_batch_sizes(const aed_bucketing* b, int64_t budget_frames, int32_t max_batch, int32_t* batch_sizes) {
    if (!b || !batch_sizes || budget_frames < 1 || max_batch < 1) return AED_BATCHING_EINVAL;
    for (int k = 0; k < b->n_in; ++k) {
        int64_t bs = b->in_upper[k] > 0 ? budget_frames / b->in_upper[k] : max_batch;
        bs = std::max<int64_t>(1, std::min<int64_t>(bs, max_batch));
        for (int j = 0; j < b->n_out; ++j) batch_sizes[(size_t)k * b->n_out + j] = (int32_t)bs;
    }
    return AED_BATCHING_OK;
}

int aed_bucketing_form_batches(const aed_bucketing* b, const int32_t* in_len, const int32_t* out_len, int64_t n,
                               int32_t mode, const int32_t* batch_sizes, int32_t* batch_of, int32_t* bucket_of_batch,
                               int32_t* n_batches) {
    if (!b || !in_len || !out_len || !batch_sizes || !batch_of || !bucket_of_batch || !n_batches || n < 1)
        return AED_BATCHING_EINVAL;
    if (mode != AED_ALLOC_STRICT && mode != AED_ALLOC_FLEXIBLE) return AED_BATCHING_EINVAL;
    const int nb = b->n_in * b->n_out;
    for (int k = 0; k < nb; ++k)
        if (batch_sizes[k] < 1) return AED_BATCHING_EINVAL;
    std::vector<int32_t> bucket(n);
    std::vector<int64_t> count(nb, 0);
    for (int64_t i = 0; i < n; ++i) {
        bucket[i] = aed_bucketing_allocate(b, in_len[i], out_len[i], mode);
        if (bucket[i] >= 0) ++count[bucket[i]];
    }
    std::vector<int64_t> first_batch(nb, 0);
    int64_t total = 0;
    for (int k = 0; k < nb; ++k) {
        first_batch[k] = total;
        const int64_t nbk = (count[k] + batch_sizes[k] - 1) / batch_sizes[k];
        for (int64_t t = 0; t < nbk; ++t) bucket_of_batch[total + t] = k;
        total += nbk;
    }
    std::vector<int64_t> seen(nb, 0);
    for (int64_t i = 0; i < n; ++i) {
        const int k = bucket[i];
        batch_of[i] = k < 0 ? -1 : (int32_t)(first_batch[k] + seen[k]++ / batch_sizes[k]);
    }
    *n_batches = (int32_t)total;
    return AED_BATCHING_OK;
}

int32_t aed_bucket_select(uint64_t seed, uint64_t step, const int32_t* available, int32_t n_buckets) {
    if (!available || n_buckets < 1) return -1;
    const int32_t want = (int32_t)(splitmix64(seed + step * 0x9E3779B97F4A7C15ull) % (uint64_t)n_buckets);
    for (int32_t dist = 0; dist < n_buckets; ++dist) {
        if (want - dist >= 0 && available[want - dist] > 0) return want - dist;
        if (want + dist < n_buckets && available[want + dist] > 0) return want + dist;
    }
    return -1;
}

}  // extern "C"
