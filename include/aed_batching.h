/*
 * aed_batching.h -- host-side 2D bucketing batch former (C ABI, no GPU work).
 *
 * The paper's sampling method, used here to shape inference batches whose
 * sequences have similar input AND output lengths: duration bins estimated for
 * equal occupancy w.r.t. cumulative duration, each split into output-length
 * sub-bins (Sec. "Experimental setup": 30 bins x 2 sub-bins); "strict" and
 * "flexible" sample-to-bucket allocation (Sec. "Methods", paragraph on the
 * token-per-second distribution); the tokens-per-second filter (same paragraph;
 * threshold 25 in Sec. "Experimental setup"); the batch size of a bucket from a
 * cumulative-duration budget (Sec. "Methods": examples are drawn until the
 * cumulative duration exceeds a threshold); and synchronized bucket selection
 * with a shared seed and fall-back to the closest non-empty bucket (Sec.
 * "Methods", "Distributed training and synchronized bucketing").
 *
 * Lengths are integers: input length in encoder frames, output length in
 * tokens.  All pointers are HOST pointers owned by the caller.  Functions
 * return 0 on success and a negative aed_batching_status on a bad argument;
 * nothing is modified on error.
 */
#ifndef AED_BATCHING_H
#define AED_BATCHING_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct aed_bucketing aed_bucketing; /* opaque: the estimated bins */

enum { AED_BATCHING_OK = 0, AED_BATCHING_EINVAL = -1 };
enum { AED_ALLOC_STRICT = 0, AED_ALLOC_FLEXIBLE = 1 };

/* Estimate bins from n samples (in_len[i] >= 1, out_len[i] >= 1).
 * Input bins: samples sorted by input length; bin edges are placed where the
 * cumulative input length crosses k/n_in_bins of the total (equal occupancy
 * w.r.t. cumulative duration); a bin's upper bound is the largest input length
 * in it; samples of equal length never straddle an edge.  Sub-bins: the samples
 * of a bin sorted by output length and cut into n_out_bins equal-count parts;
 * a sub-bin's upper bound is the largest output length in it.  Empty bins or
 * sub-bins (too few distinct samples) repeat the previous upper bound. */
int aed_bucketing_estimate(const int32_t *in_len, const int32_t *out_len, int64_t n,
                           int32_t n_in_bins, int32_t n_out_bins, aed_bucketing **out);
void aed_bucketing_free(aed_bucketing *b);

/* Copy the bounds: in_upper[n_in_bins], out_upper[n_in_bins * n_out_bins] (bin-major). */
int aed_bucketing_bounds(const aed_bucketing *b, int32_t *in_upper, int32_t *out_upper);

/* Bucket (in_bin * n_out_bins + out_bin) of one sample, or -1 if it is discarded.
 * strict: the first input bin whose upper bound >= in_len, then the first of ITS sub-bins whose upper
 *   bound >= out_len; discarded if no input bin fits or the output is longer than that bin's last sub-bin.
 * flexible: the first bucket in bin-major order that fits the sample in both dimensions (it may lie in
 *   a bin of longer inputs); discarded only if no bucket fits. */
int32_t aed_bucketing_allocate(const aed_bucketing *b, int32_t in_len, int32_t out_len, int32_t mode);

/* Tokens-per-second filter: 1 = keep (out_len / (in_len / frames_per_second) <= max_tps), 0 = drop. */
int32_t aed_tps_keep(int32_t in_len, int32_t out_len, double frames_per_second, double max_tps);

/* Batch size of every bucket from a budget of input frames per batch:
 * max(1, floor(budget_frames / in_upper[bin])), capped at max_batch.  batch_sizes[n_buckets]. */
int aed_bucketing_batch_sizes(const aed_bucketing *b, int64_t budget_frames, int32_t max_batch, int32_t *batch_sizes);

/* Form mini-batches from a pool: every kept sample goes to its bucket (allocation mode as above), and each
 * bucket's samples, in pool order, are cut into consecutive batches of that bucket's size (the last one may be
 * smaller).  batch_of[i] receives the batch id of sample i (batches numbered bucket by bucket, in order) or -1
 * if the sample was discarded; bucket_of_batch (capacity n) receives each batch's bucket; *n_batches the count. */
int aed_bucketing_form_batches(const aed_bucketing *b, const int32_t *in_len, const int32_t *out_len, int64_t n,
                               int32_t mode, const int32_t *batch_sizes, int32_t *batch_of,
                               int32_t *bucket_of_batch, int32_t *n_batches);

/* Synchronized bucket selection: every rank calls this with the same (seed, step) and its own availability
 * (available[k] = mini-batches ready in bucket k) and gets the shared pseudo-random choice if that bucket is
 * non-empty here, else the closest non-empty bucket by index distance (the lower index on a tie), else -1.
 * The shared choice is splitmix64(seed + step * 0x9E3779B97F4A7C15) mod n_buckets. */
int32_t aed_bucket_select(uint64_t seed, uint64_t step, const int32_t *available, int32_t n_buckets);

#ifdef __cplusplus
}
#endif
#endif
