"""Plain-Python oracle of the 2D bucketing batch former.  TEST INFRASTRUCTURE ONLY.

Written from the paper's description of the sampling method, independently of
the C++ component it checks (it shares no code with it):
  * duration bins of equal occupancy w.r.t. cumulative duration, each divided
    into output-length sub-bins (Sec. "Experimental setup");
  * strict allocation: the 1D bucket by input length first, then one of its
    sub-buckets by output length, a too-long transcript is discarded; flexible
    allocation: the smallest bucket that fits the sample in both dimensions
    (Sec. "Methods");
  * tokens-per-second filter (Sec. "Methods"; threshold 25 in Sec. "Experimental setup");
  * batch size from a cumulative-duration budget (Sec. "Methods");
  * synchronized bucket selection from a shared seed, falling back to the
    closest bucket that has a mini-batch (Sec. "Methods").
Readings where the paper is silent: sub-bins hold equal counts; equal input
lengths are never split over two bins; "closest" is by bucket index with the
lower index winning a tie; the shared random choice is SplitMix64 (Steele,
Lea, Flood 2014) of seed + step * golden-gamma, modulo the bucket count.
"""
from fractions import Fraction

MASK = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15


def splitmix64(x):
    x = (x + GOLDEN) & MASK
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & MASK
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & MASK
    return x ^ (x >> 31)


def estimate(in_len, out_len, n_in_bins, n_out_bins):
    """-> (in_upper [n_in], out_upper [n_in][n_out])"""
    n = len(in_len)
    order = sorted(range(n), key=lambda i: in_len[i])       # stable
    total = sum(in_len)
    in_upper, out_upper = [], []
    pos, cum = 0, 0
    prev_in, prev_out = 0, [0] * n_out_bins
    for k in range(n_in_bins):
        first = pos
        if k == n_in_bins - 1:
            pos = n
        else:
            share = Fraction(total * (k + 1), n_in_bins)
            while pos < n and cum + in_len[order[pos]] <= share:
                cum += in_len[order[pos]]
                pos += 1
            while pos < n and pos > first and in_len[order[pos]] == in_len[order[pos - 1]]:
                cum += in_len[order[pos]]
                pos += 1
        members = order[first:pos]
        if not members:
            in_upper.append(prev_in)
            out_upper.append(list(prev_out))
            continue
        prev_in = max(in_len[i] for i in members)
        in_upper.append(prev_in)
        outs = sorted(out_len[i] for i in members)
        m = len(outs)
        row, last = [], 0
        for j in range(n_out_bins):
            part = outs[m * j // n_out_bins: m * (j + 1) // n_out_bins]
            if part:
                last = part[-1]
            row.append(last)
        prev_out = row
        out_upper.append(row)
    return in_upper, out_upper


def allocate(in_upper, out_upper, in_len, out_len, flexible):
    n_out = len(out_upper[0])
    for k, ub in enumerate(in_upper):
        if ub < in_len:
            continue
        for j in range(n_out):
            if out_upper[k][j] >= out_len:
                return k * n_out + j
        if not flexible:
            return -1
    return -1


def tps_keep(in_len, out_len, frames_per_second, max_tps):
    return Fraction(out_len) / (Fraction(in_len) / Fraction(frames_per_second)) <= Fraction(max_tps)


def batch_sizes(in_upper, n_out, budget_frames, max_batch):
    out = []
    for ub in in_upper:
        bs = max(1, min(max_batch, budget_frames // ub)) if ub > 0 else max_batch
        out += [bs] * n_out
    return out


def form_batches(in_upper, out_upper, in_len, out_len, flexible, sizes):
    """-> (batch_of [n], bucket_of_batch [n_batches])"""
    n_out = len(out_upper[0])
    nb = len(in_upper) * n_out
    members = [[] for _ in range(nb)]
    for i in range(len(in_len)):
        k = allocate(in_upper, out_upper, in_len[i], out_len[i], flexible)
        if k >= 0:
            members[k].append(i)
    batch_of = [-1] * len(in_len)
    bucket_of_batch = []
    for k in range(nb):
        for s in range(0, len(members[k]), sizes[k]):
            for i in members[k][s:s + sizes[k]]:
                batch_of[i] = len(bucket_of_batch)
            bucket_of_batch.append(k)
    return batch_of, bucket_of_batch


def select(seed, step, available):
    n = len(available)
    want = splitmix64((seed + step * GOLDEN) & MASK) % n
    best = -1
    for k in range(n):
        if available[k] > 0 and (best < 0 or abs(k - want) < abs(best - want)):
            best = k
    return best
