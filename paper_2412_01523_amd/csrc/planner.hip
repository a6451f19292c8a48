// Host-side pieces of FlexSP's planner that are exact and need no external solver:
//   * adaptive sequence bucketing (paper Sec. 4.1.3, "Problem Solving": the bucketing objective
//     and its dynamic programme),
//   * memory-balanced micro-batch chunking (paper Appendix A, the min-max objective and its
//     dynamic programme),
//   * the smallest feasible number of micro-batches (Sec. 4.2, takeaway #1).
// Plain C++; nothing here touches the GPU.  Both programmes are solved exactly but faster than the
// textbook recurrences: the bucket cost is a Monge array (so the best split point moves
// monotonically with the prefix length and a row of the table is filled by divide and conquer,
// O(K log K) per bucket instead of O(K^2)); the chunking optimum is found by bisection on the
// answer with a greedy feasibility test, which on integers gives the same value as the recurrence.
#include <algorithm>
#include <cstdint>
#include <limits>
#include <new>
#include <numeric>
#include <vector>

#include "flexsp.h"

namespace {

constexpr int64_t kInf = std::numeric_limits<int64_t>::max() / 4;

struct BucketDp {
    const std::vector<int64_t> &s;    // sorted lengths, 1-based via pre[]
    std::vector<int64_t> pre;         // pre[k] = s_1 + ... + s_k
    std::vector<int64_t> prev, cur;   // err[.][q-1], err[.][q]
    std::vector<int32_t> arg;         // arg[q * (K+1) + k]: best j for err[k][q]
    int64_t K;

    explicit BucketDp(const std::vector<int64_t> &sorted) : s(sorted), K((int64_t)sorted.size())
    {
        pre.assign(K + 1, 0);
        for (int64_t k = 1; k <= K; k++) pre[k] = pre[k - 1] + s[k - 1];
    }
    // deviation of sequences j+1..k from the upper limit s_k of their bucket
    int64_t cost(int64_t j, int64_t k) const { return (k - j) * s[k - 1] - (pre[k] - pre[j]); }
    // fills cur[klo..khi] knowing that the best j lies in [jlo, jhi]
    void solve(int q, int64_t klo, int64_t khi, int64_t jlo, int64_t jhi)
    {
        if (klo > khi) return;
        const int64_t k = (klo + khi) / 2;
        int64_t best = kInf, bj = jlo;
        const int64_t top = std::min(jhi, k - 1);
        for (int64_t j = jlo; j <= top; j++) {
            if (prev[j] >= kInf) continue;
            const int64_t v = prev[j] + cost(j, k);
            if (v < best) {
                best = v;
                bj = j;
            }
        }
        cur[k] = best;
        arg[(size_t)q * (K + 1) + k] = (int32_t)bj;
        solve(q, klo, k - 1, jlo, bj);
        solve(q, k + 1, khi, bj, jhi);
    }
};

}  // namespace

extern "C" {

int flexsp_bucket_dp(const int64_t *lens, int64_t K, int32_t Q, int64_t *limits, int32_t *num_buckets,
                     int32_t *bucket_of, int64_t *error)
{
    if (K < 0 || Q <= 0 || (K > 0 && !lens) || !limits || !num_buckets || !error) return FLEXSP_INVALID_ARGUMENT;
    if (K > 0x7ffffff0) return FLEXSP_UNSUPPORTED;
    for (int64_t k = 0; k < K; k++)
        if (lens[k] < 0 || lens[k] > ((int64_t)1 << 40)) return FLEXSP_INVALID_ARGUMENT;
    *num_buckets = 0;
    *error = 0;
    if (K == 0) return FLEXSP_OK;
    try {
        std::vector<int64_t> order(K);
        std::iota(order.begin(), order.end(), (int64_t)0);
        std::stable_sort(order.begin(), order.end(), [&](int64_t a, int64_t b) { return lens[a] < lens[b]; });
        std::vector<int64_t> s(K);
        for (int64_t k = 0; k < K; k++) s[k] = lens[order[k]];
        const int nb = (int)std::min<int64_t>(Q, K);  // more buckets than sequences cannot help
        BucketDp dp(s);
        dp.arg.assign((size_t)(nb + 1) * (K + 1), 0);
        dp.prev.assign(K + 1, kInf);
        dp.cur.assign(K + 1, kInf);
        dp.prev[0] = 0;  // err[0][0] = 0
        for (int q = 1; q <= nb; q++) {
            std::fill(dp.cur.begin(), dp.cur.end(), kInf);
            // q non-empty buckets hold at least q sequences; the split j leaves q-1 for the others
            dp.solve(q, q, K, q - 1, K - 1);
            dp.prev.swap(dp.cur);
        }
        *error = dp.prev[K];
        // walk the split points back; equal lengths that ended up either side of a split share a limit
        std::vector<int64_t> ends;  // 1-based index of the last sequence of each bucket, descending
        int64_t k = K;
        for (int q = nb; q >= 1; q--) {
            ends.push_back(k);
            k = dp.arg[(size_t)q * (K + 1) + k];
        }
        std::reverse(ends.begin(), ends.end());
        int n = 0;
        for (int64_t e : ends) {
            const int64_t lim = s[e - 1];
            if (n == 0 || limits[n - 1] != lim) limits[n++] = lim;
        }
        *num_buckets = n;
        if (bucket_of)
            for (int64_t i = 0; i < K; i++)
                bucket_of[i] = (int32_t)(std::lower_bound(limits, limits + n, lens[i]) - limits);
    } catch (const std::bad_alloc &) {
        return FLEXSP_OUT_OF_MEMORY;
    }
    return FLEXSP_OK;
}

int flexsp_chunk_dp(const int64_t *lens, int64_t K, int32_t M, int64_t *ends, int64_t *max_tokens)
{
    if (K < 0 || M <= 0 || (K > 0 && !lens) || !ends || !max_tokens) return FLEXSP_INVALID_ARGUMENT;
    if (M > K) return FLEXSP_INVALID_ARGUMENT;  // every micro-batch holds at least one sequence
    int64_t total = 0, largest = 0;
    for (int64_t k = 0; k < K; k++) {
        if (lens[k] < 0 || lens[k] > ((int64_t)1 << 40)) return FLEXSP_INVALID_ARGUMENT;
        total += lens[k];
        largest = std::max(largest, lens[k]);
    }
    // chunks needed when no chunk may exceed `cap` (cap >= largest), filling greedily from the left
    auto chunks_needed = [&](int64_t cap) {
        int64_t n = 1, acc = 0;
        for (int64_t k = 0; k < K; k++) {
            if (acc + lens[k] > cap) {
                n++;
                acc = 0;
            }
            acc += lens[k];
        }
        return n;
    };
    int64_t lo = largest, hi = total;  // the optimum lies in [lo, hi]; feasibility is monotone in cap
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (chunks_needed(mid) <= M)
            hi = mid;
        else
            lo = mid + 1;
    }
    *max_tokens = lo;
    // one optimal split: fill greedily up to the optimum, but leave a sequence for every later chunk
    int64_t k = 0;
    for (int32_t i = 0; i < M; i++) {
        int64_t acc = 0;
        const int64_t must_leave = M - 1 - i;
        if (i == M - 1) {
            k = K;
        } else {
            int64_t taken = 0;
            while (k < K - must_leave && (taken == 0 || acc + lens[k] <= lo)) {
                acc += lens[k];
                k++;
                taken++;
            }
        }
        ends[i] = k;
    }
    return FLEXSP_OK;
}

int64_t flexsp_min_microbatches(int64_t batch_tokens, int64_t cluster_token_capacity)
{
    if (batch_tokens < 0 || cluster_token_capacity <= 0) return FLEXSP_INVALID_ARGUMENT;
    return (batch_tokens + cluster_token_capacity - 1) / cluster_token_capacity;
}

}  // extern "C"
