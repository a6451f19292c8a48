"""TEST INFRASTRUCTURE ONLY - plain, slow reference for the planner pieces of the library.

Written from the paper's definitions, not from the library's code, and sharing nothing with it:

* sequence bucketing (paper Sec. 4.1.3 "Problem Solving"): the objective is the total deviation
  of every length from the upper limit of its bucket, bucket q holding the lengths in
  (limit[q-1], limit[q]].  `bucket_error` evaluates that objective for given limits;
  `bucket_brute_force` minimises it by trying EVERY choice of at most Q limits among the
  distinct lengths (an optimal limit is always one of the lengths: lowering a limit to the
  largest length below it never increases any deviation); `bucket_dp_table` is the recurrence
  the paper states, filled entry by entry.
* micro-batch chunking (paper Appendix A): consecutive, non-empty micro-batches in the given
  order, minimising the largest micro-batch token count.  `chunk_brute_force` tries every
  placement of the M-1 cut points; `chunk_dp_table` is the stated recurrence.
* `naive_bucket_limits`: the fixed-interval bucketing the paper compares against (upper limits
  at multiples of a fixed interval).

Only tests may import this module.
"""
from __future__ import annotations

from itertools import combinations
from typing import List, Sequence, Tuple


def bucket_error(lens: Sequence[int], limits: Sequence[int]) -> int:
    """Sum over sequences of (upper limit of the sequence's bucket - length); limits ascending."""
    total = 0
    for s in lens:
        lim = next(l for l in limits if s <= l)   # first limit that is not below the length
        total += lim - s
    return total


def bucket_brute_force(lens: Sequence[int], Q: int) -> int:
    """Minimal bucket_error over every set of at most Q limits (the largest length is always one)."""
    distinct = sorted(set(lens))
    if not distinct:
        return 0
    top, rest = distinct[-1], distinct[:-1]
    best = None
    for n in range(0, min(Q - 1, len(rest)) + 1):
        for chosen in combinations(rest, n):
            e = bucket_error(lens, list(chosen) + [top])
            best = e if best is None or e < best else best
    return best


def bucket_dp_table(lens: Sequence[int], Q: int) -> int:
    """err[K][min(Q, K)] of the paper's recurrence err[k][q] = min_j err[j][q-1] + sum_{i=j+1..k}(s_k - s_i)."""
    s = sorted(lens)
    K = len(s)
    if K == 0:
        return 0
    INF = float("inf")
    nb = min(Q, K)
    err = [[INF] * (nb + 1) for _ in range(K + 1)]
    err[0][0] = 0
    for q in range(1, nb + 1):
        for k in range(1, K + 1):
            for j in range(0, k):
                if err[j][q - 1] == INF:
                    continue
                c = sum(s[k - 1] - s[i] for i in range(j, k))
                err[k][q] = min(err[k][q], err[j][q - 1] + c)
    return min(err[K][q] for q in range(1, nb + 1))


def naive_bucket_limits(lens: Sequence[int], interval: int) -> List[int]:
    """Fixed-interval bucketing: upper limits interval, 2*interval, ... up to the one covering the longest."""
    top = max(lens)
    n = -(-top // interval)
    return [interval * (i + 1) for i in range(n)]


def chunk_max(lens: Sequence[int], ends: Sequence[int]) -> int:
    start, worst = 0, 0
    for e in ends:
        worst = max(worst, sum(lens[start:e]))
        start = e
    return worst


def chunk_brute_force(lens: Sequence[int], M: int) -> int:
    """Minimal largest micro-batch token count over every split into M consecutive non-empty parts."""
    K = len(lens)
    best = None
    for cuts in combinations(range(1, K), M - 1):
        v = chunk_max(lens, list(cuts) + [K])
        best = v if best is None or v < best else best
    return best


def chunk_dp_table(lens: Sequence[int], M: int) -> int:
    """DP[K][M] of the paper's recurrence DP[k][i] = min_{j in [i-1, k-1]} max(DP[j][i-1], sum_{l=j+1..k} s_l)."""
    K = len(lens)
    INF = float("inf")
    dp = [[INF] * (M + 1) for _ in range(K + 1)]
    dp[0][0] = 0
    for i in range(1, M + 1):
        for k in range(i, K + 1):
            for j in range(i - 1, k):
                if dp[j][i - 1] == INF:
                    continue
                dp[k][i] = min(dp[k][i], max(dp[j][i - 1], sum(lens[j:k])))
    return dp[K][M]
