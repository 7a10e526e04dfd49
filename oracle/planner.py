"""CPU oracle for the merge planner.  TEST INFRASTRUCTURE ONLY.

Plain, slow, obviously-correct Python written from the paper; it shares no code
with the HIP/C++ library and must never be imported by the product path (only
tests, the smoke check and the benchmark's cpu_baseline leg may use it).

Conventions: layers are numbered 1..L as in the paper; Python lists are indexed
by `l - 1`.  Backward runs L -> 1.  Times are milliseconds, message sizes bytes,
gradients are fp32 so a layer of p parameters is a 4p-byte message (Section V-A).

What each function follows:
  t_ar            Eq. 9   all-reduce cost a + b*M
  backward_start  Eq. 6   tau_b
  wfbp_timeline   Eq. 7-8 tau_c and t_iter with every layer sent alone
  simulate        Eq. 7-8 generalised to merged groups by Conditions 1-3 (Eq. 14-16)
  brute_force     Eq. 19-23, the problem statement itself: minimum over every set M
  algorithm1      Algorithm 1 (with its Merge and CalculateCommStart procedures),
                  i.e. the rule of Theorem 1
Readings taken where the text is ambiguous are listed next to the code.
"""
from __future__ import annotations

from itertools import combinations
from typing import Iterable, List, Sequence, Tuple

BYTES_PER_PARAM = 4  # fp32 parameters and gradients (Section V)


def t_ar(a: float, b: float, n_bytes: int) -> float:
    """Eq. 9: T_ar(M) = a + b*M, M in bytes."""
    return a + b * n_bytes


def backward_start(tb: Sequence[float], tf: float) -> List[float]:
    """Eq. 6: tau_b[L] = t_f, tau_b[l] = tau_b[l+1] + t_b[l+1].  Returned as list index l-1."""
    L = len(tb)
    tau_b = [0.0] * L
    tau_b[L - 1] = tf
    for l in range(L - 1, 0, -1):          # l = L-1 .. 1
        tau_b[l - 1] = tau_b[l] + tb[l]
    return tau_b


def backward_finish(tb: Sequence[float], tf: float) -> List[float]:
    """mu_b[l] = tau_b[l] + t_b[l], the moment layer l's gradients exist (notation table)."""
    tau_b = backward_start(tb, tf)
    return [tau_b[i] + tb[i] for i in range(len(tb))]


def wfbp_timeline(p: Sequence[int], tb: Sequence[float], tf: float, a: float, b: float
                  ) -> Tuple[List[float], float]:
    """Eq. 7 and Eq. 8 written out directly for plain WFBP (no merging).

    Returns (tau_c, t_iter) with t_iter = t_c(1) + tau_c(1), which is Eq. 8's last line.
    """
    L = len(p)
    tau_b = backward_start(tb, tf)
    tc = [t_ar(a, b, BYTES_PER_PARAM * int(p[i])) for i in range(L)]
    tau_c = [0.0] * L
    tau_c[L - 1] = tau_b[L - 1] + tb[L - 1]
    for l in range(L - 1, 0, -1):
        tau_c[l - 1] = max(tau_c[l] + tc[l], tau_b[l - 1] + tb[l - 1])
    return tau_c, tc[0] + tau_c[0]


def simulate(p: Sequence[int], tb: Sequence[float], tf: float, a: float, b: float,
             merged: Iterable[int]) -> float:
    """Iteration time when the layers in `merged` (a subset of {2..L}) ride with layer l-1.

    Walk the backward pass L -> 1.  A merged layer sends nothing itself
    (Condition 1) and hands its parameters to layer l-1 (Condition 3).  A layer
    that is not merged sends everything accumulated so far as one message, starting
    when both the channel is free and its own gradients exist (Eq. 7; for a layer
    whose predecessor merged this is Condition 2), at cost Eq. 9.  The iteration
    ends when layer 1's message is done (Eq. 8).
    """
    L = len(p)
    mset = set(merged)
    assert all(2 <= l <= L for l in mset), "M is a subset of {2..L} (Eq. 22)"
    mu_b = backward_finish(tb, tf)
    channel_free = 0.0
    pending = 0
    for l in range(L, 0, -1):
        pending += BYTES_PER_PARAM * int(p[l - 1])
        if l in mset:
            continue
        start = max(channel_free, mu_b[l - 1])
        channel_free = start + t_ar(a, b, pending)
        pending = 0
    return channel_free


def all_merge_sets(L: int):
    """Every subset of {2..L}: the 2^(L-1) contiguous partitions of the layers."""
    cand = list(range(2, L + 1))
    for k in range(len(cand) + 1):
        for c in combinations(cand, k):
            yield c


def brute_force(p: Sequence[int], tb: Sequence[float], tf: float, a: float, b: float
                ) -> Tuple[float, Tuple[int, ...]]:
    """The optimisation problem of Eq. 19-23 solved by enumeration (tiny L only).

    Returns (minimum t_iter, one merged set attaining it).  Several sets may tie;
    only the minimum value is unique.
    """
    best_t, best_m = None, None
    for m in all_merge_sets(len(p)):
        t = simulate(p, tb, tf, a, b, m)
        if best_t is None or t < best_t:
            best_t, best_m = t, m
    return best_t, best_m


def _calculate_comm_start(tc, tb, tau_b, L):
    """Algorithm 1, procedure CalculateCommStart (Eq. 7 with the current tc)."""
    tau_c = [0.0] * (L + 1)                       # 1-based
    tau_c[L] = tau_b[L] + tb[L]
    for l in range(L - 1, 0, -1):
        tau_c[l] = max(tau_c[l + 1] + tc[l + 1], tau_b[l] + tb[l])
    return tau_c


def algorithm1(p: Sequence[int], tb_in: Sequence[float], tf: float, a: float, b: float
               ) -> List[int]:
    """Algorithm 1: the merged-gradient layers chosen by Theorem 1's rule.

    Arrays are 1-based like the listing.  Readings:
      * the listing indexes tau_b[l-2], which for l = 2 is tau_b[0] and is never
        assigned; Section IV-A uses tau_b(1) = tau_b(2) + t_b(2) for l = 3, i.e.
        tau_b[l-2] is the instant layer l-1 finishes its backward.  We extend
        Eq. 6 one step below layer 1 so that tau_b[0] = tau_b[1] + t_b[1].
      * the listing fills tau_b down to index 2 only; Eq. 6 defines index 1 too.
      * T_ar takes bytes: the message of p parameters is 4p bytes.
      * strict '<' as printed: a tie does not merge.
    Returns M in the order pushed (descending l).
    """
    L = len(p)
    pp = [0] + [int(x) for x in p]                # pp[l], mutable copy (Merge changes it)
    tb = [0.0] + [float(x) for x in tb_in]
    tc = [0.0] * (L + 1)
    for l in range(1, L + 1):
        tc[l] = t_ar(a, b, BYTES_PER_PARAM * pp[l])
    tau_b = [0.0] * (L + 1)
    tau_b[L] = tf
    for l in range(L - 1, -1, -1):                # down to index 0 (see readings)
        tau_b[l] = tau_b[l + 1] + tb[l + 1]
    tau_c = _calculate_comm_start(tc, tb, tau_b, L)
    merged: List[int] = []
    for l in range(L, 1, -1):
        if tau_b[l - 2] - tau_c[l] < a:
            # procedure Merge
            tc[l] = 0.0
            pp[l - 1] = pp[l - 1] + pp[l]
            tc[l - 1] = t_ar(a, b, BYTES_PER_PARAM * pp[l - 1])
            tau_c = _calculate_comm_start(tc, tb, tau_b, L)
            merged.append(l)
    return merged


def groups_from_merged(L: int, merged: Iterable[int]) -> List[List[int]]:
    """Groups in communication order; inside a group layers are in arrival order (high -> low)."""
    mset = set(merged)
    groups, cur = [], []
    for l in range(L, 0, -1):
        cur.append(l)
        if l not in mset:
            groups.append(cur)
            cur = []
    return groups


# ---- Table II (costs of all-reduce algorithms) -------------------------------------------

def table2_cost(algorithm: str, n: int, alpha: float, beta: float, gamma: float
                ) -> Tuple[float, float]:
    """(a, b) of Table II for one of its four all-reduce algorithms."""
    from math import log2
    if algorithm == "binary_tree":
        return 2 * alpha * log2(n), (2 * beta + gamma) * log2(n)
    if algorithm == "recursive_doubling":
        return alpha * log2(n), (beta + gamma) * log2(n)
    if algorithm == "recursive_halving_doubling":
        return 2 * alpha * log2(n), 2 * beta - (2 * beta + gamma) / n + gamma
    if algorithm == "ring":
        return 2 * (n - 1) * alpha, 2 * (n - 1) / n * beta + (n - 1) / n * gamma
    raise ValueError(algorithm)


# ---- fitting Eq. 9 to measurements (Section V-A) ---------------------------------------------

def fit_cost(nbytes: Sequence[float], ms: Sequence[float]) -> Tuple[float, float]:
    """Ordinary least squares of ms = a + b*bytes via the normal equations.

    A negative intercept is clamped to 0 and the slope refitted through the origin.
    """
    n = len(nbytes)
    sx, sy = sum(nbytes), sum(ms)
    sxx = sum(x * x for x in nbytes)
    sxy = sum(x * y for x, y in zip(nbytes, ms))
    det = n * sxx - sx * sx
    b = (n * sxy - sx * sy) / det
    a = (sy - b * sx) / n
    if a < 0:
        a, b = 0.0, sxy / sxx
    return a, max(b, 0.0)


# ---- weak-scaling speedup (Eq. 4-5) and the trace-based simulation of Section V-C ------------

def speedup(n: int, tf: float, tb_total: float, t_iter: float) -> float:
    """Eq. 4: throughput of N workers over one worker = N (t_f + t_b) / t_iter."""
    return n * (tf + tb_total) / t_iter
