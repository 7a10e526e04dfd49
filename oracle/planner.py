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
  comm_start      Eq. 7 for one layer under a given merged set
  algorithm1      the result of Algorithm 1, i.e. the rule of Theorem 1 applied top-down
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


def comm_start(p: Sequence[int], tb: Sequence[float], tf: float, a: float, b: float,
               merged: Iterable[int], layer: int) -> float:
    """tau_c(layer): when `layer` could begin to send, given that the layers in `merged`
    (all above `layer`) ride with the layer below them.

    Eq. 7 under Conditions 1-3: walk the backward pass from L down to `layer`; every layer
    above it that is not merged sends what has accumulated, as in `simulate`; `layer` itself
    can start once the channel is free and its own gradients exist.
    """
    L = len(p)
    mset = set(merged)
    mu_b = backward_finish(tb, tf)
    channel_free = 0.0
    pending = 0
    for l in range(L, layer, -1):
        pending += BYTES_PER_PARAM * int(p[l - 1])
        if l in mset:
            continue
        channel_free = max(channel_free, mu_b[l - 1]) + t_ar(a, b, pending)
        pending = 0
    return max(channel_free, mu_b[layer - 1])


def algorithm1(p: Sequence[int], tb: Sequence[float], tf: float, a: float, b: float
               ) -> List[int]:
    """The merged-gradient layers Algorithm 1 returns, i.e. the rule of Theorem 1 applied from
    the top layer down: layer l joins layer l-1 when the wait between the moment l could start
    to send and the moment l-1's gradients exist is shorter than the start-up cost a.

    Each decision sees the merges already made above it (Algorithm 1 recomputes the
    communication start times after every merge; here tau_c(l) is evaluated afresh by
    `comm_start` for the current set).  Readings:
      * the time compared with tau_c(l) is the instant layer l-1 finishes its backward pass
        (Section IV-A writes it tau_b(l-2) = tau_b(l-1) + t_b(l-1); for l = 2 that index does
        not exist in Eq. 6, the instant does: the end of the backward pass);
      * T_ar takes bytes: the message of p parameters is 4p bytes;
      * strict '<' as printed: a tie does not merge.
    Returns M in the order chosen (descending l).
    """
    L = len(p)
    mu_b = backward_finish(tb, tf)
    merged: List[int] = []
    for l in range(L, 1, -1):
        wait = mu_b[l - 2] - comm_start(p, tb, tf, a, b, merged, l)
        if wait < a:
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
