"""Trajectory placement: presorted dynamic programming (paper Sec. 5.2, Eq. 2 and Eq. 3), the
interference factor from a per-batch-size profile, and the group simulator.
TEST INFRASTRUCTURE ONLY (see package docstring).

Objective (Eq. 2): split n trajectories over m workers so that
    max_i  F(g_i) * max_{tau in g_i} L(tau) * T
is smallest; F depends on the size of a group only and does not decrease with it (premises of
Sec. 5.2).  With the trajectories in descending length order an optimal split into contiguous
runs exists (Lemma 1), and Eq. 3 finds it:

    dp[i][1] = L_1 * T * F(i)
    dp[i][j] = min_{k}  max( dp[k][j-1],  L_{k+1} * T * F(i - k) )

Everything here is written from those formulas in float64; products are evaluated left to
right as (L * T) * F so that the C++ planner can reproduce the values bit for bit.

Readings (the paper leaves them open):
  * more workers than trajectories: the surplus workers stay empty (their groups have size 0);
    with j <= i every one of the j groups is non-empty, k runs over j-1 .. i-1;
  * ties: the smallest k that reaches the minimum is taken (so the later group is as large as
    it can be); sizes are reported in worker order 1..m, the group with the longest trajectories
    first;
  * aggregation of short trajectories (the paper only says that trajectories under a threshold
    are merged after the sort, to shrink n): consecutive sorted trajectories shorter than the
    threshold are bundled, `bundle` at a time, into one element that carries its member count and the length of
    its first (longest) member; the DP then runs over elements, a group's size being the sum of
    its elements' counts.
"""
from __future__ import annotations

import itertools

import numpy as np


def group_cost(L_first: float, T: float, F, size: int) -> float:
    return (float(L_first) * float(T)) * float(F[size])


def placement_dp(lengths_desc, m: int, F, T: float = 1.0, counts=None):
    """lengths_desc: element lengths, descending.  F: table, F[s] for group size s = 0..total.
    counts: members per element (default 1 each).  Returns (makespan, sizes[m]) with sizes in
    elements per worker (sum = n)."""
    L = [float(x) for x in lengths_desc]
    n = len(L)
    if n == 0:
        return 0.0, [0] * m
    if any(L[i] < L[i + 1] for i in range(n - 1)):
        raise ValueError("lengths must be in descending order")
    cnt = [1] * n if counts is None else [int(c) for c in counts]
    cum = [0]
    for c in cnt:
        cum.append(cum[-1] + c)                      # members among the first i elements
    J = min(m, n)
    INF = float("inf")
    dp = [[INF] * (J + 1) for _ in range(n + 1)]
    arg = [[-1] * (J + 1) for _ in range(n + 1)]
    dp[0][0] = 0.0
    for i in range(1, n + 1):
        dp[i][1] = group_cost(L[0], T, F, cum[i])
        arg[i][1] = 0
    for j in range(2, J + 1):
        for i in range(j, n + 1):
            best, best_k = INF, -1
            for k in range(j - 1, i):                # first k elements on j-1 workers, k+1..i on worker j
                v = max(dp[k][j - 1], group_cost(L[k], T, F, cum[i] - cum[k]))
                if v < best:
                    best, best_k = v, k
            dp[i][j], arg[i][j] = best, best_k
    sizes = []
    i = n
    for j in range(J, 0, -1):
        k = arg[i][j]
        sizes.append(i - k)
        i = k
    sizes.reverse()
    return dp[n][J], sizes + [0] * (m - J)


def makespan_of_sizes(lengths_desc, sizes, F, T: float = 1.0, counts=None) -> float:
    """Objective value of a contiguous split given as elements per worker."""
    cnt = [1] * len(lengths_desc) if counts is None else list(counts)
    worst, i = 0.0, 0
    for s in sizes:
        if s:
            worst = max(worst, group_cost(lengths_desc[i], T, F, sum(cnt[i:i + s])))
        i += s
    return worst


def brute_force_contiguous(lengths_desc, m: int, F, T: float = 1.0, counts=None) -> float:
    """Smallest objective over every split of the sorted list into at most m contiguous runs."""
    n = len(lengths_desc)
    best = float("inf")
    for parts in range(1, min(m, n) + 1):
        for cuts in itertools.combinations(range(1, n), parts - 1):
            edges = (0,) + cuts + (n,)
            sizes = [edges[i + 1] - edges[i] for i in range(parts)]
            best = min(best, makespan_of_sizes(lengths_desc, sizes, F, T, counts))
    return best


def brute_force_any_partition(lengths, m: int, F, T: float = 1.0) -> float:
    """Smallest objective over every assignment of trajectories to m workers (m^n of them):
    what Lemma 1 says the contiguous optimum equals when F is monotone in the group size."""
    n = len(lengths)
    best = float("inf")
    for assign in itertools.product(range(m), repeat=n):
        worst = 0.0
        for w in range(m):
            members = [lengths[i] for i in range(n) if assign[i] == w]
            if members:
                worst = max(worst, group_cost(max(members), T, F, len(members)))
        best = min(best, worst)
    return best


def aggregate_short(lengths_desc, threshold: float, bundle: int):
    """Elements after bundling the short tail: (first_index[], count[]).  Trajectories with
    length >= threshold stay single; the rest are taken `bundle` at a time in sorted order."""
    n = len(lengths_desc)
    first, count = [], []
    i = 0
    while i < n:
        if lengths_desc[i] >= threshold or bundle <= 1:
            first.append(i)
            count.append(1)
            i += 1
        else:
            c = min(bundle, n - i)
            first.append(i)
            count.append(c)
            i += c
    return first, count


def profile_time(batch_sizes, step_time):
    """t(s): the profiled step time interpolated linearly between its points, held flat below
    the first point and continued with the last segment's slope above the last."""
    bs = [float(b) for b in batch_sizes]
    ts = [float(t) for t in step_time]
    if len(bs) < 1 or len(bs) != len(ts) or any(bs[i] >= bs[i + 1] for i in range(len(bs) - 1)):
        raise ValueError("batch sizes must be strictly increasing, one time each")

    def t_of(s):
        if s <= bs[0] or len(bs) == 1:
            return ts[0]
        for i in range(len(bs) - 1):
            if s <= bs[i + 1]:
                return ts[i] + (ts[i + 1] - ts[i]) * ((s - bs[i]) / (bs[i + 1] - bs[i]))
        return ts[-1] + (ts[-1] - ts[-2]) * ((s - bs[-1]) / (bs[-1] - bs[-2]))

    return t_of


def interference_table(batch_sizes, step_time, n: int):
    """F[s] for s = 0..n from a profile of the time of one decode step at a few batch sizes
    (Sec. 5.2, "Interference Factor": per-token time across a spectrum of batch sizes).
    F[s] = t(s) / t(1), forced non-decreasing by a running maximum (the DP's premise); F[0] = 0."""
    t_of = profile_time(batch_sizes, step_time)
    t1 = t_of(1.0)
    F = [0.0]
    for s in range(1, n + 1):
        F.append(max(t_of(float(s)) / t1, F[-1]))
    return F


def simulate_group(lengths, batch_sizes, step_time) -> float:
    """Time to finish a group whose trajectories all decode concurrently, one token per step
    (the simulator of Sec. 5.2 in its simplest form, no queueing): while a of them are still
    running a step takes t(a), and a trajectory of length L leaves after L steps.  Returns the
    total time in the profile's unit."""
    L = sorted((int(x) for x in lengths), reverse=True)
    t_of = profile_time(batch_sizes, step_time)
    total, steps_done = 0.0, 0
    for active in range(len(L), 0, -1):      # the shortest trajectory still running ends this phase
        upto = L[active - 1]
        total += (upto - steps_done) * t_of(float(active))
        steps_done = upto
    return total
