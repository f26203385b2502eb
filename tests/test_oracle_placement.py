"""Pins of the placement oracle (presorted DP of Eq. 3, interference table, group simulator)
against things other than itself: hand-worked tables, exhaustive search over every assignment
(which also checks Lemma 1), closed forms, a step-by-step simulation."""
import json
import os

import numpy as np
import pytest

from oracle import placement as pl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_worked_examples():
    for ex in json.load(open(os.path.join(GOLDEN, "placement_worked_examples.json")))["examples"]:
        mk, sizes = pl.placement_dp(ex["lengths"], ex["m"], ex["F"], ex["T"])
        assert mk == ex["makespan"] and sizes == ex["sizes"]


def monotone_F(rng, n):
    return np.concatenate([[0.0], 1.0 + np.cumsum(rng.uniform(0.0, 0.6, n))]).tolist()


def test_dp_equals_exhaustive_search_over_all_assignments():
    """Eq. 2 minimised over all m^n assignments equals the DP over contiguous runs of the
    sorted list (Lemma 1) when F grows with the group size."""
    rng = np.random.default_rng(1)
    for trial in range(40):
        n, m = int(rng.integers(1, 8)), int(rng.integers(1, 4))
        L = sorted(rng.integers(1, 50, n).tolist(), reverse=True)
        F = monotone_F(rng, n)
        T = float(rng.uniform(0.5, 2.0))
        mk, sizes = pl.placement_dp(L, m, F, T)
        assert sum(sizes) == n and len(sizes) == m
        assert mk == pytest.approx(pl.brute_force_any_partition(L, m, F, T), rel=1e-12)
        assert mk == pl.makespan_of_sizes(L, sizes, F, T)


def test_dp_equals_exhaustive_contiguous_search_for_any_F():
    rng = np.random.default_rng(2)
    for trial in range(60):
        n, m = int(rng.integers(1, 11)), int(rng.integers(1, 6))
        L = sorted(rng.integers(1, 1000, n).tolist(), reverse=True)
        F = [0.0] + rng.uniform(0.5, 4.0, n).tolist()           # not monotone
        mk, sizes = pl.placement_dp(L, m, F, 1.0)
        # with an F that may fall, using fewer than min(n, m) groups can be better; the DP of
        # Eq. 3 fills min(n, m) workers, so compare on exactly that many runs
        J = min(n, m)
        import itertools
        best = min(pl.makespan_of_sizes(L, [e2 - e1 for e1, e2 in zip((0,) + c, c + (n,))], F)
                   for c in itertools.combinations(range(1, n), J - 1))
        assert mk == best and mk == pl.makespan_of_sizes(L, sizes, F)


def test_closed_forms():
    L = [90, 70, 70, 30, 10, 5]
    n = len(L)
    ones = [0.0] + [1.0] * n
    lin = [float(s) for s in range(n + 1)]
    for m in (1, 2, 3, 6, 9):
        assert pl.placement_dp(L, m, ones, 2.0)[0] == 180.0                      # no interference: longest * T
    assert pl.placement_dp(L, 1, lin, 1.0) == (90.0 * 6, [6])                    # one worker: L1 * F(n)
    mk, sizes = pl.placement_dp(L, 9, lin, 1.0)                                  # more workers than trajectories
    assert mk == 90.0 and sizes == [1] * 6 + [0] * 3
    eq = [40] * 10
    lin10 = [float(s) for s in range(11)]
    for m in (1, 2, 3, 4, 7, 10):
        assert pl.placement_dp(eq, m, lin10, 1.0)[0] == 40.0 * -(-10 // m)       # equal lengths: ceil(n/m)
    assert pl.placement_dp([], 3, [0.0], 1.0) == (0.0, [0, 0, 0])
    with pytest.raises(ValueError):
        pl.placement_dp([1, 2], 2, lin, 1.0)


def test_more_workers_never_hurt_and_straggler_is_isolated():
    rng = np.random.default_rng(3)
    L = sorted(rng.lognormal(8, 1.0, 60).astype(int).tolist(), reverse=True)
    F = monotone_F(rng, 60)
    prev = float("inf")
    for m in range(1, 12):
        mk, sizes = pl.placement_dp(L, m, F, 1.0)
        assert mk <= prev
        prev = mk
    # a straggler far longer than the rest ends up in a smaller group than the short ones
    L2 = [100000] + [100] * 40
    mk, sizes = pl.placement_dp(L2, 2, [float(s) for s in range(42)], 1.0)
    assert sizes == [1, 40] and mk == 100000.0


def test_aggregation_of_short_trajectories():
    rng = np.random.default_rng(4)
    for trial in range(30):
        n, m = int(rng.integers(2, 12)), int(rng.integers(1, 5))
        L = sorted(rng.integers(1, 100, n).tolist(), reverse=True)
        F = monotone_F(rng, n)
        thr, bundle = int(rng.integers(1, 100)), int(rng.integers(1, 5))
        first, count = pl.aggregate_short(L, thr, bundle)
        assert sum(count) == n and first[0] == 0
        assert all(first[i + 1] == first[i] + count[i] for i in range(len(first) - 1))
        assert all(c == 1 for f, c in zip(first, count) if L[f] >= thr)
        assert all(c <= max(bundle, 1) for c in count)
        Le = [L[f] for f in first]
        mk, sizes = pl.placement_dp(Le, m, F, 1.0, counts=count)
        J = min(len(Le), m)
        assert mk == pytest.approx(min(pl.makespan_of_sizes(Le, s, F, 1.0, count) for s in compositions(len(Le), J)))
        full, _ = pl.placement_dp(L, m, F, 1.0)
        if len(Le) >= min(n, m):
            assert mk >= full - 1e-12                  # bundling only removes choices
    first, count = pl.aggregate_short([9, 5, 3], 0, 4)
    assert count == [1, 1, 1]


def compositions(n, parts):
    import itertools
    for c in itertools.combinations(range(1, n), parts - 1):
        e = (0,) + c + (n,)
        yield [e[i + 1] - e[i] for i in range(parts)]


def test_interference_table():
    bs, ts = [1, 4, 16], [10.0, 13.0, 37.0]
    F = pl.interference_table(bs, ts, 20)
    assert F[0] == 0.0 and F[1] == 1.0
    assert F[4] == pytest.approx(1.3) and F[16] == pytest.approx(3.7)
    assert F[2] == pytest.approx(1.1) and F[10] == pytest.approx((13 + 24 * 6 / 12) / 10)
    assert F[20] == pytest.approx((37 + 2.0 * 4) / 10)                    # last slope continued
    # a dip in the profile is flattened: the premise of the DP is a non-decreasing F
    F2 = pl.interference_table([1, 2, 3, 4], [10.0, 14.0, 12.0, 20.0], 4)
    assert F2 == pytest.approx([0.0, 1.0, 1.4, 1.4, 2.0])
    # profile that does not start at batch 1: flat below its first point
    F3 = pl.interference_table([2, 4], [10.0, 20.0], 4)
    assert F3 == pytest.approx([0.0, 1.0, 1.0, 1.5, 2.0])
    with pytest.raises(ValueError):
        pl.interference_table([2, 2], [1.0, 2.0], 3)


def test_simulator_against_step_by_step():
    bs, ts = [1, 2, 8], [1.0, 1.5, 4.0]
    assert pl.simulate_group([37], bs, ts) == 37.0
    assert pl.simulate_group([5] * 8, bs, ts) == 5 * 4.0
    assert pl.simulate_group([], bs, ts) == 0.0
    t_of = pl.profile_time(bs, ts)
    rng = np.random.default_rng(6)
    for trial in range(20):
        L = rng.integers(1, 30, int(rng.integers(1, 10))).tolist()
        total, step = 0.0, 0
        while True:
            active = sum(1 for x in L if x > step)
            if active == 0:
                break
            total += t_of(float(active))
            step += 1
        assert pl.simulate_group(L, bs, ts) == pytest.approx(total, rel=1e-12)
