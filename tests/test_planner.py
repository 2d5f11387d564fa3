"""Scale-up model and Algorithm 1 (Section 4.1): the oracle against closed forms and invariants,
and the library's host functions against the oracle.  No GPU."""
import math
import random

import pytest

from oracle import planner as P
from paper_2507_18006_amd import binding as B


# ---------------------------------------------------------------- oracle pins
def test_no_replication_means_no_speedup():
    for n in (1, 5, 40):
        assert P.speedup_homo([1] * n, 0.0) == 1.0
        assert P.speedup_homo([1] * n, 0.3) == 1.0
        bs = [[8.0]] * n
        assert P.speedup([1] * n, bs, [[3.0]] * n, [[1.0]] * n, 5120.0, 256.0, 2.0) == 1.0


def test_uniform_parallelism_is_amdahls_law():
    """With the same degree p everywhere Eq. 4 is Amdahl's law with serial fraction gamma."""
    for p in (2, 3, 8):
        for gamma in (0.0, 0.05, 0.5):
            want = 1.0 / (gamma + (1.0 - gamma) / p)
            assert math.isclose(P.speedup_homo([p] * 7, gamma), want, rel_tol=1e-15)
    assert P.speedup_homo([4] * 3, 0.0) == 4.0          # free communication: the ideal speed-up
    assert math.isclose(P.speedup_homo([10 ** 6] * 3, 0.25), 4.0, rel_tol=1e-5)   # bounded by 1 / gamma


def test_general_form_reduces_to_the_homogeneous_one():
    """Even splits on equal devices: Eq. 3 equals Eq. 4 with gamma = delta C / (d B)."""
    rng = random.Random(3)
    for _ in range(20):
        n = rng.randint(1, 12)
        p = [rng.randint(1, 5) for _ in range(n)]
        d, l, C, Bw, delta, batch = 5120.0, 256.0, 3.0e5, 40.0, rng.uniform(0.5, 3.0), 64.0
        bs = [[batch / p[i]] * p[i] for i in range(n)]
        cap = [[C] * p[i] for i in range(n)]
        bw = [[Bw] * p[i] for i in range(n)]
        gamma = delta * C / (d * Bw)
        assert math.isclose(P.speedup(p, bs, cap, bw, d, l, delta), P.speedup_homo(p, gamma), rel_tol=1e-12)


def test_slowest_replica_sets_a_layers_time():
    """Eq. 1 takes the maximum over a layer's instances: moving work to the slower one hurts."""
    d, l = 64.0, 16.0
    even = P.speedup([2], [[8.0, 8.0]], [[1.0, 1.0]], [[1e30, 1e30]], d, l, 1.0)
    skew = P.speedup([2], [[4.0, 12.0]], [[1.0, 1.0]], [[1e30, 1e30]], d, l, 1.0)
    assert math.isclose(even, 2.0, rel_tol=1e-12) and math.isclose(skew, 16.0 / 12.0, rel_tol=1e-12)
    # shares proportional to capacity equalise the instances
    prop = P.speedup([2], [[4.0, 12.0]], [[1.0, 3.0]], [[1e30, 1e30]], d, l, 1.0)
    assert math.isclose(prop, 4.0, rel_tol=1e-12)


def test_continuity_ordering():
    assert P.sort_candidates_by_continuity([], 8, 3) == [0, 1, 2]          # empty node: layer order
    assert P.sort_candidates_by_continuity([5, 6], 8, 3) == [4, 3, 2]      # grow the run, lower index on ties
    assert P.sort_candidates_by_continuity([0, 1, 2], 3, 5) == []
    assert P.sort_candidates_by_continuity([2], 4, 10) == [1, 0, 3]
    # joining two runs beats extending one
    assert P.sort_candidates_by_continuity([0, 1, 3, 4], 8, 1) == [2]


def test_greedy_scale_up_properties():
    rng = random.Random(11)
    for _ in range(30):
        n = rng.randint(2, 40)
        p0 = [rng.randint(1, 2) for _ in range(n)]
        nodes = [rng.randint(0, 12) * 100 + rng.randint(0, 99) for _ in range(rng.randint(0, 5))]
        gamma = rng.uniform(0.0, 0.4)
        p, placed, sp = P.plan_scale_up(p0, gamma, nodes, 100)
        assert all(a >= b for a, b in zip(p, p0))
        assert sum(p) - sum(p0) == sum(sum(r) for r in placed)
        for g, avail in enumerate(nodes):
            assert sum(placed[g]) <= avail // 100
            held = [i for i in range(n) if placed[g][i]]
            if held:                                                        # an empty node fills one contiguous run from layer 0
                assert held == list(range(len(held)))
        assert sp >= P.speedup_homo(p0, gamma) and math.isclose(sp, P.speedup_homo(p, gamma), rel_tol=1e-15)
    # gamma >= 1: replication cannot help, nothing is placed
    p, placed, sp = P.plan_scale_up([1] * 6, 1.0, [1000], 100)
    assert p == [1] * 6 and sp == 1.0 and sum(placed[0]) == 0


def test_greedy_scale_up_is_the_best_subset_of_its_offers():
    """Eq. 4 grows with every p_i while gamma < 1, so no subset of the offers beats taking them
    all: the fold's result equals an exhaustive search over the subsets (small cases)."""
    import itertools
    rng = random.Random(13)
    for _ in range(25):
        n = rng.randint(1, 6)
        p0 = [rng.randint(1, 3) for _ in range(n)]
        nodes = [rng.randint(0, 350) for _ in range(rng.randint(1, 3))]
        gamma = rng.uniform(0.0, 0.6)
        placed0 = [[0] * n for _ in nodes]
        offers = P.scale_up_offers(n, nodes, 100, placed0)
        best = 0.0
        for r in range(len(offers) + 1):
            for sub in itertools.combinations(offers, r):
                p = list(p0)
                for _, layer in sub:
                    p[layer] += 1
                best = max(best, P.speedup_homo(p, gamma))
        got = P.plan_scale_up(p0, gamma, nodes, 100)
        assert math.isclose(got[2], best, rel_tol=1e-14)
        assert sum(got[0]) - sum(p0) == len(offers)


# ---------------------------------------------------------------- batch shares from capacities (Eq. 1)
def compositions(n, k):
    if k == 1:
        yield (n,)
        return
    for first in range(n + 1):
        for rest in compositions(n - first, k - 1):
            yield (first,) + rest


def test_shares_from_capacity_minimise_the_slowest_instance():
    """Against exhaustive search over every way to cut n into k non-negative integers."""
    rng = random.Random(17)
    for _ in range(200):
        k = rng.randint(1, 4)
        n = rng.randint(0, 14)
        cap = [rng.choice([1.0, 2.0, 3.0, 0.5, 10.0, 1.7]) for _ in range(k)]
        got = P.shares_from_capacity(n, cap)
        assert len(got) == k and sum(got) == n and min(got) >= 0
        best = min(P.slowest_instance(c, cap) for c in compositions(n, k))
        assert P.slowest_instance(got, cap) == best, (n, cap, got)


def test_shares_from_capacity_special_cases():
    import oracle
    # equal capacities: the paper's contiguous split, 15 -> 7 + 8 (Section 3.1)
    assert P.shares_from_capacity(15, [1.0, 1.0]) == [7, 8]
    for n in (0, 1, 7, 15, 64, 1000):
        for k in (1, 2, 3, 4, 7, 16):
            b = oracle.split_bounds(n, k)
            assert P.shares_from_capacity(n, [2.5] * k) == [b[j + 1] - b[j] for j in range(k)]
    # shares proportional to capacity: 1 : 3 on 16 -> 4 + 12, the case the speed-up model prices above
    assert P.shares_from_capacity(16, [1.0, 3.0]) == [4, 12]
    assert P.shares_from_capacity(5, [10.0, 1.0]) == [5, 0]     # the weighted floor split alone would say 4 + 1
    assert P.shares_from_capacity(5, [1.0, 10.0]) == [0, 5]
    # the model's own arithmetic: proportional shares equalise the instances (Eq. 1)
    sh = P.shares_from_capacity(64, [1.0, 3.0])
    assert sh == [16, 48] and P.slowest_instance(sh, [1.0, 3.0]) == 16.0


def test_library_shares_match_oracle():
    rng = random.Random(19)
    for _ in range(300):
        k = rng.randint(1, 16)
        n = rng.choice([0, 1, 2, 15, 64, 100, 4096, rng.randint(0, 100000)])
        cap = [rng.choice([1.0, 1.0, 2.0, 3.0, 0.25, rng.uniform(0.1, 50.0)]) for _ in range(k)]
        assert B.shares_from_capacity(n, cap) == P.shares_from_capacity(n, cap), (n, cap)
    for bad in ((5, []), (5, [1.0, 0.0]), (5, [1.0, -2.0]), (-1, [1.0]), (5, [float("nan")]), (5, [1.0] * 17)):
        with pytest.raises(B.CcsError):
            B.shares_from_capacity(*bad)


# ---------------------------------------------------------------- library == oracle
def test_library_speedup_matches_oracle():
    rng = random.Random(5)
    for _ in range(50):
        n = rng.randint(1, 30)
        p = [rng.randint(1, 6) for _ in range(n)]
        gamma = rng.uniform(0.0, 0.9)
        assert math.isclose(B.speedup_homo(p, gamma), P.speedup_homo(p, gamma), rel_tol=1e-14)
        bs = [[rng.uniform(1, 16) for _ in range(p[i])] for i in range(n)]
        cap = [[rng.uniform(1, 9) for _ in range(p[i])] for i in range(n)]
        bw = [[rng.uniform(1, 9) for _ in range(p[i])] for i in range(n)]
        a = B.speedup(p, bs, cap, bw, 5120.0, 256.0, 1.7)
        assert math.isclose(a, P.speedup(p, bs, cap, bw, 5120.0, 256.0, 1.7), rel_tol=1e-12)
    assert B.speedup_homo([1, 0, 2], 0.1) == 0.0


def test_library_planner_matches_oracle():
    rng = random.Random(7)
    for _ in range(60):
        n = rng.randint(1, 48)
        p0 = [rng.randint(1, 3) for _ in range(n)]
        nodes = [rng.randint(0, 2000) for _ in range(rng.randint(0, 6))]
        placed = [[1 if rng.random() < 0.2 else 0 for _ in range(n)] for _ in nodes] if rng.random() < 0.5 else None
        gamma = rng.choice([0.0, 0.02, 0.3, 1.0, 1.5])
        want = P.plan_scale_up(p0, gamma, nodes, 150, placed)
        got = B.plan_scale_up(p0, gamma, nodes, 150, placed)
        assert got[0] == want[0] and got[1] == want[1]
        assert math.isclose(got[2], want[2], rel_tol=1e-14)
    with pytest.raises(B.CcsError):
        B.plan_scale_up([1, 0], 0.1, [500], 100)
