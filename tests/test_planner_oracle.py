"""Pins for the reference cache-pool planner (App. C, App. D of the paper)."""
import itertools
import math

import numpy as np
import pytest

from oracle import planner as pl


def zipf_inclusion(n, k, s):
    """inclusion probabilities of a k-subset drawn with weights r^-s: exact, by enumeration"""
    w = [(r + 1) ** -s for r in range(n)]
    total = sum(math.prod(c) for c in itertools.combinations(w, k))
    return [w[i] * sum(math.prod(c) for c in itertools.combinations(w[:i] + w[i + 1:], k - 1)) / total for i in range(n)]


def test_elementary_symmetric_is_the_coefficient_of_the_product_polynomial():
    rng = np.random.default_rng(0)
    w = rng.uniform(0.1, 2.0, 9)
    coeffs = np.poly(-w)                       # prod (x + w_i): coefficient of x^(9-n) is R(n)
    for n in range(10):
        assert math.isclose(pl.elementary_symmetric(list(w), n), coeffs[n], rel_tol=1e-10)


@pytest.mark.parametrize("n,k,s", [(6, 2, 1.0), (8, 3, 1.2), (10, 4, 0.7), (7, 1, 2.0), (5, 4, 1.0)])
def test_fitted_probabilities_reproduce_the_inclusion_probabilities(n, k, s):
    f = zipf_inclusion(n, k, s)
    assert math.isclose(sum(f), k, rel_tol=1e-12)
    q, iters = pl.selection_probabilities(f, k)
    assert iters < 5000 and all(0 < x < 1 for x in q)
    # brute force over every k-subset with P(S) ~ prod q/(1-q)
    w = [x / (1 - x) for x in q]
    subsets = list(itertools.combinations(range(n), k))
    p = np.array([math.prod(w[i] for i in S) for S in subsets])
    p /= p.sum()
    for i in range(n):
        assert math.isclose(sum(pi for pi, S in zip(p, subsets) if i in S), f[i], abs_tol=1e-9)
    # the same, as the conditional of independent selections given that exactly k occur (Sec. 3.4)
    joint = np.array([math.prod(q[i] if i in S else 1 - q[i] for i in range(n)) for S in subsets])
    assert np.allclose(joint / joint.sum(), p, atol=1e-12)


def test_uniform_inclusion_gives_equal_probabilities():
    q, _ = pl.selection_probabilities([3 / 12] * 12, 3)
    assert max(q) - min(q) < 1e-12


@pytest.mark.parametrize("n", [1, 4, 9])
def test_hit_distribution_against_enumeration_and_binomial(n):
    rng = np.random.default_rng(n)
    q = list(rng.uniform(0.02, 0.9, n))
    phi = pl.hit_distribution(q)
    brute = [0.0] * (n + 1)
    for bits in itertools.product((0, 1), repeat=n):
        brute[sum(bits)] += math.prod(qi if b else 1 - qi for qi, b in zip(q, bits))
    assert np.allclose(phi, brute, atol=1e-14) and math.isclose(sum(phi), 1.0, rel_tol=1e-12)
    same = pl.hit_distribution([0.3] * n)
    assert np.allclose(same, [math.comb(n, h) * 0.3 ** h * 0.7 ** (n - h) for h in range(n + 1)], atol=1e-14)
    assert pl.hit_distribution([]) == [1.0]


def test_makespan_worked_example():
    # n_SM = 3*(4-3) = 3, n_E = 3*4*(4-2) = 24, T_IO = 3*3 + 24*0.5 = 21, n_D = 3*4*3 = 36, T_dec = (12 + 72)/2 = 42
    assert pl.makespan(4, (1, 1, 1, 0), c=2.0, v=0.5, u=3.0, L=2, K=4, n=3) == 42.0
    # everything in F costs nothing; everything missed reads and decompresses all of it
    assert pl.makespan(4, (4, 0, 0, 0), 2.0, 0.5, 3.0, 2, 4, 3) == 0.0
    assert pl.makespan(2, (0, 0, 0, 0), c=1.0, v=1.0, u=10.0, L=4, K=2, n=1) == max(2 * 10 + 4 * 1, (4 + 4) / 4)
    # SM-pool hits save SM reads only, E-pool hits save E-chunk reads only
    assert pl.makespan(2, (0, 0, 2, 0), 1.0, 1.0, 10.0, 4, 2, 1) == 4.0
    assert pl.makespan(2, (0, 0, 0, 2), 1.0, 1.0, 10.0, 4, 2, 1) == 20.0


@pytest.mark.parametrize("slots", [(2, 0, 0, 0), (1, 2, 1, 3), (0, 3, 0, 2), (3, 3, 2, 2), (0, 0, 0, 0)])
def test_expected_makespan_closed_forms(slots):
    """with delays chosen so that the makespan is linear in the hits, the expectation under the hit-pattern
    distribution must come out as k minus the inclusion probabilities of the ranks the pools cover"""
    n, k = 10, 3
    f = zipf_inclusion(n, k, 1.1)
    q, _ = pl.selection_probabilities(f, k)
    # c = 1, no I/O cost, one thread, one shard, one tensor: makespan = k - h_F
    got = pl.expected_makespan(q, slots, k, c=1.0, v=0.0, u=0.0, L=1, K=1, n=1)
    assert math.isclose(got, k - sum(f[: slots[0]]), abs_tol=1e-8)
    # only SM reads cost: makespan = k - h_F - h_C - h_S
    got = pl.expected_makespan(q, slots, k, c=0.0, v=0.0, u=1.0, L=1, K=1, n=1)
    assert math.isclose(got, k - sum(f[: slots[0] + slots[1] + slots[2]]), abs_tol=1e-8)
    # only E-chunk reads cost (L large so the I/O side dominates): makespan = k - h_F - h_C - h_E
    got = pl.expected_makespan(q, slots, k, c=0.0, v=1.0, u=0.0, L=1000, K=1, n=1)
    covered = sum(f[: slots[0] + slots[1]]) + sum(f[slots[0] + slots[1] + slots[2]: sum(slots)])
    assert math.isclose(got, k - covered, abs_tol=1e-8)


def test_slots_for_ratios():
    assert pl.slots_for_ratios((0.5, 0.25, 0.25, 0.0), 100.0, (10.0, 7.0, 5.0, 2.0), 60) == [5, 3, 5, 0]
    assert pl.slots_for_ratios((1.0, 0.0, 0.0, 0.0), 1000.0, (10.0, 7.0, 5.0, 2.0), 8) == [8, 0, 0, 0]
    assert pl.slots_for_ratios((0.5, 0.5, 0.0, 0.0), 1000.0, (10.0, 7.0, 5.0, 2.0), 8) == [8, 0, 0, 0]


def test_plan_degenerate_cases():
    n, k = 8, 2
    f = zipf_inclusion(n, k, 1.0)
    sizes = (12.0, 8.5, 6.0, 2.5)
    common = dict(k=k, c=1.0, v=0.4, u=1.0, L=4, K=4, n=3, bytes_per_expert=sizes, grid=4)
    ratios, slots, cost = pl.plan_pools(f, memory=12.0 * 8, active=(True,) * 4, **common)
    assert ratios == [1.0, 0.0, 0.0, 0.0] and slots == [8, 0, 0, 0] and cost == 0.0
    ratios, slots, cost = pl.plan_pools(f, memory=30.0, active=(False, True, False, False), **common)
    assert ratios == [0.0, 1.0, 0.0, 0.0] and slots == [3, 0, 0, 0][1:2] * 0 + [0, 3, 0, 0]
    # the chosen partition is at least as good as giving all memory to one pool
    ratios, slots, best = pl.plan_pools(f, memory=30.0, active=(True,) * 4, **common)
    q, _ = pl.selection_probabilities(f, k)
    for p in range(4):
        one = [0.0] * 4
        one[p] = 1.0
        s = pl.slots_for_ratios(one, 30.0, sizes, n)
        assert best <= pl.expected_makespan(q, s, k, 1.0, 0.4, 1.0, 4, 4, 3) + 1e-12
