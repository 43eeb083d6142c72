"""The library's cache-pool planner against the reference planner (float64; tolerance 1e-8 relative: both
run the same fixed-point iteration to an inclusion-probability error below 1e-12 and then only add and
multiply a few thousand positive terms)."""
import math

import numpy as np
import pytest

from oracle import planner as pl
from paper_2601_21198_amd import zipmoe as zm
from test_planner_oracle import zipf_inclusion

TOL = 1e-8


def skewed_inclusion(n, k, s=1.2, scale=3.0):
    """a feasible rank-based inclusion list for n ranks: the inclusion probabilities of independent draws with
    odds scale * r^-s, conditioned on exactly k of them, from the reference hit-count recursion"""
    w = scale * np.arange(1, n + 1, dtype=np.float64) ** -s
    q = list(w / (1 + w))
    all_k = pl.hit_distribution(q)[k]
    return np.array([q[i] * pl.hit_distribution(q[:i] + q[i + 1:])[k - 1] / all_k for i in range(n)])


def costs(c, v, u, L, K, n):
    return zm.PlanCosts(c, v, u, L, K, n)


@pytest.mark.parametrize("n,k,s", [(6, 2, 1.0), (8, 3, 1.2), (12, 4, 0.7), (7, 1, 2.0), (5, 4, 1.0), (16, 4, 1.1)])
def test_selection_probabilities(n, k, s):
    f = zipf_inclusion(n, k, s)
    q, iters = zm.plan_selection_probabilities(f, k)
    ref, ref_iters = pl.selection_probabilities(f, k)
    assert iters == ref_iters
    assert np.allclose(q, ref, rtol=TOL, atol=0)


def test_selection_probabilities_at_model_size_reproduce_inclusion():
    """60 experts, top-4 (too many subsets to enumerate in the reference): the inclusion probabilities implied
    by q, computed with the reference hit-count recursion, must be the input"""
    n, k = 60, 4
    f = skewed_inclusion(n, k)
    assert math.isclose(f.sum(), k, rel_tol=1e-12)
    q, iters = zm.plan_selection_probabilities(f, k)
    assert iters < 5000
    all_k = pl.hit_distribution(list(q))[k]
    for i in (0, 1, 7, 30, 59):
        others = list(q[:i]) + list(q[i + 1:])
        assert math.isclose(q[i] * pl.hit_distribution(others)[k - 1] / all_k, f[i], abs_tol=1e-9)


def test_hit_distribution():
    rng = np.random.default_rng(2)
    for n in (0, 1, 5, 40):
        q = rng.uniform(0.01, 0.9, n)
        assert np.allclose(zm.plan_hit_distribution(q), pl.hit_distribution(list(q)), rtol=TOL, atol=1e-300)


def test_makespan():
    rng = np.random.default_rng(3)
    for _ in range(200):
        k = int(rng.integers(1, 9))
        h = [0, 0, 0, 0]
        for _ in range(int(rng.integers(0, k + 1))):
            h[int(rng.integers(0, 4))] += 1
        c, v, u = rng.uniform(0, 5, 3)
        L, K, n = int(rng.integers(1, 9)), int(rng.integers(1, 9)), int(rng.integers(1, 4))
        assert math.isclose(zm.plan_makespan(k, h, costs(c, v, u, L, K, n)), pl.makespan(k, h, c, v, u, L, K, n), rel_tol=1e-12)
    assert zm.plan_makespan(4, (1, 1, 1, 0), costs(2.0, 0.5, 3.0, 2, 4, 3)) == 42.0     # the worked example
    with pytest.raises(zm.ZipMoEError):
        zm.plan_makespan(2, (2, 1, 0, 0), costs(1, 1, 1, 1, 1, 1))


@pytest.mark.parametrize("slots", [(2, 0, 0, 0), (1, 2, 1, 3), (0, 3, 0, 2), (3, 3, 2, 2), (0, 0, 0, 0), (10, 0, 0, 0)])
def test_expected_makespan(slots):
    n, k = 10, 3
    f = zipf_inclusion(n, k, 1.1)
    q, _ = pl.selection_probabilities(f, k)
    for c, v, u, L, K, nt in ((1.0, 0.4, 1.0, 4, 4, 3), (0.2, 2.0, 0.1, 2, 8, 1), (1.0, 0.0, 0.0, 1, 1, 1)):
        got = zm.plan_expected_makespan(q, slots, k, costs(c, v, u, L, K, nt))
        assert math.isclose(got, pl.expected_makespan(q, slots, k, c, v, u, L, K, nt), rel_tol=TOL, abs_tol=1e-12)
    # closed form: with only decompression costing, the expectation is k minus the inclusion mass of F
    got = zm.plan_expected_makespan(q, slots, k, costs(1.0, 0.0, 0.0, 1, 1, 1))
    assert math.isclose(got, k - sum(f[: slots[0]]), abs_tol=1e-8)


@pytest.mark.parametrize("memory,mask", [(30.0, 15), (55.0, 15), (20.0, 0b0110), (96.0, 15), (40.0, 0b1010), (0.0, 15)])
def test_plan_pools(memory, mask):
    n, k = 8, 2
    f = zipf_inclusion(n, k, 1.0)
    sizes = (12.0, 8.5, 6.0, 2.5)
    c, v, u, L, K, nt = 1.0, 0.4, 1.0, 4, 4, 3
    active = [bool((mask >> p) & 1) for p in range(4)]
    ref_ratios, ref_slots, ref_cost = pl.plan_pools(f, k, c, v, u, L, K, nt, memory, sizes, 4, active)
    ratios, slots, cost = zm.plan_pools(f, k, costs(c, v, u, L, K, nt), memory, sizes, 4, mask)
    assert math.isclose(cost, ref_cost, rel_tol=TOL, abs_tol=1e-12)
    assert ratios == ref_ratios and slots == ref_slots


def test_plan_feeds_the_cache_configuration():
    """a budget of 40 % of the bf16 size of a 60-expert layer, costs in the proportions measured on an MI355X
    (SM bytes cross the host link 2.4 times slower than E-chunks; decode is far cheaper than either)"""
    n, k = 60, 4
    f = skewed_inclusion(n, k)
    sizes = (17.3e6, 12.2e6, 8.65e6, 3.55e6)
    ratios, slots, cost = zm.plan_pools(f, k, costs(0.05, 0.4, 1.0, 1, 1, 3), 0.4 * 60 * 17.3e6, sizes, 10)
    assert math.isclose(sum(ratios), 1.0, rel_tol=1e-12) and sum(slots) <= n and all(s >= 0 for s in slots)
    q, _ = zm.plan_selection_probabilities(f, k)
    for single in range(4):
        r = [0.0] * 4
        r[single] = 1.0
        s = pl.slots_for_ratios(r, 0.4 * 60 * 17.3e6, sizes, n)
        assert cost <= zm.plan_expected_makespan(q, s, k, costs(0.05, 0.4, 1.0, 1, 1, 3)) + 1e-12


def test_bad_arguments():
    with pytest.raises(zm.ZipMoEError):
        zm.plan_selection_probabilities([0.5, 0.5], 3)
    with pytest.raises(zm.ZipMoEError):
        zm.plan_selection_probabilities([0.5, 1.5], 1)
    with pytest.raises(zm.ZipMoEError):
        zm.plan_expected_makespan([0.5] * 4, (3, 3, 0, 0), 2, costs(1, 1, 1, 1, 1, 1))
    with pytest.raises(zm.ZipMoEError):
        zm.plan_pools([0.5] * 4, 2, costs(1, 1, 1, 1, 1, 1), 10.0, (1.0, 1.0, 1.0, 1.0), 4, 0)
    with pytest.raises(zm.ZipMoEError):
        zm.plan_pools([0.5] * 4, 2, costs(1, 1, 1, 0, 1, 1), 10.0, (1.0, 1.0, 1.0, 1.0), 4, 15)
