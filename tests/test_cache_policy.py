"""The rank-threshold dispatch rule of the expert cache (Sec. 3.4), a pure host function."""
import numpy as np
import pytest

from paper_2601_21198_amd import zipmoe as zm

F, C, S, E, NONE = zm.POOL_FULL, zm.POOL_COMPRESSED, zm.POOL_SM, zm.POOL_E, zm.POOL_NONE


def pools_by_rank(slots, tolerance, n=20):
    counts = np.arange(n, 0, -1).astype(np.uint64) * 10          # expert i has rank i
    return [zm.cache_dispatch(counts, slots, tolerance, e) for e in range(n)]


def test_thresholds_are_cumulative_capacities_plus_tolerance():
    # tau_F = 2, tau_C = 5, tau_S = 9, tau_E = 14 : r < tau_i picks the first pool
    assert pools_by_rank((2, 3, 4, 5), 0) == [F] * 2 + [C] * 3 + [S] * 4 + [E] * 5 + [NONE] * 6
    # a tolerance of 1 shifts every threshold by one rank
    assert pools_by_rank((2, 3, 4, 5), 1) == [F] * 3 + [C] * 3 + [S] * 4 + [E] * 5 + [NONE] * 5
    assert pools_by_rank((2, 3, 4, 5), 3) == [F] * 5 + [C] * 3 + [S] * 4 + [E] * 5 + [NONE] * 3


def test_empty_pools_are_skipped():
    assert pools_by_rank((0, 3, 0, 2), 1) == [C] * 4 + [E] * 2 + [NONE] * 14
    assert pools_by_rank((0, 0, 0, 0), 5) == [NONE] * 20
    assert pools_by_rank((4, 0, 0, 0), 0) == [F] * 4 + [NONE] * 16


def test_rank_comes_from_counts_with_ties_to_the_lower_id():
    counts = np.array([5, 9, 9, 1, 5, 0], np.uint64)            # order: 1, 2, 0, 4, 3, 5
    got = [zm.cache_dispatch(counts, (1, 1, 1, 1), 0, e) for e in range(6)]
    assert got == [S, F, C, NONE, E, NONE]


def test_bad_arguments():
    counts = np.ones(4, np.uint64)
    for args in (((1, 1, 1, 1), 0, 4), ((1, 1, 1, 1), 0, -1), ((1, 1, 1, 1), -1, 0)):
        with pytest.raises(zm.ZipMoEError):
            zm.cache_dispatch(counts, *args)
