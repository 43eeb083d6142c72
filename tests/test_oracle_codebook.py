"""Pins for the reference codec's codebook: optimal length-limited lengths and canonical codes."""
import heapq
import itertools
from fractions import Fraction

import numpy as np
import pytest

from oracle import oracle as zo
from paper_2601_21198_amd import synth


def hist_of(pairs):
    h = np.zeros(256, np.uint64)
    for s, c in pairs:
        h[s] = c
    return h


def cost(hist, lengths):
    return int((hist.astype(object) * lengths.astype(object)).sum())


def huffman_lengths(weights):
    """textbook heap construction; returns code lengths for the given positive weights"""
    if len(weights) == 1:
        return [1]
    heap = [(w, i, [i]) for i, w in enumerate(weights)]
    heapq.heapify(heap)
    depth = [0] * len(weights)
    tie = len(weights)
    while len(heap) > 1:
        a = heapq.heappop(heap)
        b = heapq.heappop(heap)
        for i in a[2] + b[2]:
            depth[i] += 1
        heapq.heappush(heap, (a[0] + b[0], tie, a[2] + b[2]))
        tie += 1
    return depth


def brute_force_cost(weights, max_len):
    best = None
    for ls in itertools.product(range(1, max_len + 1), repeat=len(weights)):
        if sum(Fraction(1, 2 ** l) for l in ls) <= 1:
            c = sum(w * l for w, l in zip(weights, ls))
            best = c if best is None else min(best, c)
    return best


def test_no_symbols_and_one_symbol():
    assert not zo.code_lengths(np.zeros(256, np.uint64), 8).any()
    l = zo.code_lengths(hist_of([(121, 1000)]), 8)
    assert l[121] == 1 and l.sum() == 1
    assert zo.kraft_units(l) == 1 << (zo.MAX_LEN - 1)


def test_dyadic_distribution_gets_its_exact_lengths():
    """counts 8,4,2,1,1 are a dyadic distribution: the optimal lengths are 1,2,3,4,4, uniquely"""
    l = zo.code_lengths(hist_of([(10, 8), (20, 4), (30, 2), (40, 1), (50, 1)]), 8)
    assert [l[s] for s in (10, 20, 30, 40, 50)] == [1, 2, 3, 4, 4]


def test_uniform_256_symbols_all_get_eight_bits():
    l = zo.code_lengths(np.full(256, 7, np.uint64), 8)
    assert np.all(l == 8)
    with pytest.raises(zo.OracleError):
        zo.code_lengths(np.full(256, 7, np.uint64), 7)        # 256 symbols do not fit in 7 bits


@pytest.mark.parametrize("max_len", [1, 2, 3, 4])
def test_brute_force_small_alphabets(max_len):
    rng = np.random.default_rng(max_len)
    cases = [[1, 1, 2, 3, 5], [5, 5, 5], [100, 1, 1, 1], [1, 2, 4, 8, 16], [7], [3, 3], [1, 1, 1, 1, 1]]
    cases += [list(rng.integers(1, 50, rng.integers(1, 6))) for _ in range(40)]
    for weights in cases:
        if len(weights) > 2 ** max_len:
            continue
        syms = list(range(100, 100 + len(weights)))
        h = hist_of(zip(syms, weights))
        l = zo.code_lengths(h, max_len)
        assert l.max() <= max_len and np.all(l[syms] >= 1)
        assert zo.kraft_units(l) <= 1 << zo.MAX_LEN
        assert cost(h, l) == brute_force_cost(weights, max_len), weights


def test_equals_huffman_when_the_limit_does_not_bind():
    rng = np.random.default_rng(11)
    for trial in range(30):
        k = int(rng.integers(2, 40))
        weights = [int(x) for x in rng.integers(1, 1000, k)]
        depth = huffman_lengths(weights)
        if max(depth) > zo.MAX_LEN:
            continue
        syms = rng.choice(256, k, replace=False)
        h = hist_of(zip(syms, weights))
        l = zo.code_lengths(h, zo.MAX_LEN)
        assert cost(h, l) == sum(w * d for w, d in zip(weights, depth))


def test_limit_binds_on_fibonacci_weights():
    """Fibonacci weights give the deepest Huffman tree; under a limit the cost rises, never falls,
    and tightening the limit never lowers the cost."""
    fib = [1, 1, 2, 3, 5, 8, 13, 21, 34, 55, 89, 144, 233, 377]
    h = hist_of(zip(range(14), fib))
    depth = huffman_lengths(fib)
    assert max(depth) == 13
    unlimited = sum(w * d for w, d in zip(fib, depth))
    prev = None
    for max_len in range(12, 3, -1):
        l = zo.code_lengths(h, max_len)
        assert l.max() <= max_len
        c = cost(h, l)
        assert c > unlimited
        assert prev is None or c >= prev
        prev = c
        assert zo.kraft_units(l) == 1 << zo.MAX_LEN            # an optimal code is complete


def test_workload_codebooks_are_complete_monotone_and_near_entropy():
    for kind, max_len in (("gauss", 8), ("gauss", 12), ("rare_last", 8), ("wide", 8), ("wide", 12)):
        w = synth.special_tensor(kind, 200000, seed=2)
        e, _ = zo.split(w)
        h = zo.histogram(e)
        l = zo.code_lengths(h, max_len)
        present = np.nonzero(h)[0]
        assert np.all(l[present] >= 1) and not l[h == 0].any() and l.max() <= max_len
        assert zo.kraft_units(l) == 1 << zo.MAX_LEN
        # a more frequent symbol never has a longer code
        for a in present:
            for b in present:
                if h[a] > h[b]:
                    assert l[a] <= l[b]
        p = h[present].astype(np.float64) / h.sum()
        H = -(p * np.log2(p)).sum()
        mean_len = cost(h, l) / int(h.sum())
        assert H <= mean_len < H + 1
        if kind == "gauss":
            assert mean_len < H + 0.12      # Gaussian exponents: within about 0.1 bit of the entropy
        # the limit never helps
        if max_len == 8:
            assert cost(h, l) >= cost(h, zo.code_lengths(h, 12))


def test_canonical_codes_prefix_free_and_ordered():
    rng = np.random.default_rng(5)
    for trial in range(20):
        k = int(rng.integers(2, 60))
        syms = np.sort(rng.choice(256, k, replace=False))
        h = hist_of(zip(syms, [int(x) for x in rng.integers(1, 10000, k)]))
        l = zo.code_lengths(h, 12 if trial % 2 else 8)
        code, n = zo.canonical(l)
        assert n == k
        words = {int(s): format(int(code[s]), "b").zfill(int(l[s])) for s in syms}
        assert all(len(words[int(s)]) == l[s] for s in syms)     # the code value fits in its length
        for a, b in itertools.permutations(syms, 2):
            assert not words[int(b)].startswith(words[int(a)])
        # closed form of the canonical assignment: in (length, symbol) order the codes, read as binary
        # fractions, start at 0 and each begins where the previous one's interval ends
        order = sorted(syms, key=lambda s: (l[s], s))
        acc = Fraction(0)
        for s in order:
            assert Fraction(int(code[s]), 2 ** int(l[s])) == acc
            acc += Fraction(1, 2 ** int(l[s]))
        assert acc == 1
