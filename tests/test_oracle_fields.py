"""Pins for the bit-field decomposition of the reference codec (Sec. 2.2, Sec. 3.1, Sec. 3.3)."""
import math

import numpy as np

from oracle import oracle as zo
from paper_2601_21198_amd import synth


def all_words():
    return np.arange(65536, dtype=np.uint32).astype(np.uint16)


def test_split_merge_exhaustive():
    w = all_words()
    e, sm = zo.split(w)
    assert e.dtype == np.uint8 and sm.dtype == np.uint8
    assert e.size == w.size and sm.size == w.size      # each stream is half of the tensor's bytes (Sec. 2.3 (III))
    assert np.array_equal(zo.merge(e, sm), w)


def test_fields_match_bf16_value_formula():
    """value = (-1)^sign * 2^(exponent-127) * 1.mantissa (Sec. 2.2), checked for every normal pattern
    against the float32 that the same 16 bits denote."""
    w = all_words()
    e, sm = zo.split(w)
    with np.errstate(invalid="ignore"):
        val = synth.bf16_to_float(w).astype(np.float64)
    normal = (e > 0) & (e < 255)
    sign = (sm >> 7).astype(np.float64)
    mant = (sm & 0x7F).astype(np.float64)
    want = (-1.0) ** sign * np.exp2(e.astype(np.float64) - 127.0) * (1.0 + mant / 128.0)
    assert np.array_equal(val[normal], want[normal])
    # exponent 0: zeros and subnormals, |v| < 2^-126; exponent 255: inf / nan
    assert np.all(np.abs(val[e == 0]) < 2.0 ** -126)
    assert np.all(~np.isfinite(val[e == 255]))
    # the sign bit of the sign-mantissa byte is the sign of the value
    finite_nonzero = np.isfinite(val) & (val != 0)
    assert np.array_equal(sm[finite_nonzero] >> 7, (val[finite_nonzero] < 0).astype(np.uint8))


def test_merge_is_injective_on_pairs():
    """all 65536 (exponent, sign-mantissa) pairs give distinct words"""
    e = np.repeat(np.arange(256, dtype=np.uint8), 256)
    sm = np.tile(np.arange(256, dtype=np.uint8), 256)
    w = zo.merge(e, sm)
    assert np.unique(w).size == 65536


def test_histogram_counts():
    rng = np.random.default_rng(3)
    e = rng.integers(0, 256, 10000, dtype=np.uint8)
    assert np.array_equal(zo.histogram(e), np.bincount(e, minlength=256).astype(np.uint64))


def gaussian_exponent_pmf(sigma: float) -> np.ndarray:
    """P(exponent field = e) for a N(0, sigma^2) draw rounded to bf16 (nearest, ties to even).
    A value rounds into binade e when |x| lies in [2^(e-127) - h_lo, 2^(e-126) - h_hi) with h the half
    ulp of the binade below / of this binade; ties have probability 0."""
    p = np.zeros(256)
    cdf = lambda a: math.erf(a / (sigma * math.sqrt(2.0)))
    for e in range(1, 255):
        lo = 2.0 ** (e - 127)
        hi = 2.0 ** (e - 126)
        lo_edge = lo - (lo / 2) / 256.0 if e > 1 else lo - 2.0 ** -134     # half ulp of the binade below
        hi_edge = hi - lo / 256.0                                           # half ulp of this binade
        p[e] = cdf(hi_edge) - cdf(lo_edge)
    p[0] = 1.0 - p.sum()
    return p


def test_exponent_histogram_matches_gaussian_closed_form():
    """The exponent field the split extracts has the distribution mathematics predicts for the generator."""
    sigma = 0.02
    w = synth.special_tensor("gauss", 1 << 20, seed=5)
    e, _ = zo.split(w)
    emp = zo.histogram(e).astype(np.float64) / e.size
    pmf = gaussian_exponent_pmf(sigma)
    big = pmf > 1e-3
    assert np.all(np.abs(emp[big] - pmf[big]) < 5 * np.sqrt(pmf[big] / e.size) + 1e-4)
    # the most likely exponents of N(0, 0.02^2): 121 (0.0156..0.0312) then 120
    assert int(np.argmax(emp)) == 121 and int(np.argsort(emp)[-2]) == 120
    H = -(pmf[pmf > 0] * np.log2(pmf[pmf > 0])).sum()
    # the real expert weights measured in Fig. 2 have 2.55 .. 2.65 bits; the stand-in is close to that
    assert 2.45 < H < 2.70


def test_workload_entropy_close_to_paper():
    for wl in (synth.CFG1, synth.CFG2):
        w = synth.expert_matrix(wl, 0, 0, 0)
        e, _ = zo.split(w)
        h = zo.histogram(e).astype(np.float64)
        p = h[h > 0] / h.sum()
        H = -(p * np.log2(p)).sum()
        assert 2.4 < H < 2.8, (wl.name, H)
        assert (h > 0).sum() <= 48       # the paper's models use 29..38 of the 256 exponent values
