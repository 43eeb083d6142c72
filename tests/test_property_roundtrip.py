"""Randomised round trips over tensor length, exponent statistics and codec geometry (CPU only)."""
import numpy as np
from hypothesis import HealthCheck, given, settings, strategies as st

from oracle import oracle as zo
from paper_2601_21198_amd import zipmoe as zm


@st.composite
def cases(draw):
    n = draw(st.integers(0, 6000))
    k = draw(st.integers(1, 60))                      # distinct exponent values
    skew = draw(st.floats(0.0, 3.0))
    seed = draw(st.integers(0, 2 ** 31 - 1))
    W = draw(st.sampled_from([512, 1024, 2048]))
    C = W * draw(st.sampled_from([1, 2, 4]))
    max_len = draw(st.sampled_from([6, 8, 9, 12]))
    return n, k, skew, seed, C, W, max_len


@settings(max_examples=120, deadline=None, suppress_health_check=[HealthCheck.too_slow])
@given(cases())
def test_random_tensors_round_trip_everywhere(case):
    n, k, skew, seed, C, W, max_len = case
    rng = np.random.default_rng(seed)
    if k > 2 ** max_len:
        k = 2 ** max_len
    exps = rng.choice(256, k, replace=False)
    p = (np.arange(1, k + 1, dtype=np.float64)) ** (-skew)
    p /= p.sum()
    e = exps[rng.choice(k, n, p=p)].astype(np.uint16)
    w = (rng.integers(0, 2, n, dtype=np.uint16) << 15) | (e << 7) | rng.integers(0, 128, n, dtype=np.uint16)
    w = w.astype(np.uint16)

    hist = zm.exponent_histogram(w)
    lengths = zm.build_codebook(hist, max_len)
    ref_lengths = zo.code_lengths(hist, max_len)
    assert int((hist * lengths).sum()) == int((hist * ref_lengths).sum())

    blob, offs = zm.encode(w, C, W, lengths)
    assert np.array_equal(blob, zo.encode(w, C, W, lengths))          # library and reference agree byte for byte
    zm.validate_blob(blob)
    assert zo.check_table(blob) == zo.OK
    assert np.array_equal(zo.decode(blob), w)                           # reference decoder: lossless
    assert np.array_equal(zm.decode_exponents_host(blob, n_threads=2), zo.split(w)[0])
    # the reference encoder with its own lengths also round-trips, through both decoders
    blob2 = zo.encode(w, C, W, ref_lengths)
    assert np.array_equal(zo.decode(blob2), w)
    if n:
        zm.validate_blob(blob2)
        assert np.array_equal(zm.decode_exponents_host(blob2), zo.split(w)[0])
