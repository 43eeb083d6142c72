"""Pins for the reference codec's serialised format: exact round trip, sizes, structure."""
import itertools
import os

import numpy as np
import pytest

from oracle import oracle as zo
from paper_2601_21198_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def roundtrip(w, C, W, max_len=8):
    blob, lengths = zo.encode_tensor(w, C, W, max_len)
    assert zo.check_table(blob) == zo.OK
    out = zo.decode(blob)
    assert out.dtype == np.uint16 and np.array_equal(out, np.asarray(w).reshape(-1))
    return blob, lengths


def chunk_table(blob):
    """(header, 64-bit offset|mode word of every table entry, stream offsets of every entry)"""
    h = zo.header(blob)
    stride = h["table_stride"]
    assert stride == -(-(8 + 4 * (h["chunk_values"] // h["stream_values"] + 1)) // 8) * 8
    raw = blob[h["table_offset"]: h["table_offset"] + stride * (h["n_chunks"] + 1)].reshape(h["n_chunks"] + 1, stride)
    words = np.ascontiguousarray(raw[:, :8]).view("<u8").reshape(-1)
    offs = np.ascontiguousarray(raw[:, 8:]).view("<u4").reshape(h["n_chunks"] + 1, -1)
    return h, words, offs


def test_all_65536_patterns_round_trip():
    """losslessness holds for every bit pattern: zeros, subnormals, infinities, NaN payloads included"""
    w = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    rng = np.random.default_rng(0)
    roundtrip(w, 4096, 4096)
    roundtrip(rng.permutation(w), 4096, 2048, 12)


@pytest.mark.parametrize("kind", ["all_equal", "two_exponents", "uniform_u16", "rare_last", "gauss", "wide"])
@pytest.mark.parametrize("n", [0, 1, 7, 8, 9, 511, 512, 513, 4095, 4096, 4097, 9000])
def test_sizes_and_kinds_round_trip(kind, n):
    w = synth.special_tensor(kind, n, seed=n)
    for C, W, max_len in ((4096, 4096, 8), (4096, 1024, 12), (1024, 512, 8)):
        blob, _ = roundtrip(w, C, W, max_len)
        h = zo.header(blob)
        assert h["n_values"] == n and h["n_chunks"] == -(-n // C)
        assert h["blob_size"] == blob.size and blob.size % 256 == 0
        assert blob.size <= zo.lib().zo_encode_bound(n, C, W)
        # the sign-mantissa section is exactly one byte per value (half of the tensor, Sec. 2.3 (III))
        assert h["e_offset"] - h["sm_offset"] == -(-n // 256) * 256
        _, sm = zo.split(w)
        assert np.array_equal(blob[h["sm_offset"]: h["sm_offset"] + n], sm)


def test_every_short_sequence_over_three_symbols():
    """brute force on tiny inputs: all sequences of length <= 6 over 3 exponent values"""
    patterns = [0x3C00 | 0x15, 0x3C80 | 0x6A, 0xBD00 | 0x01]       # three exponents, mixed signs
    lengths = np.zeros(256, np.uint8)
    for n in range(1, 7):
        for seq in itertools.product(patterns, repeat=n):
            w = np.array(seq, np.uint16)
            e, _ = zo.split(w)
            lengths[:] = 0
            lengths[:] = zo.code_lengths(zo.histogram(e), 8)
            blob = zo.encode(w, 512, 512, lengths)
            assert np.array_equal(zo.decode(blob), w)


def expected_stream_words(e, lengths, R):
    """Words of one woven stream, from the schedule's invariant: every lane holds words q and q+1 of its
    own bitstream at the start of a round, so it takes 2 words at the start plus one for every word
    boundary its bit count has crossed by the end of the last-but-one round."""
    n = e.size
    tiles = -(-n // 512)
    pad = min((int(l), s) for s, l in enumerate(lengths) if l)[1]
    full = np.full(tiles * 512, pad, np.int64)
    full[:n] = e
    per_lane = full.reshape(tiles, 64, 8).transpose(1, 0, 2).reshape(64, tiles * 8)   # lane -> its symbols in order
    bits = lengths[per_lane].astype(np.int64)
    used_before_last_round = bits[:, : tiles * 8 - R].sum(axis=1)
    words = int((2 + used_before_last_round // 32).sum())
    return -(-words // 4) * 4, int(bits.sum())


@pytest.mark.parametrize("max_len", [8, 12])
def test_stream_sizes_match_closed_form(max_len):
    kind = "gauss" if max_len == 8 else "wide"
    w = synth.special_tensor(kind, 3 * 4096 + 2500, seed=9)
    C, W = 4096, 2048
    blob, lengths = roundtrip(w, C, W, max_len)
    h, table, stream_offs = chunk_table(blob)
    assert h["L"] == lengths.max() and h["R"] == (4 if h["L"] <= 8 else 2)
    e, _ = zo.split(w)
    total_code_bits = 0
    for c in range(h["n_chunks"]):
        at, mode = int(table[c]) & ~15, int(table[c]) & 15
        assert mode == zo.MODE_CODED
        cn = min(C, w.size - c * C)
        S = -(-cn // W)
        offs = stream_offs[c]
        assert offs[0] == 0 and offs[S] == (int(table[c + 1]) & ~15) - at and not offs[S + 1:].any()
        for s in range(S):
            es = e[c * C + s * W: c * C + min(cn, (s + 1) * W)]
            words, bits = expected_stream_words(es, lengths, h["R"])
            assert (offs[s + 1] - offs[s]) // 4 == words
            total_code_bits += bits
    # the payload can not be smaller than the code bits it carries
    assert (int(table[-1]) - h["e_offset"]) * 8 >= total_code_bits


def test_first_words_hold_each_lanes_first_codes():
    """the stream opens with words 0 and 1 of lane 0, lane 1, ...: decode the first symbol of every lane
    straight from those words with the canonical code, bit by bit"""
    w = synth.special_tensor("gauss", 4096, seed=1)
    blob, lengths = roundtrip(w, 4096, 4096)
    code, _ = zo.canonical(lengths)
    book = {(int(lengths[s]), int(code[s])): s for s in range(256) if lengths[s]}
    h, table, stream_offs = chunk_table(blob)
    at = int(table[0]) & ~15
    offs = stream_offs[0]
    words = blob[at + offs[0]: at + offs[1]].view("<u4")
    e, _ = zo.split(w)
    for lane in range(64):
        pair = int(words[2 * lane]) | (int(words[2 * lane + 1]) << 32)
        acc, l = 0, 0
        while (l, acc) not in book:
            acc = (acc << 1) | ((pair >> l) & 1)
            l += 1
        assert book[(l, acc)] == e[8 * lane]


def test_incompressible_chunks_are_stored_raw():
    w = synth.special_tensor("uniform_u16", 3 * 4096, seed=4)
    blob, _ = roundtrip(w, 4096, 1024)
    h, table, stream_offs = chunk_table(blob)
    assert all(int(t) & 15 == zo.MODE_RAW for t in table[:-1])
    assert int(table[-1]) - h["e_offset"] == w.size and not stream_offs.any()
    # a tensor whose first chunk is Gaussian and whose second is uniform noise mixes both modes
    mixed = np.concatenate([synth.special_tensor("gauss", 3 * 4096, 1), synth.special_tensor("uniform_u16", 4096, 2)])
    blob, _ = roundtrip(mixed, 4096, 4096, 12)     # 256 symbols present: only codes longer than 8 bits can compress
    _, table, _ = chunk_table(blob)
    assert [int(t) & 15 for t in table[:-1]] == [zo.MODE_CODED] * 3 + [zo.MODE_RAW]


def entropy_bits(e):
    h = np.bincount(e, minlength=256).astype(np.float64)
    p = h[h > 0] / h.sum()
    return float(-(p * np.log2(p)).sum())


def test_paper_entropy_bound_formula():
    """(8 + H) / 16 reproduces the two bound values of Sec. 2.2 that are printed consistently"""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "entropy_bound.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) == 2
    for H, pct in rows:
        assert round((8 + float(H)) / 16 * 100, 2) == float(pct)


@pytest.mark.parametrize("wl,C", [(synth.CFG1, 4096), (synth.CFG2, 16384)])
def test_compressed_size_against_entropy_bound(wl, C):
    """size / bf16 size is at least the Shannon bound (8+H)/16 of Sec. 2.2 and close to it; the paper's
    off-the-shelf backends reach 74 % (LZ4HC) and 68 % (ZSTD)"""
    w = synth.expert_matrix(wl, 0, 0, 0)
    W = 4096
    blob, lengths = roundtrip(w, C, W)
    e, _ = zo.split(w)
    H = entropy_bits(e)
    ratio = blob.size / (2 * w.size)
    bound = (8 + H) / 16
    assert ratio >= bound
    # code redundancy (< 0.12 bit) + per-stream lookahead words (64 lanes * about 48 bits per stream)
    slack = 0.12 / 16 + (64 * 64 / 8) / (2 * W) + 4096 / (2 * w.size)
    assert ratio < bound + slack, (ratio, bound, slack)
    assert ratio < 0.74


def test_partial_decode_touches_only_its_chunks():
    w = synth.special_tensor("gauss", 5 * 1024 + 100, seed=3)
    blob, _ = zo.encode_tensor(w, 1024, 512)
    out = np.full(w.size, 0xFFFF, np.uint16)
    zo.decode_chunks(blob, 2, 4, out)
    assert np.array_equal(out[2048:4096], w[2048:4096])
    assert np.all(out[:2048] == 0xFFFF) and np.all(out[4096:] == 0xFFFF)


def test_damaged_objects_are_rejected():
    w = synth.special_tensor("gauss", 8192, seed=6)
    blob, lengths = zo.encode_tensor(w, 4096, 2048)
    h, table, stream_offs = chunk_table(blob)
    for off in (0, 4, 16, 20, 24, 28, 32, 44, 56, 64, 72, 80, 88):
        bad = blob.copy()
        bad[off] ^= 0x5A
        with pytest.raises(zo.OracleError):
            zo.decode(bad)
    bad = blob.copy()                                   # codebook no longer satisfies Kraft
    bad[h["len_offset"] + int(np.argmax(lengths))] = 1
    with pytest.raises(zo.OracleError):
        zo.decode(bad)
    entry0 = h["table_offset"]
    for off in (entry0 + 8, entry0 + 12, entry0 + 16, entry0 + h["table_stride"] - 4, entry0 + h["table_stride"] + 8):
        bad = blob.copy()                               # stream offsets of a table entry damaged
        bad[off] ^= 0x10
        with pytest.raises(zo.OracleError):
            zo.decode(bad)
    bad = blob.copy()                                   # non-zero padding word after a stream
    at = int(table[0]) & ~15
    end0 = at + int(stream_offs[0][1])
    if not bad[end0 - 4: end0].any():
        bad[end0 - 1] = 0x80
        with pytest.raises(zo.OracleError):
            zo.decode(bad)
    with pytest.raises(zo.OracleError):
        zo.decode(blob[:-256])                          # truncated
    # encoding with a codebook that lacks a symbol that occurs is refused
    short = lengths.copy()
    short[int(np.argmax(lengths))] = 0
    with pytest.raises(zo.OracleError):
        zo.encode(w, 4096, 2048, short)
    with pytest.raises(zo.OracleError):
        zo.encode(w, 4096, 1000, lengths)               # stream length must be a multiple of 512
    with pytest.raises(zo.OracleError):
        zo.encode(w, 4096 + 512, 1024, lengths)         # chunk length must be a multiple of the stream length
