"""The library's host side against the reference codec: same codebook cost, byte-identical blobs,
blobs the reference decoder accepts, loadable C ABI."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import oracle as zo
from paper_2601_21198_amd import synth, zipmoe as zm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "zipmoe.h")).read()
    declared = set(re.findall(r"\b(zm_[a-z_]+)\s*\(", text))
    assert declared == set(zm.EXPORTS)
    L = ctypes.CDLL(zm.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name
    assert zm.version() >= 20000
    assert zm.strerror(zm.E_FORMAT) and zm.strerror(12345)


def test_struct_layout_matches_header():
    assert ctypes.sizeof(zm.TensorInfo) == 80


@pytest.mark.parametrize("kind,max_len", [("gauss", 8), ("gauss", 12), ("wide", 8), ("wide", 12), ("rare_last", 8),
                                          ("two_exponents", 8), ("all_equal", 8), ("uniform_u16", 8)])
def test_codebook_cost_equals_reference(kind, max_len):
    w = synth.special_tensor(kind, 50000, seed=1)
    hist = zm.exponent_histogram(w)
    e, _ = zo.split(w)
    assert np.array_equal(hist, zo.histogram(e))
    mine, ref = zm.build_codebook(hist, max_len), zo.code_lengths(hist, max_len)
    assert mine.max() <= max_len and np.array_equal(mine > 0, hist > 0)
    assert int((hist * mine).sum()) == int((hist * ref).sum())
    assert zo.kraft_units(mine) == zo.kraft_units(ref)


def test_codebook_random_histograms():
    rng = np.random.default_rng(0)
    for trial in range(60):
        k = int(rng.integers(1, 80))
        hist = np.zeros(256, np.uint64)
        hist[rng.choice(256, k, replace=False)] = rng.integers(1, 10 ** int(rng.integers(1, 7)), k)
        for max_len in (8, 10, 12):
            if k > 2 ** max_len:
                continue
            mine, ref = zm.build_codebook(hist, max_len), zo.code_lengths(hist, max_len)
            assert int((hist * mine).sum()) == int((hist * ref).sum()), (trial, max_len)
    with pytest.raises(zm.ZipMoEError):
        zm.build_codebook(np.ones(256, np.uint64), 7)
    with pytest.raises(zm.ZipMoEError):
        zm.build_codebook(np.ones(256, np.uint64), 13)


@pytest.mark.parametrize("kind", ["all_equal", "two_exponents", "uniform_u16", "rare_last", "gauss", "wide"])
@pytest.mark.parametrize("n", [0, 1, 9, 511, 512, 513, 4096, 4097, 20000])
def test_blobs_identical_to_reference_and_decodable(kind, n):
    w = synth.special_tensor(kind, n, seed=n + 1)
    for C, W, max_len in ((4096, 4096, 8), (4096, 1024, 12), (2048, 512, 8)):
        lengths = zm.build_codebook(zm.exponent_histogram(w), max_len)
        blob, offs = zm.encode(w, C, W, lengths)
        ref = zo.encode(w, C, W, lengths)
        assert blob.size == ref.size and np.array_equal(blob, ref)
        assert np.array_equal(zo.decode(blob), w)
        zm.validate_blob(blob)
        info = zm.blob_info(blob)
        h = zo.header(blob)
        assert (info.n_values, info.chunk_values, info.stream_values, info.n_chunks, info.max_len,
                info.lane_quantum, info.n_present) == (n, C, W, h["n_chunks"], h["L"], h["quantum"], h["n_present"])
        assert (info.lut_offset, info.table_offset, info.sm_offset, info.e_offset, info.blob_size) == \
               (h["lut_offset"], h["table_offset"], h["sm_offset"], h["e_offset"], h["blob_size"])
        table = blob[h["table_offset"]: h["table_offset"] + h["table_stride"] * (h["n_chunks"] + 1)].view("<u8")
        assert info.table_stride == h["table_stride"] and np.array_equal(offs.reshape(-1), table)


def test_workload_tensors_match_reference():
    for wl, m in ((synth.CFG1, 0), (synth.CFG2, 2)):
        w = synth.expert_matrix(wl, 0, 0, m)
        blob, _ = zm.compress(w, wl.chunk_values, 4096, 8)
        lengths = blob[128:384]
        assert np.array_equal(blob, zo.encode(w, wl.chunk_values, 4096, lengths))
        assert np.array_equal(zo.decode(blob), w.reshape(-1))


def test_encode_rejects_bad_arguments():
    w = synth.special_tensor("gauss", 5000, 0)
    lengths = zm.build_codebook(zm.exponent_histogram(w), 8)
    for C, W in ((4096, 1000), (4096 + 512, 1024), (0, 512), (512, 0)):
        with pytest.raises(zm.ZipMoEError):
            zm.encode(w, C, W, lengths)
    short = lengths.copy()
    short[int(np.argmax(lengths))] = 0            # a symbol that occurs has no code (and Kraft is no longer 1)
    with pytest.raises(zm.ZipMoEError):
        zm.encode(w, 4096, 1024, short)
    over = lengths.copy()
    over[lengths > 0] = 1                          # violates Kraft
    with pytest.raises(zm.ZipMoEError):
        zm.encode(w, 4096, 1024, over)


def test_validate_rejects_damage():
    w = synth.special_tensor("gauss", 3 * 4096, 2)
    blob, offs = zm.compress(w, 4096, 2048)
    zm.validate_blob(blob)
    info = zm.blob_info(blob)
    for off in (0, 4, 8, 16, 20, 24, 28, 32, 36, 40, 44, 56, 64, 72, 80, 88, 100,
                128 + int(np.argmax(blob[128:384])), info.lut_offset + 3, info.table_offset, info.table_offset + 9,
                info.table_offset + 12, info.table_offset + info.table_stride + 16, info.table_offset + info.table_stride - 1):
        bad = blob.copy()
        bad[off] ^= 0x11
        with pytest.raises(zm.ZipMoEError):
            zm.validate_blob(bad)
    with pytest.raises(zm.ZipMoEError):
        zm.validate_blob(blob[:-256])


@pytest.mark.parametrize("kind,max_len", [("gauss", 8), ("wide", 12), ("uniform_u16", 8), ("rare_last", 8), ("all_equal", 8)])
def test_host_exponent_decoder_matches_reference_split(kind, max_len):
    """zm_decode_exponents_host (the paper's CPU-side decompression) returns the exponent bytes the
    reference codec's split gives for the original tensor"""
    for n in (1, 513, 4096, 3 * 4096 + 77):
        w = synth.special_tensor(kind, n, seed=n)
        blob, _ = zm.compress(w, 4096, 1024, max_len)
        ref_e, ref_sm = zo.split(w)
        for threads in (1, 3):
            assert np.array_equal(zm.decode_exponents_host(blob, n_threads=threads), ref_e)
        # the decoded exponents and the blob's SM section give back the tensor through the reference merge
        info = zm.blob_info(blob)
        sm = blob[info.sm_offset: info.sm_offset + n]
        assert np.array_equal(sm, ref_sm)
        assert np.array_equal(zo.merge(zm.decode_exponents_host(blob), sm), w)


def test_host_exponent_decoder_chunk_ranges_and_errors():
    w = synth.special_tensor("gauss", 5 * 2048 + 300, seed=8)
    blob, _ = zm.compress(w, 2048, 512)
    ref_e, _ = zo.split(w)
    out = np.full(w.size, 0xEE, np.uint8)
    zm.decode_exponents_host(blob, 2, 4, n_threads=2, out=out)
    assert np.array_equal(out[4096:8192], ref_e[4096:8192])
    assert np.all(out[:4096] == 0xEE) and np.all(out[8192:] == 0xEE)
    zm.decode_exponents_host(blob, 5, 6, out=out)                      # the short last chunk
    assert np.array_equal(out[10240:], ref_e[10240:])
    with pytest.raises(zm.ZipMoEError):
        zm.decode_exponents_host(blob, 3, 7)
    with pytest.raises(zm.ZipMoEError):
        zm.decode_exponents_host(blob, 4, 3)
    bad = blob.copy()
    bad[0] ^= 1
    with pytest.raises(zm.ZipMoEError):
        zm.decode_exponents_host(bad)
    with pytest.raises(zm.ZipMoEError):
        zm.decode_exponents_host(blob[:-256])


def test_host_exponent_decoder_on_workload_tensor():
    w = synth.expert_matrix(synth.CFG2, 0, 0, 1)
    blob, _ = zm.compress(w, 16384, 4096)
    assert np.array_equal(zm.decode_exponents_host(blob, n_threads=4), zo.split(w)[0])


def test_decode_entry_points_refuse_bad_arguments_before_any_launch():
    """argument checks of the device entry points are host logic: they return before touching the GPU"""
    w = synth.special_tensor("gauss", 5000, 0)
    blob, _ = zm.compress(w, 4096, 4096)
    info = zm.blob_info(blob)
    infos = (zm.TensorInfo * 1)(info)
    P = ctypes.POINTER(ctypes.c_void_p)
    good = 0x10000                                             # an aligned, non-null address; never dereferenced
    outs = (ctypes.c_void_p * 1)(good)
    L = zm.lib()
    parts = (zm.TensorParts * 1)(zm.TensorParts(good, good, good, good))
    assert L.zm_decode_tensors(parts, infos, 0, outs, None) == zm.OK           # nothing to do
    assert L.zm_decode_tensors(None, infos, 1, outs, None) == zm.E_ARG
    assert L.zm_decode_tensors(parts, infos, 257, outs, None) == zm.E_ARG
    for bad in (zm.TensorParts(good + 4, good, good, good), zm.TensorParts(good, good + 1, good, good),
                zm.TensorParts(good, good, good + 8, good), zm.TensorParts(good, good, good, None)):
        assert L.zm_decode_tensors((zm.TensorParts * 1)(bad), infos, 1, outs, None) == zm.E_ARG
    assert L.zm_decode_tensors(parts, infos, 1, (ctypes.c_void_p * 1)(good + 2), None) == zm.E_ARG
    broken = zm.TensorInfo.from_buffer_copy(info)
    broken.stream_values = 1000
    assert L.zm_decode_tensors(parts, (zm.TensorInfo * 1)(broken), 1, outs, None) == zm.E_ARG
    broken = zm.TensorInfo.from_buffer_copy(info)
    broken.table_stride = 8
    assert L.zm_decode_tensors(parts, (zm.TensorInfo * 1)(broken), 1, outs, None) == zm.E_ARG
    blobs = (ctypes.c_void_p * 1)(good)
    ids = (ctypes.c_int32 * 1)(0)
    assert L.zm_decode_experts(blobs, blobs, infos, 1, 1, ids, 0, outs, None) == zm.OK
    assert L.zm_decode_experts(blobs, blobs, infos, 1, 1, (ctypes.c_int32 * 1)(1), 1, outs, None) == zm.E_ARG
    assert L.zm_decode_experts(blobs, blobs, infos, 0, 1, ids, 1, outs, None) == zm.E_ARG
    assert L.zm_decode_experts((ctypes.c_void_p * 1)(good + 8), blobs, infos, 1, 1, ids, 1, outs, None) == zm.E_ARG
    assert L.zm_recover(None, ctypes.c_void_p(good), 8, ctypes.c_void_p(good), None) == zm.E_ARG
    assert L.zm_recover(ctypes.c_void_p(good), ctypes.c_void_p(good), 0, ctypes.c_void_p(good), None) == zm.OK
    # the store policy of zm_decode_experts_stores is one of three values
    assert L.zm_decode_experts_stores(blobs, blobs, infos, 1, 1, ids, 1, outs, 3, None) == zm.E_ARG
    assert L.zm_decode_experts_stores(blobs, blobs, infos, 1, 1, ids, 1, outs, -1, None) == zm.E_ARG
    assert L.zm_decode_experts_stores(blobs, blobs, infos, 1, 1, ids, 0, outs, zm.STORES_STREAMING, None) == zm.OK
    # the lane quantum in the info must be the one the geometry defines
    broken = zm.TensorInfo.from_buffer_copy(info)
    broken.lane_quantum += 1
    assert L.zm_decode_tensors(parts, (zm.TensorInfo * 1)(broken), 1, outs, None) == zm.E_ARG
    # the staged and the probe entry points check their arguments on the host as well
    host = (ctypes.c_void_p * 1)(blob.ctypes.data)
    assert L.zm_decode_host_tensors(host, infos, 0, outs, None) == zm.OK
    assert L.zm_decode_host_tensors(None, infos, 1, outs, None) == zm.E_ARG
    assert L.zm_decode_host_tensors(host, infos, 257, outs, None) == zm.E_ARG
    huge = zm.TensorInfo.from_buffer_copy(info)
    huge.blob_size = (zm.STAGING_BYTES + 256)
    assert L.zm_decode_host_tensors(host, (zm.TensorInfo * 1)(huge), 1, outs, None) == zm.E_SIZE
    assert L.zm_mover_probe(None, ctypes.c_void_p(good), 16, 16, 1, 0, None) == zm.E_ARG
    assert L.zm_mover_probe(ctypes.c_void_p(good), ctypes.c_void_p(good), 24, 16, 1, 0, None) == zm.E_ARG
    assert L.zm_mover_probe(ctypes.c_void_p(good), ctypes.c_void_p(good), 16, 16, 3, 0, None) == zm.E_ARG


def test_layer_handle_checks_everything_before_it_touches_the_device():
    """zm_layer_create validates sizes, alignment and every blob on the host first: all of these fail (or succeed
    trivially) without a device"""
    L = zm.lib()
    w = synth.special_tensor("gauss", 20000, 1)
    blob, _ = zm.compress(w, 4096, 4096, 8)
    sizes = (ctypes.c_size_t * 2)(int(blob.size), int(blob.size))
    need = ctypes.c_size_t(0)
    assert L.zm_layer_arena_bytes(sizes, 2, ctypes.byref(need)) == zm.OK and need.value == 2 * int(blob.size)
    odd = (ctypes.c_size_t * 2)(1000, 257)
    assert L.zm_layer_arena_bytes(odd, 2, ctypes.byref(need)) == zm.OK and need.value == 1024 + 512
    assert L.zm_layer_arena_bytes(None, 2, ctypes.byref(need)) == zm.E_ARG
    assert L.zm_layer_arena_bytes(sizes, 0, ctypes.byref(need)) == zm.E_ARG
    ptrs = (ctypes.c_void_p * 2)(blob.ctypes.data, blob.ctypes.data)
    handle = ctypes.c_void_p(None)
    arena = ctypes.c_void_p(1 << 20)                 # an aligned address that is never dereferenced by these calls
    big = 1 << 30
    assert L.zm_layer_create(None, sizes, 2, 1, arena, big, ctypes.byref(handle)) == zm.E_ARG
    assert L.zm_layer_create(ptrs, sizes, 0, 1, arena, big, ctypes.byref(handle)) == zm.E_ARG
    assert L.zm_layer_create(ptrs, sizes, 2, 1, None, big, ctypes.byref(handle)) == zm.E_ARG
    assert L.zm_layer_create(ptrs, sizes, 2, 1, ctypes.c_void_p((1 << 20) + 16), big, ctypes.byref(handle)) == zm.E_ARG
    assert L.zm_layer_create(ptrs, sizes, 2, 1, arena, 2 * int(blob.size) - 1, ctypes.byref(handle)) == zm.E_SIZE
    damaged = blob.copy()
    damaged[130] ^= 0x3F                             # a code length: the codebook no longer matches the table
    bad = (ctypes.c_void_p * 2)(blob.ctypes.data, damaged.ctypes.data)
    assert L.zm_layer_create(bad, sizes, 2, 1, arena, big, ctypes.byref(handle)) == zm.E_FORMAT
    short = (ctypes.c_size_t * 2)(int(blob.size), int(blob.size) - 256)
    assert L.zm_layer_create(ptrs, short, 2, 1, arena, big, ctypes.byref(handle)) == zm.E_FORMAT
    assert handle.value is None
    info = zm.TensorInfo()
    assert L.zm_layer_tensor_info(None, 0, 0, ctypes.byref(info), None) == zm.E_ARG
    assert L.zm_layer_decode(None, None, 0, None, 0, None) == zm.E_ARG
    L.zm_layer_destroy(None)


def test_launch_shapes_follow_code_length_stream_length_and_output_size():
    """zm_decode_launch_shapes is host logic: the same rule the decode calls launch by"""
    def info_of(kind, n, C, W, max_len):
        return zm.blob_info(zm.compress(synth.special_tensor(kind, n, 3), C, W, max_len)[0][:384])

    short, long_ = info_of("gauss", 50000, 16384, 4096, 8), info_of("wide", 50000, 16384, 4096, 12)
    assert short.max_len <= 8 < long_.max_len
    shapes = zm.decode_launch_shapes([short, long_, short])
    assert [(s.round_symbols, s.waves_per_workgroup, s.streaming_stores, s.tensors) for s in shapes] == [(4, 2, 0, 2), (2, 2, 0, 1)]
    assert shapes[0].workgroups == -(-(-(-50000 // 4096)) // 2) and shapes[0].lds_bytes < 10 * 1024
    assert all(s.streaming_stores == 1 for s in zm.decode_launch_shapes([short, long_], zm.STORES_STREAMING))
    # more than 48 tensors of a kind are split over launches
    assert [s.tensors for s in zm.decode_launch_shapes([short] * 100)] == [48, 48, 4]
    # streams too long for two of them to share a workgroup's LDS get a workgroup each
    wide_stream = info_of("gauss", 70000, 32768, 32768, 8)
    assert [(s.round_symbols, s.waves_per_workgroup) for s in zm.decode_launch_shapes([wide_stream])] == [(4, 1)]
    # a call that writes more than 256 MB streams its stores when the policy is left to the library
    big = zm.TensorInfo.from_buffer_copy(short)
    big.n_values = 140 << 20
    big.e_offset = big.sm_offset + (big.n_values + 255) // 256 * 256
    big.blob_size = big.e_offset + 256
    big.n_chunks = -(-big.n_values // big.chunk_values)
    assert [s.streaming_stores for s in zm.decode_launch_shapes([big])] == [1]
    assert [s.streaming_stores for s in zm.decode_launch_shapes([big], zm.STORES_CACHED)] == [0]


def test_cache_configuration_is_checked_on_the_host():
    w = synth.special_tensor("gauss", 5000, 0)
    blob, _ = zm.compress(w, 4096, 4096)
    infos = (zm.TensorInfo * 2)(zm.blob_info(blob), zm.blob_info(blob))
    need = ctypes.c_size_t(0)
    ok = zm.CacheConfig(2, 1, (ctypes.c_int32 * 4)(1, 1, 0, 0), 0, 2)
    assert zm.lib().zm_cache_arena_bytes(ctypes.byref(ok), infos, ctypes.byref(need)) == zm.OK
    info = infos[0]
    sm, e, full = -(-(info.e_offset - info.sm_offset) // 256) * 256, -(-(info.blob_size - info.e_offset) // 256) * 256, -(-2 * 5000 // 256) * 256
    assert need.value >= full + (sm + e) + 2 * (sm + e + full)             # pools F and C plus two transient buffers
    for bad in (zm.CacheConfig(0, 1, (ctypes.c_int32 * 4)(1, 1, 0, 0), 0, 2), zm.CacheConfig(2, 1, (ctypes.c_int32 * 4)(-1, 1, 0, 0), 0, 2),
                zm.CacheConfig(2, 1, (ctypes.c_int32 * 4)(1, 1, 0, 0), -1, 2), zm.CacheConfig(2, 1, (ctypes.c_int32 * 4)(1, 1, 0, 0), 0, 300)):
        assert zm.lib().zm_cache_arena_bytes(ctypes.byref(bad), infos, ctypes.byref(need)) == zm.E_ARG


def test_serialised_format_is_stable():
    """the stored digests were written by the reference codec alone (tests/golden/make_format_digests.py);
    the reference codec of today and the library must both still produce those bytes"""
    import hashlib
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "format_digests.txt")) if not l.startswith("#")]
    assert len(rows) == 6
    for kind, n, C, W, max_len, version, size, digest in rows:
        w = synth.special_tensor(kind, int(n), seed=1)
        ref, lengths = zo.encode_tensor(w, int(C), int(W), int(max_len))
        assert zo.header(ref)["version"] == int(version) and ref.size == int(size)
        assert hashlib.sha256(ref.tobytes()).hexdigest() == digest
        mine, _ = zm.encode(w, int(C), int(W), lengths)
        assert hashlib.sha256(mine.tobytes()).hexdigest() == digest


def test_missing_library_is_an_error_not_a_fallback():
    # the product path has no CPU fallback: without the built library every call fails at load time
    import subprocess
    import sys
    env = dict(os.environ, ZIPMOE_LIBRARY="/nonexistent/libzipmoe.so")
    code = ("import numpy as np\n"
            "from paper_2601_21198_amd import zipmoe as zm\n"
            "zm.compress(np.zeros(4096, np.uint16), 4096)\n")
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode != 0 and "is not built" in r.stderr


def test_product_sources_do_not_touch_the_reference_codec():
    # the reference implementations are test infrastructure: nothing in the package imports, opens or links them
    pkg = os.path.join(ROOT, "paper_2601_21198_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"\boracle\b|zm_oracle|libzm_oracle", text), os.path.join(dirpath, f)
    text = open(os.path.join(ROOT, "include", "zipmoe.h")).read()
    assert not re.search(r"zm_oracle|libzm_oracle", text)


def test_host_decoder_does_not_trust_the_blobs_decode_table():
    # the table copy inside the blob serves the GPU; the host decoder rebuilds its own from the code lengths,
    # so a damaged copy (which zm_validate_blob reports) cannot send it astray
    w = synth.special_tensor("gauss", 20000, 5)
    blob, _ = zm.compress(w, 4096, 1024, 8)
    info = zm.blob_info(blob[:384])
    bad = blob.copy()
    bad[info.lut_offset: info.lut_offset + 512] = 0xFF          # lengths of 255 bits everywhere
    with pytest.raises(zm.ZipMoEError):
        zm.validate_blob(bad)
    assert np.array_equal(zm.decode_exponents_host(bad, n_threads=3), zo.split(w)[0])
    unaligned = np.zeros(blob.size + 1, np.uint8)[1:]            # a host copy at an odd address
    unaligned[:] = blob
    assert np.array_equal(zm.decode_exponents_host(unaligned, n_threads=2), zo.split(w)[0])


def test_packed_expert_image_layout():
    # zm_cache_pack_expert: the SM sections of an expert's tensors, then their E-chunk regions, each at the
    # offset the largest expert's tensor of that index needs (256-byte aligned), zeros in between
    rng = np.random.default_rng(5)
    sizes = [(9000, 4096), (5000, 12000)]                 # two experts, two tensors each, different sizes
    blobs, infos_list = [], []
    for e, ns in enumerate(sizes):
        for n in ns:
            w = synth.bf16_round(rng.standard_normal(n, dtype=np.float32) * np.float32(0.02))
            b, _ = zm.compress(w, 4096, 1024)
            blobs.append(b)
            infos_list.append(zm.blob_info(b[:384]))
    infos = (zm.TensorInfo * 4)(*infos_list)
    cfg = zm.CacheConfig(2, 2, (ctypes.c_int32 * 4)(1, 1, 1, 1), 0, 2)
    ptrs = (ctypes.c_void_p * 4)(*[b.ctypes.data for b in blobs])
    size = ctypes.c_size_t(0)
    assert zm.lib().zm_cache_image_bytes(ctypes.byref(cfg), infos, ctypes.byref(size)) == zm.OK
    up = lambda x: (x + 255) // 256 * 256
    sm_cap = [max(up(int(infos_list[e * 2 + m].e_offset - infos_list[e * 2 + m].sm_offset)) for e in range(2)) for m in range(2)]
    e_cap = [max(up(int(infos_list[e * 2 + m].blob_size - infos_list[e * 2 + m].e_offset)) for e in range(2)) for m in range(2)]
    assert size.value == sum(sm_cap) + sum(e_cap)
    for e in range(2):
        img = np.full(size.value, 0xEE, np.uint8)
        assert zm.lib().zm_cache_pack_expert(ctypes.byref(cfg), infos, ptrs, e, ctypes.c_void_p(img.ctypes.data), size.value) == zm.OK
        want = np.zeros(size.value, np.uint8)
        at = 0
        for m in range(2):
            i, b = infos_list[e * 2 + m], blobs[e * 2 + m]
            want[at: at + int(i.e_offset - i.sm_offset)] = b[i.sm_offset: i.e_offset]
            at += sm_cap[m]
        for m in range(2):
            i, b = infos_list[e * 2 + m], blobs[e * 2 + m]
            want[at: at + int(i.blob_size - i.e_offset)] = b[i.e_offset: i.blob_size]
            at += e_cap[m]
        assert np.array_equal(img, want)
    small = np.zeros(size.value - 1, np.uint8)
    assert zm.lib().zm_cache_pack_expert(ctypes.byref(cfg), infos, ptrs, 0, ctypes.c_void_p(small.ctypes.data), small.size) == zm.E_SIZE
    assert zm.lib().zm_cache_pack_expert(ctypes.byref(cfg), infos, ptrs, 2, ctypes.c_void_p(small.ctypes.data), small.size) == zm.E_ARG


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=ROOT)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""
