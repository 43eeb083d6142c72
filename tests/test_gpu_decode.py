"""GPU parity: zm_decode_experts (through the C ABI) against the reference codec, bit for bit."""
import ctypes
import sys
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

from oracle import oracle as zo
from paper_2601_21198_amd import synth, zipmoe as zm

pytestmark = pytest.mark.gpu

GUARD = 64          # int16 guard words on each side of every output buffer
GUARD_WORD = 0x5A5A


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def gpu_decode_tensors(blobs, repeat_ids=None, stores=None):
    """Decodes each blob as a one-tensor expert; returns the decoded uint16 arrays (with guard check).
    stores: None = zm_decode_experts, else the policy handed to zm_decode_experts_stores."""
    import torch
    layer = zm.ExpertLayer([[b] for b in blobs])
    ids = list(range(len(blobs))) if repeat_ids is None else repeat_ids
    outs = []
    ptrs = (ctypes.c_void_p * len(ids))()
    for j, e in enumerate(ids):
        n = int(layer.infos[e].n_values)
        buf = torch.full((n + 2 * GUARD,), GUARD_WORD, dtype=torch.int16, device="cuda")
        outs.append(buf)
        ptrs[j] = buf.data_ptr() + 2 * GUARD
    idarr = (ctypes.c_int32 * len(ids))(*ids)
    outp = ctypes.cast(ptrs, ctypes.POINTER(ctypes.c_void_p))
    stream = torch.cuda.current_stream().cuda_stream
    if stores is None:
        zm.decode_experts(layer._ptr_blobs, layer._ptr_tables, layer._ptr_infos, layer.n_experts, 1, idarr, len(ids), outp, stream)
    else:
        rc = zm.lib().zm_decode_experts_stores(layer._ptr_blobs, layer._ptr_tables, layer._ptr_infos, layer.n_experts, 1,
                                               idarr, len(ids), outp, stores, ctypes.c_void_p(stream))
        if rc != zm.OK:
            raise zm.ZipMoEError(rc, "zm_decode_experts_stores")
    torch.cuda.synchronize()
    res = []
    for buf in outs:
        a = buf.cpu().numpy().view(np.uint16)
        assert np.all(a[:GUARD] == GUARD_WORD) and np.all(a[-GUARD:] == GUARD_WORD), "guard words overwritten"
        res.append(a[GUARD:-GUARD].copy())
    return res


KINDS = ["all_equal", "two_exponents", "uniform_u16", "rare_last", "gauss", "wide", "many_long"]
SIZES = [0, 1, 7, 8, 9, 511, 512, 513, 4095, 4096, 4097, 9000, 3 * 16384 + 1234]


@pytest.mark.parametrize("C,W,max_len", [(4096, 4096, 8), (16384, 4096, 8), (4096, 1024, 12), (2048, 512, 8),
                                         (16384, 16384, 8), (8192, 2048, 12), (32768, 8192, 12),
                                         # streams so long that fewer of them share a workgroup
                                         (16384, 16384, 12), (32768, 32768, 12), (32768, 32768, 8)])
def test_edge_cases_bit_exact(C, W, max_len):
    tensors, blobs = [], []
    for kind in KINDS:
        for n in SIZES:
            w = synth.special_tensor(kind, n, seed=n + 3)
            blob, _ = zm.compress(w, C, W, max_len)
            tensors.append(w)
            blobs.append(blob)
    say(f"edge cases C={C} W={W} L<={max_len}: {len(blobs)} tensors in one call")
    refs = [zo.decode(blob) for blob in blobs]
    for stores in (None, zm.STORES_CACHED, zm.STORES_STREAMING):      # the library's own choice, and both kernels by name
        got = gpu_decode_tensors(blobs, stores=stores)
        for w, ref, g in zip(tensors, refs, got):
            assert np.array_equal(g, ref)                    # against the reference decoder
            assert np.array_equal(g, w)                      # and against the original: lossless


def test_all_bit_patterns_and_duplicates():
    w = np.random.default_rng(1).permutation(np.arange(65536, dtype=np.uint32)).astype(np.uint16)
    blob8, _ = zm.compress(w, 4096, 4096, 8)
    blob12, _ = zm.compress(w, 4096, 2048, 12)
    got = gpu_decode_tensors([blob8, blob12], repeat_ids=[1, 0, 1, 1])      # duplicate ids are decoded again
    for g in got:
        assert np.array_equal(g, w)
    assert np.array_equal(got[0], zo.decode(blob12))


def test_mixed_geometries_in_one_call():
    # tensors with different chunk lengths, stream lengths and code-length limits share a call: both round
    # lengths are launched, and the staging area is sized for the longest stream of each group.  Every other
    # blob comes from the reference encoder.
    rng = np.random.default_rng(77)
    geometries = [(4096, 512, 8), (4096, 4096, 8), (16384, 4096, 8), (16384, 2048, 11), (8192, 8192, 9),
                  (2048, 1024, 12), (16384, 16384, 8), (1024, 512, 10)]
    tensors, blobs = [], []
    for i in range(48):
        C, W, max_len = geometries[int(rng.integers(len(geometries)))]
        kind = KINDS[int(rng.integers(len(KINDS)))]
        n = int(rng.integers(1, 70000))
        w = synth.special_tensor(kind, n, seed=1000 + i)
        if i % 2:
            blob = zo.encode(w, C, W, zo.code_lengths(zo.histogram(zo.split(w)[0]), max_len))
        else:
            blob, _ = zm.compress(w, C, W, max_len)
        tensors.append(w)
        blobs.append(blob)
    say(f"mixed geometries: {len(blobs)} tensors in one call")
    got = gpu_decode_tensors(blobs)
    for w, blob, g in zip(tensors, blobs, got):
        assert np.array_equal(g, w) and np.array_equal(g, zo.decode(blob))


def chunk_modes(blob):
    """mode of every chunk (0 coded, 1 raw), read from the blob's chunk table"""
    h = zo.header(blob)
    table = np.asarray(blob[h["table_offset"]: h["table_offset"] + h["table_stride"] * h["n_chunks"]], np.uint8)
    return table.reshape(h["n_chunks"], h["table_stride"])[:, 0] & 15


def patchwork_tensor(rng, n):
    """segments of very different exponent statistics in one tensor: with one codebook for the whole tensor some
    chunks compress and others are stored raw, and streams differ widely in length"""
    parts, left = [], n
    while left > 0:
        m = int(min(left, rng.integers(1, 40000)))
        k = int(rng.integers(5))
        if k == 0:
            seg = rng.integers(0, 65536, m, dtype=np.uint16)                                     # incompressible
        elif k == 1:
            seg = np.full(m, 0x3F80, np.uint16) | rng.integers(0, 128, m, dtype=np.uint16)      # one exponent
        elif k == 2:
            seg = synth.bf16_round(rng.standard_normal(m, dtype=np.float32) * np.float32(10.0 ** rng.uniform(-4, 2)))
        elif k == 3:
            e = rng.geometric(0.5, m).clip(1, 40).astype(np.uint16) + 90                         # geometric exponents
            seg = (e << 7) | rng.integers(0, 128, m, dtype=np.uint16) | (rng.integers(0, 2, m, dtype=np.uint16) << 15)
        else:
            e = rng.choice(np.array([1, 2, 127, 128, 254, 255], np.uint16), m, p=[0.5, 0.25, 0.12, 0.07, 0.04, 0.02])
            seg = (e << 7) | rng.integers(0, 128, m, dtype=np.uint16)
        parts.append(seg.astype(np.uint16))
        left -= m
    return np.concatenate(parts) if parts else np.zeros(0, np.uint16)


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_patchwork_tensors(seed):
    rng = np.random.default_rng(seed)
    geometries = [(4096, 512, 8), (4096, 4096, 8), (16384, 4096, 8), (16384, 4096, 12), (16384, 2048, 9), (8192, 8192, 8),
                  (2048, 1024, 12), (16384, 16384, 10), (1024, 512, 8), (32768, 4096, 8)]
    tensors, blobs, n_raw, n_coded = [], [], 0, 0
    for i in range(64):
        C, W, max_len = geometries[int(rng.integers(len(geometries)))]
        w = patchwork_tensor(rng, int(rng.integers(1, 150000)))
        n_present = np.unique(zo.split(w)[0]).size
        while (1 << max_len) < n_present:
            max_len += 1
        if i % 2:
            blob = zo.encode(w, C, W, zo.code_lengths(zo.histogram(zo.split(w)[0]), max_len))
        else:
            blob, _ = zm.compress(w, C, W, max_len)
        modes = chunk_modes(blob)
        n_raw += int((modes == 1).sum())
        n_coded += int((modes == 0).sum())
        tensors.append(w)
        blobs.append(blob)
    say(f"patchwork seed {seed}: {len(blobs)} tensors, {n_coded} coded and {n_raw} raw chunks")
    assert n_raw > 20 and n_coded > 20
    for stores in (None, zm.STORES_STREAMING):
        got = gpu_decode_tensors(blobs, stores=stores)
        for w, blob, g in zip(tensors, blobs, got):
            assert np.array_equal(g, w)
    for blob, w in list(zip(blobs, tensors))[::4]:
        assert np.array_equal(zo.decode(blob), w)


@pytest.mark.parametrize("kind,W,max_len", [("gauss", 4096, 8), ("wide", 4096, 12), ("wide", 16384, 12),
                                            ("wide", 32768, 12), ("gauss", 32768, 8)])
def test_outputs_larger_than_the_last_level_cache(kind, W, max_len):
    """a call that writes more than 256 MB takes the launch variant with non-temporal stores; every workgroup
    width is covered (streams of 16384 and 32768 values leave room for fewer streams per workgroup)"""
    import torch
    unit = synth.special_tensor(kind, (1 << 20) + 12345, seed=W + max_len)
    tensors = [np.tile(unit, 45)[: 45 * (1 << 20) + 777 * i] for i in range(3)]          # 3 x 47 M values: 283 MB of bf16
    say(f"{kind} W={W} L<={max_len}: compressing 3 x {tensors[0].size} values")
    with ThreadPoolExecutor(3) as ex:
        blobs = list(ex.map(lambda w: zm.compress(w, 32768, W, max_len)[0], tensors))
    assert sum(2 * w.size for w in tensors) > 256 << 20
    layer = zm.ExpertLayer([blobs], validate=False)
    for b in blobs:
        zm.validate_blob(b)
        assert (zm.blob_info(b[:384]).max_len > 8) == (kind == "wide")       # "wide" takes the long-code kernels
    bufs, starts, vals = layer.alloc_outputs(1)
    bufs[0].fill_(0x3333)
    layer.decode([0], bufs, starts, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got = bufs[0].cpu().numpy().view(np.uint16)
    say("decoding with the reference codec")
    for m, (w, blob) in enumerate(zip(tensors, blobs)):
        g = got[starts[m]: starts[m] + vals[m]]
        assert np.array_equal(g, w)
        h = zo.header(blob)
        ref = np.zeros(w.size, np.uint16)
        step = -(-h["n_chunks"] // 64)
        with ThreadPoolExecutor(16) as ex:
            list(ex.map(lambda c0: zo.decode_chunks(blob, c0, min(h["n_chunks"], c0 + step), ref), range(0, h["n_chunks"], step)))
        assert np.array_equal(g, ref)


def test_bad_arguments_are_refused_on_the_host():
    import torch
    w = synth.special_tensor("gauss", 5000, 0)
    blob, _ = zm.compress(w, 4096, 4096)
    layer = zm.ExpertLayer([[blob]])
    out = torch.empty(5008, dtype=torch.int16, device="cuda")
    ptrs = (ctypes.c_void_p * 1)(out.data_ptr())
    P = ctypes.POINTER(ctypes.c_void_p)
    call = lambda ids, outs=ptrs, n=1: zm.decode_experts(layer._ptr_blobs, layer._ptr_tables, layer._ptr_infos, 1, 1,
                                                         (ctypes.c_int32 * 1)(ids), n, ctypes.cast(outs, P), 0)
    call(0)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().view(np.uint16)[:5000], w)
    for bad_id in (-1, 1):
        with pytest.raises(zm.ZipMoEError):
            call(bad_id)
    with pytest.raises(zm.ZipMoEError):
        call(0, (ctypes.c_void_p * 1)(out.data_ptr() + 2))        # misaligned output
    with pytest.raises(zm.ZipMoEError):
        call(0, (ctypes.c_void_p * 1)(None))
    call(0, n=0)                                                   # nothing selected: no launch, no error


def oracle_decode_parallel(blobs, workers=16):
    with ThreadPoolExecutor(workers) as ex:
        return list(ex.map(zo.decode, blobs))


def compress_expert(wl, layer, expert, stream_values=4096):
    return [zm.compress(m, wl.chunk_values, stream_values)[0] for m in synth.expert_tensors(wl, layer, expert)]


def test_config1_single_matrix():
    w = synth.expert_matrix(synth.CFG1, 0, 0, 0)
    lengths = zo.code_lengths(zo.histogram(zo.split(w)[0]), 8)
    ref_blob = zo.encode(w, 4096, 4096, lengths)             # the reference encoder's own blob
    got = gpu_decode_tensors([ref_blob])[0]
    assert np.array_equal(got, zo.decode(ref_blob)) and np.array_equal(got, w.reshape(-1))


def test_config2_one_expert_with_outliers():
    import torch
    wl = synth.CFG2
    tensors = synth.expert_tensors(wl, 0, 0)
    blobs = compress_expert(wl, 0, 0)
    layer = zm.ExpertLayer([blobs])
    bufs, starts, vals = layer.alloc_outputs(1)
    layer.decode([0], bufs, starts, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got = bufs[0].cpu().numpy().view(np.uint16)
    ref = oracle_decode_parallel(blobs)
    for m in range(3):
        g = got[starts[m]: starts[m] + vals[m]]
        assert np.array_equal(g, ref[m]) and np.array_equal(g, tensors[m].reshape(-1))


def test_config3_layer_top8_zipf():
    import torch
    wl = synth.CFG3
    say("config 3: generating and compressing 64 experts")
    with ThreadPoolExecutor(16) as ex:
        all_blobs = list(ex.map(lambda e: compress_expert(wl, 0, e), range(wl.n_experts)))
    layer = zm.ExpertLayer(all_blobs, validate=False)
    bufs, starts, vals = layer.alloc_outputs(wl.top_k)
    stream = torch.cuda.current_stream().cuda_stream
    for call in range(6):
        ids = synth.route(wl, 0, call)
        assert len(set(ids.tolist())) == wl.top_k
        for b in bufs:
            b.fill_(0x1111)
        layer.decode(ids, bufs, starts, stream)
        torch.cuda.synchronize()
        say(f"config 3 call {call}: experts {ids.tolist()}")
        flat = [all_blobs[e][m] for e in ids for m in range(3)]
        ref = oracle_decode_parallel(flat) if call < 2 else None
        for j, e in enumerate(ids):
            got = bufs[j].cpu().numpy().view(np.uint16)
            orig = synth.expert_tensors(wl, 0, int(e))
            for m in range(3):
                g = got[starts[m]: starts[m] + vals[m]]
                assert np.array_equal(g, orig[m].reshape(-1))
                if ref is not None:
                    assert np.array_equal(g, ref[3 * j + m])


def test_decode_tensors_with_parts_in_separate_allocations():
    """zm_decode_tensors: decode table, chunk table, SM section and E-chunks each in an allocation of its own"""
    import torch
    tensors = [synth.special_tensor(k, n, seed=n) for k, n in (("gauss", 3 * 16384 + 700), ("wide", 20000),
                                                               ("uniform_u16", 9000), ("two_exponents", 4096))]
    blobs = [zm.compress(w, 16384, 4096, 12 if i == 1 else 8)[0] for i, w in enumerate(tensors)]
    n = len(blobs)
    parts, infos, outs = (zm.TensorParts * n)(), (zm.TensorInfo * n)(), (ctypes.c_void_p * n)()
    keep = []
    for i, b in enumerate(blobs):
        info = zm.blob_info(b)
        infos[i] = info
        cut = lambda lo, hi: torch.from_numpy(b[lo:hi].copy()).cuda()
        pieces = [cut(info.lut_offset, info.table_offset), cut(info.table_offset, info.table_offset + info.table_stride * (info.n_chunks + 1)),
                  cut(info.sm_offset, info.e_offset), cut(info.e_offset, info.blob_size)]
        out = torch.full((int(info.n_values) + 2 * GUARD,), GUARD_WORD, dtype=torch.int16, device="cuda")
        keep.append((pieces, out))
        parts[i] = zm.TensorParts(*[p.data_ptr() for p in pieces])
        outs[i] = out.data_ptr() + 2 * GUARD
    zm.decode_tensors(parts, infos, n, ctypes.cast(outs, ctypes.POINTER(ctypes.c_void_p)), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for (pieces, out), w, b in zip(keep, tensors, blobs):
        a = out.cpu().numpy().view(np.uint16)
        assert np.all(a[:GUARD] == GUARD_WORD) and np.all(a[-GUARD:] == GUARD_WORD)
        assert np.array_equal(a[GUARD:-GUARD], zo.decode(b)) and np.array_equal(a[GUARD:-GUARD], w)


def test_limits_of_one_call():
    """256 tensors in one call is the most a call takes (six launches); one more is refused; a stream too long to
    stage in LDS is refused on the host; the longest stream one wave can stage decodes correctly"""
    import torch
    small = [synth.special_tensor("gauss", 600 + i, seed=i) for i in range(256)]
    blobs = [zm.compress(w, 1024, 512)[0] for w in small]
    got = gpu_decode_tensors(blobs)
    for w, g in zip(small, got):
        assert np.array_equal(g, w)
    with pytest.raises(zm.ZipMoEError):
        gpu_decode_tensors(blobs + blobs[:1])
    # streams of 32768 values: only one fits the LDS of a workgroup
    w = synth.special_tensor("gauss", 2 * 32768 + 999, seed=3)
    blob, _ = zm.compress(w, 32768, 32768)
    assert np.array_equal(gpu_decode_tensors([blob])[0], w) and np.array_equal(zo.decode(blob), w)
    # streams of 131072 values can not be staged: refused, nothing launched
    big, _ = zm.compress(synth.special_tensor("gauss", 131072, seed=4), 131072, 131072)
    with pytest.raises(zm.ZipMoEError):
        gpu_decode_tensors([big])
    assert np.array_equal(zo.decode(big), synth.special_tensor("gauss", 131072, seed=4))
    torch.cuda.synchronize()


def test_layer_handle_decodes_like_the_array_call():
    """zm_layer_create / zm_layer_decode: the library's own handle for a layer's resident experts"""
    import torch
    rng = np.random.default_rng(5)
    n_experts, per = 5, 3
    tensors = [[synth.special_tensor(KINDS[int(rng.integers(len(KINDS)))], int(rng.integers(1, 90000)), seed=50 + 3 * e + m)
                for m in range(per)] for e in range(n_experts)]
    blobs = [[(zm.compress(w, 16384, 4096, 8)[0] if (e + m) % 2 else zo.encode_tensor(w, 16384, 4096, 8)[0])
              for m, w in enumerate(ts)] for e, ts in enumerate(tensors)]
    layer = zm.Layer(blobs)
    for e in range(n_experts):
        for m in range(per):
            a, b = layer.tensor_info(e, m), zm.blob_info(blobs[e][m][:384])
            assert bytes(a) == bytes(b)
    ids = [3, 0, 3, 4]                                           # a duplicate is decoded twice
    outs = [[torch.full((tensors[e][m].size + 2 * GUARD,), GUARD_WORD, dtype=torch.int16, device="cuda") for m in range(per)]
            for e in ids]
    ptrs = [o.data_ptr() + 2 * GUARD for row in outs for o in row]
    for stores in (zm.STORES_AUTO, zm.STORES_STREAMING):
        layer.decode(ids, ptrs, torch.cuda.current_stream().cuda_stream, stores)
        torch.cuda.synchronize()
        for j, e in enumerate(ids):
            for m in range(per):
                a = outs[j][m].cpu().numpy().view(np.uint16)
                assert np.all(a[:GUARD] == GUARD_WORD) and np.all(a[-GUARD:] == GUARD_WORD)
                assert np.array_equal(a[GUARD:-GUARD], tensors[e][m])
                assert np.array_equal(a[GUARD:-GUARD], zo.decode(blobs[e][m]))
                outs[j][m][GUARD:-GUARD].zero_()
    with pytest.raises(zm.ZipMoEError):
        layer.decode([n_experts], ptrs[:per])                    # id out of range
    layer.close()


def test_decode_call_can_be_captured_in_a_hip_graph():
    """the hot call allocates nothing and copies nothing, so it can be recorded into a graph; every replay,
    with eager work and synchronisations in between, must give the eager result"""
    import torch
    wl = synth.CFG2
    tensors = synth.expert_tensors(wl, 0, 0)
    blobs = compress_expert(wl, 0, 0)
    layer = zm.ExpertLayer([blobs, blobs])
    bufs, starts, vals = layer.alloc_outputs(2)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    call = layer.make_call([1, 0], bufs, starts)
    with torch.cuda.stream(side):
        call(side.cuda_stream)                                  # eager warm-up on the capture stream
    side.synchronize()
    eager = [b.clone() for b in bufs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call(torch.cuda.current_stream().cuda_stream)
    for replay in range(4):
        for b in bufs:
            b.fill_(0x2222 + replay)                            # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for b, e in zip(bufs, eager):
            assert torch.equal(b, e), replay
    got = bufs[0].cpu().numpy().view(np.uint16)
    for m in range(3):
        assert np.array_equal(got[starts[m]: starts[m] + vals[m]], tensors[m].reshape(-1))
