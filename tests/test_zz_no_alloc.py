"""zm_decode_host_tensors (the entry point that allocates nothing: compressed bytes are staged in the library's
fixed device array) against zm_cache_fetch on a cache without pool slots (the existing entry point that stages the
same bytes in a caller-provided arena), bit for bit, on two calls in a row, the second with a smaller input."""
import ctypes

import numpy as np
import pytest

from oracle import oracle as zo
from paper_2601_21198_amd import synth, zipmoe as zm

pytestmark = pytest.mark.gpu


def pinned_copy(blob):
    import torch
    t = torch.empty(blob.size, dtype=torch.uint8, pin_memory=True)
    t.numpy()[:] = blob
    return t


def staged_decode(blobs, stream):
    """every blob through zm_decode_host_tensors in one call; returns the uint16 outputs"""
    import torch
    n = len(blobs)
    pinned = [pinned_copy(b) for b in blobs]
    infos = (zm.TensorInfo * n)(*[zm.blob_info(b[:384]) for b in blobs])
    outs = [torch.full((int(i.n_values) + 16,), 0x5A5A, dtype=torch.int16, device="cuda") for i in infos]
    host = (ctypes.c_void_p * n)(*[p.data_ptr() for p in pinned])
    dev = (ctypes.c_void_p * n)(*[o.data_ptr() for o in outs])
    zm.decode_host_tensors(host, infos, n, dev, stream)
    torch.cuda.synchronize()
    res = []
    for o, i in zip(outs, infos):
        a = o.cpu().numpy().view(np.uint16)
        assert np.all(a[int(i.n_values):] == 0x5A5A)                       # nothing written past the tensor
        res.append(a[: int(i.n_values)].copy())
    return res


def cache_decode(expert_blobs, stream):
    """the same experts through zm_cache_fetch with no pool slots: every part is copied from the host into
    the cache's arena and decoded from there"""
    import torch
    cache = zm.ExpertCache(expert_blobs, (0, 0, 0, 0), 0, max_selected=len(expert_blobs), packed=False)
    ptrs, found = cache.fetch(list(range(len(expert_blobs))), stream)
    torch.cuda.synchronize()
    assert all(f == zm.POOL_NONE for f in found)
    res = []
    for e, tensors in enumerate(expert_blobs):
        for m, b in enumerate(tensors):
            n = int(zm.blob_info(b[:384]).n_values)
            off = ptrs[e][m] - cache.arena.data_ptr()
            assert 0 <= off and off + 2 * n <= cache.arena.numel()
            res.append(cache.arena[off: off + 2 * n].cpu().numpy().view(np.uint16).copy())
    cache.close()
    return res


def test_two_calls_in_a_row_match_the_cache_path_and_the_reference():
    import torch
    stream = torch.cuda.current_stream().cuda_stream
    wl = synth.CFG3
    # first call: two experts of configuration 3 (6 tensors, 12.6 M values, 17 MB of blobs)
    big = [[zm.compress(m, wl.chunk_values, 4096)[0] for m in synth.expert_tensors(wl, 0, e)] for e in (3, 11)]
    flat = [b for t in big for b in t]
    got = staged_decode(flat, stream)
    want = cache_decode(big, stream)
    for g, w, b in zip(got, want, flat):
        assert np.array_equal(g, w)
    originals = [m.reshape(-1) for e in (3, 11) for m in synth.expert_tensors(wl, 0, e)]
    for g, orig in zip(got, originals):
        assert np.array_equal(g, orig)
    assert np.array_equal(got[0], zo.decode(flat[0]))
    # second call, smaller, of other geometry (long codes, ragged tail, a raw chunk): the area still holds the
    # first call's bytes
    small_tensors = [synth.special_tensor("wide", 70001, seed=5), synth.special_tensor("uniform_u16", 5000, seed=6),
                     synth.special_tensor("gauss", 513, seed=7)]
    small = [zm.compress(w, 4096, 1024, 12 if i == 0 else 8)[0] for i, w in enumerate(small_tensors)]
    got = staged_decode(small, stream)
    want = cache_decode([small], stream)
    for g, w, b, orig in zip(got, want, small, small_tensors):
        assert np.array_equal(g, w) and np.array_equal(g, zo.decode(b)) and np.array_equal(g, orig)


def test_a_call_beyond_the_staging_area_is_refused():
    import torch
    w = synth.special_tensor("gauss", 9 << 20, seed=1)
    blob = zm.compress(w, 16384, 4096)[0]
    blobs = [blob] * 3                                   # 3 x 12.8 MB > 32 MiB
    assert sum(b.size for b in blobs) > zm.STAGING_BYTES
    with pytest.raises(zm.ZipMoEError) as err:
        staged_decode(blobs, torch.cuda.current_stream().cuda_stream)
    assert err.value.status == zm.E_SIZE
    assert np.array_equal(staged_decode(blobs[:2], torch.cuda.current_stream().cuda_stream)[1], w)
