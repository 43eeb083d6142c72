"""GPU parity of the stand-alone tensor recovery kernel (Sec. 3.3) and of the paper's split path:
exponents decompressed on host threads, merged on the GPU."""
import numpy as np
import pytest

from oracle import oracle as zo
from paper_2601_21198_amd import synth, zipmoe as zm

pytestmark = pytest.mark.gpu
GUARD = 64


def gpu_recover(e, sm):
    import torch
    n = e.size
    pad = -n % 8
    de = torch.from_numpy(np.concatenate([e, np.zeros(pad, np.uint8)])).cuda()
    ds = torch.from_numpy(np.concatenate([sm, np.zeros(pad, np.uint8)])).cuda()
    out = torch.full((n + 2 * GUARD,), 0x5A5A, dtype=torch.int16, device="cuda")
    zm.recover(de.data_ptr(), ds.data_ptr(), n, out.data_ptr() + 2 * GUARD, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    a = out.cpu().numpy().view(np.uint16)
    assert np.all(a[:GUARD] == 0x5A5A) and np.all(a[n + GUARD:] == 0x5A5A), "guard words overwritten"
    return a[GUARD: GUARD + n].copy()


@pytest.mark.parametrize("n", [0, 1, 7, 8, 9, 511, 512, 513, 4095, 4096, 16383, 16384, 16385, 1000003])
def test_recover_matches_reference_merge(n):
    rng = np.random.default_rng(n)
    e = rng.integers(0, 256, n, dtype=np.uint8)
    sm = rng.integers(0, 256, n, dtype=np.uint8)
    assert np.array_equal(gpu_recover(e, sm), zo.merge(e, sm))


def test_recover_launch_larger_than_half_the_last_level_cache():
    """a launch that moves more than 128 MB stores non-temporally: same words; the length is no multiple of a tile"""
    n = (40 << 20) + 1237
    rng = np.random.default_rng(77)
    e = rng.integers(0, 256, n, dtype=np.uint8)
    sm = rng.integers(0, 256, n, dtype=np.uint8)
    assert np.array_equal(gpu_recover(e, sm), zo.merge(e, sm))


def test_recover_all_pairs():
    e = np.repeat(np.arange(256, dtype=np.uint8), 256)
    sm = np.tile(np.arange(256, dtype=np.uint8), 256)
    got = gpu_recover(e, sm)
    assert np.array_equal(got, zo.merge(e, sm)) and np.unique(got).size == 65536


def test_recover_refuses_bad_pointers():
    import torch
    x = torch.zeros(64, dtype=torch.uint8, device="cuda")
    o = torch.zeros(64, dtype=torch.int16, device="cuda")
    with pytest.raises(zm.ZipMoEError):
        zm.recover(x.data_ptr() + 1, x.data_ptr(), 8, o.data_ptr())
    with pytest.raises(zm.ZipMoEError):
        zm.recover(x.data_ptr(), x.data_ptr(), 8, o.data_ptr() + 2)
    with pytest.raises(zm.ZipMoEError):
        zm.recover(0, x.data_ptr(), 8, o.data_ptr())


def test_paper_split_path_config2():
    """host threads decompress the E-chunks, the GPU merges: same tensor as the reference decoder"""
    wl = synth.CFG2
    for m, w in enumerate(synth.expert_tensors(wl, 0, 0)):
        blob, _ = zm.compress(w, wl.chunk_values, 4096)
        info = zm.blob_info(blob)
        e = zm.decode_exponents_host(blob, n_threads=8)
        sm = blob[info.sm_offset: info.sm_offset + w.size]
        got = gpu_recover(e, sm)
        assert np.array_equal(got, zo.decode(blob)) and np.array_equal(got, w.reshape(-1))
