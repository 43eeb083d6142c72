"""The measurement aid zm_mover_probe moves what it says and stays inside its buffers: vector i of the output is
vector i of the input where the input reaches, the fill pattern (1, 2, 3, 4) beyond."""
import numpy as np
import pytest

from paper_2601_21198_amd import zipmoe as zm

pytestmark = pytest.mark.gpu
GUARD = 256        # bytes on each side of the output


@pytest.mark.parametrize("pieces", [1, 8])
@pytest.mark.parametrize("streaming", [False, True])
@pytest.mark.parametrize("read_vectors,write_vectors", [(1, 1), (255, 257), (2048, 2048), (5000, 3000), (3000, 5000),
                                                        (70001, 99991)])
def test_mover_probe_copies_and_fills(pieces, streaming, read_vectors, write_vectors):
    import torch
    rng = np.random.default_rng(read_vectors + write_vectors)
    src = rng.integers(0, 2**32, (read_vectors, 4), dtype=np.uint32)
    dsrc = torch.from_numpy(src.view(np.int32)).cuda()
    out = torch.full((GUARD + 16 * write_vectors + GUARD,), 0x5A, dtype=torch.uint8, device="cuda")
    assert (out.data_ptr() + GUARD) % 16 == 0
    zm.mover_probe(dsrc.data_ptr(), out.data_ptr() + GUARD, 16 * read_vectors, 16 * write_vectors, pieces, streaming,
                   torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    a = out.cpu().numpy()
    assert np.all(a[:GUARD] == 0x5A) and np.all(a[-GUARD:] == 0x5A), "guard bytes overwritten"
    got = a[GUARD:-GUARD].view(np.uint32).reshape(write_vectors, 4)
    n = min(read_vectors, write_vectors)
    assert np.array_equal(got[:n], src[:n])
    assert np.all(got[n:] == np.array([1, 2, 3, 4], np.uint32))
