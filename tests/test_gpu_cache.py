"""GPU tests of the compression-aware expert cache: whatever state an expert is in, a fetch yields its
tensors bit for bit; the pool each expert ends up in follows the rules of Sec. 3.4."""
import numpy as np
import pytest

from oracle import oracle as zo
from paper_2601_21198_amd import synth, zipmoe as zm

pytestmark = pytest.mark.gpu
F, C, S, E, NONE = zm.POOL_FULL, zm.POOL_COMPRESSED, zm.POOL_SM, zm.POOL_E, zm.POOL_NONE


class PolicyModel:
    """The cache's bookkeeping rules restated in Python (no data): counts, rank thresholds, promotion
    only, eviction of the least activated member that the call does not use."""

    def __init__(self, n, slots, tolerance):
        self.n, self.slots, self.tol = n, list(slots), tolerance
        self.count = [0] * n
        self.pool = [NONE] * n
        self.members = [set() for _ in range(4)]
        self.limbo = [0] * 4

    def rank(self, e):
        return sum(1 for x in range(self.n) if self.count[x] > self.count[e] or (self.count[x] == self.count[e] and x < e))

    def target(self, e):
        cum, r = 0, self.rank(e)
        for p in range(4):
            cum += self.slots[p]
            if self.slots[p] > 0 and r < cum + self.tol:
                return p
        return NONE

    def fetch(self, ids):
        self.limbo = [0] * 4
        for e in ids:
            self.count[e] += 1
        found = []
        for e in ids:
            cur = self.pool[e]
            found.append(cur)
            t = min(self.target(e), cur)
            if t == cur:
                continue
            if len(self.members[t]) + self.limbo[t] < self.slots[t]:
                ok = True
            else:
                cand = [x for x in self.members[t] if x not in ids]
                ok = False
                if cand:
                    victim = min(cand, key=lambda x: (self.count[x], -x))
                    if self.count[victim] <= self.count[e]:
                        self.members[t].discard(victim)
                        self.pool[victim] = NONE
                        ok = True
            if ok:
                if cur != NONE:
                    self.members[cur].discard(e)
                    self.limbo[cur] += 1
                self.members[t].add(e)
                self.pool[e] = t
        return found


def make_layer(n_experts, shapes, seed):
    rng = np.random.default_rng(seed)
    tensors, blobs = [], []
    for e in range(n_experts):
        ts = [synth.bf16_round(rng.standard_normal(n, dtype=np.float32) * np.float32(0.01 + 0.01 * (e % 3))) for n in shapes]
        tensors.append(ts)
        blobs.append([zm.compress(t, 4096, 4096)[0] for t in ts])
    return tensors, blobs


def read_back(cache, ptr, n):
    off = ptr - cache.arena.data_ptr()
    assert 0 <= off and off + 2 * n <= cache.arena.numel()
    return cache.arena[off: off + 2 * n].cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("slots,tolerance", [((2, 3, 3, 3), 1), ((0, 0, 0, 0), 0), ((3, 0, 0, 0), 0), ((0, 4, 0, 0), 2),
                                             ((0, 0, 4, 0), 0), ((0, 0, 0, 4), 0), ((1, 1, 1, 1), 0), ((16, 0, 0, 0), 0)])
@pytest.mark.parametrize("packed", [True, False])
def test_fetch_is_bit_exact_in_every_state_and_follows_the_policy(slots, tolerance, packed):
    import torch
    n_experts, k = 16, 4
    shapes = (20000, 12345, 4096)
    tensors, blobs = make_layer(n_experts, shapes, seed=sum(slots) + tolerance)
    cache = zm.ExpertCache(blobs, slots, tolerance, max_selected=k, packed=packed)
    model = PolicyModel(n_experts, slots, tolerance)
    stream = torch.cuda.current_stream().cuda_stream
    rng = np.random.default_rng(7)
    p = np.arange(1, n_experts + 1, dtype=np.float64) ** -1.2
    p /= p.sum()
    seen = set()
    for step in range(150):
        ids = [int(x) for x in rng.choice(n_experts, k, replace=False, p=p)]
        ptrs, found = cache.fetch(ids, stream)
        torch.cuda.synchronize()
        assert found == model.fetch(ids), step
        seen.update(found)
        for j, e in enumerate(ids):
            for m, n in enumerate(shapes):
                assert ptrs[j][m] % 16 == 0
                assert np.array_equal(read_back(cache, ptrs[j][m], n), tensors[e][m]), (step, e, m, found[j])
        assert [cache.pool_of(e) for e in range(n_experts)] == model.pool, step
        for pool in range(4):
            assert sum(1 for e in range(n_experts) if cache.pool_of(e) == pool) <= slots[pool]
    if slots == (2, 3, 3, 3):
        assert seen == {F, C, S, E, NONE}            # every compression state was exercised
    # the reference decoder agrees with what the cache serves
    ptrs, _ = cache.fetch([0, 1], stream)
    torch.cuda.synchronize()
    for j in range(2):
        for m, n in enumerate(shapes):
            assert np.array_equal(read_back(cache, ptrs[j][m], n), zo.decode(blobs[j][m]))
    cache.close()


def test_fetch_refuses_bad_requests():
    tensors, blobs = make_layer(4, (5000,), seed=1)
    cache = zm.ExpertCache(blobs, (1, 1, 1, 1), 0, max_selected=2)
    for ids in ([0, 0], [4], [-1], [0, 1, 2]):
        with pytest.raises(zm.ZipMoEError):
            cache.fetch(ids)
    cache.close()


@pytest.mark.parametrize("packed", [True, False])
def test_back_to_back_fetches_without_host_synchronisation(packed):
    """fetches and their consumers are only ordered by the stream: each fetch's outputs are copied away by
    work queued on the same stream, the next fetch follows at once, everything is checked at the end"""
    import torch
    n_experts, k = 12, 3
    shapes = (30000, 8192)
    tensors, blobs = make_layer(n_experts, shapes, seed=11)
    cache = zm.ExpertCache(blobs, (2, 2, 2, 2), 1, max_selected=k, packed=packed)
    stream = torch.cuda.current_stream().cuda_stream
    rng = np.random.default_rng(3)
    steps = 60
    saved, wanted = [], []
    for step in range(steps):
        ids = [int(x) for x in rng.choice(n_experts, k, replace=False)]
        ptrs, _ = cache.fetch(ids, stream)
        for j, e in enumerate(ids):
            for m, n in enumerate(shapes):
                off = ptrs[j][m] - cache.arena.data_ptr()
                keep = torch.empty(2 * n, dtype=torch.uint8, device="cuda")
                keep.copy_(cache.arena[off: off + 2 * n], non_blocking=True)
                saved.append(keep)
                wanted.append(tensors[e][m])
    torch.cuda.synchronize()
    for got, want in zip(saved, wanted):
        assert np.array_equal(got.cpu().numpy().view(np.uint16), want)
    cache.close()
