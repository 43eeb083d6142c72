"""The library's scheduler (zm_sched_build, zm_sched_simulate, zm_sched_lower_bounds) against the reference
scheduler in oracle/: same blocks, same timeline, event by event.  Host only."""
import random

import numpy as np
import pytest

from oracle import scheduler as ref
from paper_2601_21198_amd import zipmoe as zm

STATES = ((1, 1, 1), (1, 0, 1), (0, 1, 1), (0, 0, 1), (0, 0, 0))       # (needs_sm, needs_e, needs_decode)


def both(tasks, p, u, v, c, r, L, K):
    """The same request set in the two vocabularies."""
    lib_tasks = [zm.SchedTask(e, sm, en, dec) for (e, sm, en, dec) in tasks]
    ref_tasks = [ref.Task(e, bool(sm), bool(en), bool(dec)) for (e, sm, en, dec) in tasks]
    return lib_tasks, zm.SchedCosts(u, v, c, r, L, K), ref_tasks, ref.Costs(u, v, c, r, L, K)


def random_request(rng, dyadic, big=False):
    K = rng.choice([1, 2, 3, 4, 8] + ([16, 32] if big else []))
    L = rng.choice([1, 2, 3, 4, 8])
    n_exp = rng.randint(1, 8 if big else 4)
    n_tensors = rng.choice([1, 2, 3])
    tasks = []
    for e in range(n_exp):
        st = rng.choice(STATES)
        tasks += [(e, *st)] * n_tensors
    rng.shuffle(tasks)
    if dyadic:
        draw = lambda: rng.choice([0.125, 0.25, 0.5, 0.75, 1.0, 1.5, 2.0, 3.0])
    else:
        draw = lambda: rng.uniform(0.05, 3.0)
    p = [draw() for _ in range(n_exp)]
    if rng.random() < 0.3 and n_exp > 1:
        p[1] = p[0]                                       # ties in the token counts
    return tasks, p, draw(), draw() / K, draw(), rng.choice([0.0, draw() / 4]), L, K


def compare(tasks, p, u, v, c, r, L, K, exact):
    lt, lc, rt, rc = both(tasks, p, u, v, c, r, L, K)
    want_blocks = ref.build_blocks(rt, p, rc)
    got_blocks = zm.sched_build(lt, p, lc)
    assert got_blocks == want_blocks
    want = ref.simulate(rt, p, rc, want_blocks)
    res, worker_end, events = zm.sched_simulate(lt, p, lc, got_blocks)
    close = (lambda a, b: a == b) if exact else (lambda a, b: a == pytest.approx(b, rel=1e-12, abs=1e-12))
    assert close(res.makespan, want.makespan) and close(res.io_end, want.io_end) and close(res.charge, want.charge)
    assert len(worker_end) == L and all(close(a, b) for a, b in zip(worker_end, want.worker_end))
    assert len(events) == len(want.events)
    for g, w in zip(events, want.events):                 # placed in the same order, too
        assert (g.kind, g.task, g.chunk, g.unit) == (w.kind, w.task, w.chunk, w.unit)
        assert close(g.start, w.start) and close(g.end, w.end)
    lb = zm.sched_lower_bounds(lt, p, lc)
    wb = ref.lower_bounds(rt, p, rc)
    assert all(close(a, b) for a, b in zip(lb, [wb["I"], wb["C/L"], wb["P"], wb["Z"]]))
    assert all(res.makespan >= x - 1e-9 for x in lb)
    return res


def test_exports_and_struct_sizes():
    import ctypes
    assert ctypes.sizeof(zm.SchedTask) == 16 and ctypes.sizeof(zm.SchedCosts) == 40
    assert ctypes.sizeof(zm.SchedEvent) == 32 and ctypes.sizeof(zm.SchedResult) == 24
    for name in ("zm_sched_build", "zm_sched_simulate", "zm_sched_lower_bounds"):
        assert hasattr(zm.lib(), name)


def test_hand_worked_request_through_the_library():
    # Sec. 3.3: one missing expert (5 time units of tokens) and one compressed expert (2), L = 1, K = 2, u = 4,
    # E-chunk read 1, decompression 1: the compressed expert's chunks fill the wait for the first E-chunk, the
    # missing expert runs right after its SM-chunk has arrived at 6 and ends at 11 (the timeline is worked out
    # in the oracle's tests).
    tasks = [(0, 1, 1, 1), (1, 0, 0, 1)]
    res = compare(tasks, [5.0, 2.0], 4.0, 1.0, 1.0, 0.0, 1, 2, exact=True)
    assert res.makespan == 11.0 and res.charge == 0.0 and res.io_end == 6.0


@pytest.mark.parametrize("seed", range(6))
def test_random_requests_with_exact_arithmetic(seed):
    rng = random.Random(1000 + seed)
    for _ in range(40):
        compare(*random_request(rng, dyadic=True), exact=True)


@pytest.mark.parametrize("seed", range(3))
def test_random_requests_with_real_delays(seed):
    rng = random.Random(2000 + seed)
    for _ in range(30):
        compare(*random_request(rng, dyadic=False), exact=False)


def test_larger_requests():
    rng = random.Random(3)
    for _ in range(6):
        compare(*random_request(rng, dyadic=True, big=True), exact=True)


def test_a_layer_sized_request_runs_fast():
    # 8 experts x 3 tensors x 128 E-chunks, 16 threads: the builder simulates a few hundred candidate lists
    import time
    rng = random.Random(5)
    tasks = []
    for e in range(8):
        tasks += [(e, *rng.choice(STATES[:4]))] * 3
    p = [rng.choice([1.0, 2.0, 3.0, 4.0]) * 1e-5 for _ in range(8)]
    lt = [zm.SchedTask(*t) for t in tasks]
    costs = zm.SchedCosts(60e-6, 0.25e-6, 1e-6, 2e-6, 16, 128)
    t0 = time.perf_counter()
    blocks = zm.sched_build(lt, p, costs)
    res, worker_end, _ = zm.sched_simulate(lt, p, costs, blocks, events=False)
    took = time.perf_counter() - t0
    assert sorted(j for b in blocks for j in b) == list(range(24))
    assert all(res.makespan >= x - 1e-12 for x in zm.sched_lower_bounds(lt, p, costs))
    assert took < 2.0


def test_simulate_takes_any_priority_list_and_subsets():
    tasks = [(0, 1, 1, 1), (1, 1, 1, 1), (2, 0, 0, 1)]
    p = [1.0, 1.0, 0.5]
    lt, lc, rt, rc = both(tasks, p, 2.0, 1.0, 1.0, 0.0, 1, 1)
    for blocks in ([[0, 1]], [[0], [1]], [[2], [1, 0]], [[1]], []):
        want = ref.simulate(rt, p, rc, blocks)
        res, _, events = zm.sched_simulate(lt, p, lc, blocks)
        assert (res.makespan, res.io_end, res.charge) == (want.makespan, want.io_end, want.charge)
        assert len(events) == len(want.events)


def test_argument_errors():
    lt = [zm.SchedTask(0, 1, 1, 1), zm.SchedTask(1, 0, 0, 1)]
    good = zm.SchedCosts(1.0, 0.5, 1.0, 0.0, 2, 2)
    for bad in (zm.SchedCosts(-1.0, 0.5, 1.0, 0.0, 2, 2), zm.SchedCosts(1.0, float("nan"), 1.0, 0.0, 2, 2),
                zm.SchedCosts(1.0, 0.5, float("inf"), 0.0, 2, 2), zm.SchedCosts(1.0, 0.5, 1.0, 0.0, 0, 2),
                zm.SchedCosts(1.0, 0.5, 1.0, 0.0, 2, 0)):
        with pytest.raises(zm.ZipMoEError):
            zm.sched_build(lt, [1.0, 1.0], bad)
        with pytest.raises(zm.ZipMoEError):
            zm.sched_lower_bounds(lt, [1.0, 1.0], bad)
    with pytest.raises(zm.ZipMoEError):
        zm.sched_build(lt, [1.0], good)                   # expert 1 has no execution time
    with pytest.raises(zm.ZipMoEError):
        zm.sched_build(lt, [1.0, -2.0], good)
    with pytest.raises(zm.ZipMoEError):
        zm.sched_simulate(lt, [1.0, 1.0], good, [[0, 0]])  # a task twice
    with pytest.raises(zm.ZipMoEError):
        zm.sched_simulate(lt, [1.0, 1.0], good, [[0, 2]])  # no such task
    assert zm.sched_build([], [], good) == []


def test_block_structure_properties():
    # Sec. 3.3: every block but a trailing all-Type-II one opens with... contains a Type-I base; with decoding
    # slower than reading and enough Type-II work, blocks close as compute-dominant before all tasks are used.
    rng = random.Random(11)
    seen_many = False
    for _ in range(60):
        tasks, p, u, v, c, r, L, K = random_request(rng, dyadic=True)
        lt, lc, rt, rc = both(tasks, p, u, v, c, r, L, K)
        blocks = zm.sched_build(lt, p, lc)
        one = {j for j, t in enumerate(rt) if ref.is_type_one(t)}
        for b in blocks[:-1]:
            assert one & set(b)
        if blocks and not (one & set(blocks[-1])):
            assert all(j not in one for j in blocks[-1])
        for i in range(len(blocks) - 1):                  # a closed block followed by one with a base was dominant
            if one & set(blocks[i + 1]):
                res, worker_end, _ = zm.sched_simulate(lt, p, lc, blocks[: i + 1], events=False)
                ends = sorted(worker_end)
                assert all(ends[l - 1] - res.io_end >= l * v for l in range(1, min(L, K) + 1))
        seen_many = seen_many or len(blocks) > 2
    assert seen_many
