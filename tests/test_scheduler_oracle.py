"""Pins of the reference scheduler (oracle/scheduler.py) against things that are not the scheduler itself:
timelines worked out by hand, a validity checker written from the model's rules (Sec. 3.3), the optimum by
exhaustive search on tiny instances with the factor 3 - 1/L of Sec. 3.3, the lower bounds of App. B, and
closed forms for degenerate request sets."""
import math
import random

import pytest

from oracle import scheduler as sch
from oracle.scheduler import Costs, Task

MISSING = dict(needs_sm=True, needs_e=True)
STATE_E = dict(needs_sm=True, needs_e=False)       # E-chunks cached, SM-chunk to read
STATE_S = dict(needs_sm=False, needs_e=True)       # SM-chunk cached, E-chunks to read
STATE_C = dict(needs_sm=False, needs_e=False)
STATE_F = dict(needs_sm=False, needs_e=False, needs_decode=False)
STATES = (MISSING, STATE_E, STATE_S, STATE_C, STATE_F)


# ---------------------------------------------------------------- validity checker (independent of the oracle)

def ops_of(tasks, p, costs):
    """Every operation the request set must run: key -> (resource, duration, predecessor keys)."""
    ops = {}
    for j, t in enumerate(tasks):
        if not t.needs_decode:
            continue
        for i in range(costs.K):
            if t.needs_e:
                ops[("E", j, i)] = (sch.IO, costs.v, [])
            ops[("D", j, i)] = (sch.WORKER, costs.c, [("E", j, i)] if t.needs_e else [])
        if t.needs_sm:
            ops[("S", j, 0)] = (sch.IO, costs.u, [])
        ops[("R", j, 0)] = (sch.GPU, costs.r, [("D", j, i) for i in range(costs.K)] + ([("S", j, 0)] if t.needs_sm else []))
    for n in sorted({t.expert for t in tasks}):
        ops[("X", n, 0)] = (sch.GPU, p[n], [("R", j, 0) for j, t in enumerate(tasks) if t.expert == n and t.needs_decode])
    return ops


KIND = {sch.E_READ: "E", sch.SM_READ: "S", sch.DECOMPRESS: "D", sch.RECOVER: "R", sch.EXECUTE: "X"}


def check_timeline(tasks, p, costs, blocks, tl):
    ops = ops_of(tasks, p, costs)
    seen = {}
    for e in tl.events:
        key = (KIND[e.kind], e.task, e.chunk)
        assert key not in seen, f"{key} runs twice"
        seen[key] = e
        res, dur, _ = ops[key]
        assert e.resource == res
        assert e.end == pytest.approx(e.start + dur, abs=1e-12)
        assert e.start >= 0
    assert set(seen) == set(ops)
    # exclusive resources
    lanes = {}
    for e in tl.events:
        lanes.setdefault((e.resource, e.unit), []).append((e.start, e.end))
    assert all(unit == 0 for (res, unit) in lanes if res != sch.WORKER)
    assert all(0 <= unit < costs.L for (res, unit) in lanes if res == sch.WORKER)
    for spans in lanes.values():
        spans.sort()
        for a, b in zip(spans, spans[1:]):
            assert a[1] <= b[0] + 1e-12
    # precedence
    for key, (_, _, preds) in ops.items():
        for q in preds:
            assert seen[key].start >= seen[q].end - 1e-12, (key, q)
    # the I/O thread never waits and follows the block rule: E-chunk reads of a block, then its SM-chunk reads
    io = sorted((e for e in tl.events if e.resource == sch.IO), key=lambda e: e.start)
    want = []
    for B in blocks:
        want += [("E", j, i) for j in B if tasks[j].needs_decode and tasks[j].needs_e for i in range(costs.K)]
        want += [("S", j, 0) for j in B if tasks[j].needs_decode and tasks[j].needs_sm]
    assert [(KIND[e.kind], e.task, e.chunk) for e in io] == want
    at = 0.0
    for e in io:
        assert e.start == pytest.approx(at, abs=1e-12)
        at = e.end
    # work conservation and priority on the decompression threads
    order = [j for B in blocks for j in B]
    rank = {j: r for r, j in enumerate(order)}
    dec = [e for e in tl.events if e.kind == sch.DECOMPRESS]
    ready = {(e.task, e.chunk): (seen[("E", e.task, e.chunk)].end if tasks[e.task].needs_e else 0.0) for e in dec}
    marks = sorted({0.0} | {e.start for e in dec} | {e.end for e in dec} | set(ready.values()))
    for e in dec:
        for a, b in zip(marks, marks[1:]):
            if a >= ready[(e.task, e.chunk)] - 1e-12 and b <= e.start + 1e-12:      # e is waiting although ready
                busy = sum(1 for o in dec if o.start <= a + 1e-12 and o.end >= b - 1e-12)
                assert busy == costs.L, f"a thread idles in [{a},{b}) while {e} is ready"
        for o in dec:                                   # nobody of lower priority overtakes a ready operation
            if (rank[o.task], o.chunk) > (rank[e.task], e.chunk) and ready[(e.task, e.chunk)] <= o.start + 1e-12:
                assert o.start >= e.start - 1e-12, (o, e)
    # the GPU stream does not wait while something is ready
    gpu = sorted((e for e in tl.events if e.resource == sch.GPU), key=lambda e: (e.start, e.end))
    for prev, e in zip([None] + gpu, gpu):
        _, _, preds = ops[(KIND[e.kind], e.task, e.chunk)]
        rdy = max([seen[q].end for q in preds] + [0.0])
        free = prev.end if prev else 0.0
        assert e.start == pytest.approx(max(rdy, free), abs=1e-12)
    assert tl.makespan == pytest.approx(max([e.end for e in tl.events] + [0.0]), abs=1e-12)
    assert tl.io_end == pytest.approx(max([e.end for e in io] + [0.0]), abs=1e-12)


# ---------------------------------------------------------------- optimum by exhaustive search

def optimum(tasks, p, costs, upper):
    """Smallest makespan over all feasible schedules.  Makespan is a regular objective, so an optimal
    schedule exists among the active ones, and those are what placing operations one by one, each at the
    earliest feasible time (gaps included), in every precedence-feasible order produces."""
    ops = ops_of(tasks, p, costs)
    keys = list(ops)
    cap = {sch.IO: 1, sch.WORKER: costs.L, sch.GPU: 1}
    succ_tail = {}

    def tail(k):                                         # longest path from the start of k to the end
        if k not in succ_tail:
            nxt = [q for q in keys if k in ops[q][2]]
            succ_tail[k] = ops[k][1] + max([tail(q) for q in nxt] + [0.0])
        return succ_tail[k]

    best = [upper]

    def earliest(res, dur, ready, placed):
        spans = [(s, e) for (r, s, e) in placed.values() if r == res and e > s]
        points = sorted({ready} | {e for _, e in spans if e >= ready})
        for t in points:
            marks = sorted({t} | {s for s, _ in spans if t < s < t + dur})
            if all(sum(1 for s, e in spans if s <= m < e) < cap[res] for m in marks):
                return t
        raise AssertionError

    def go(placed, span):
        if span >= best[0] - 1e-12:
            return
        if len(placed) == len(keys):
            best[0] = span
            return
        for k in keys:
            if k in placed or any(q not in placed for q in ops[k][2]):
                continue
            res, dur, preds = ops[k]
            ready = max([placed[q][2] for q in preds] + [0.0])
            t = earliest(res, dur, ready, placed)
            if t + tail(k) >= best[0] - 1e-12:
                continue
            placed[k] = (res, t, t + dur)
            go(placed, max(span, t + dur))
            del placed[k]

    go({}, 0.0)
    return best[0]


# ---------------------------------------------------------------- timelines worked by hand

def find(tl, kind, task, chunk=0):
    (e,) = [e for e in tl.events if e.kind == kind and e.task == task and e.chunk == chunk]
    return (e.start, e.end)


def test_hand_worked_type_two_fills_the_wait_for_the_first_e_chunk():
    # L = 1, K = 2, u = 4, v = 1, c = 1, r = 0.  Task 0: expert 0 (p = 5), nothing cached.  Task 1: expert 1
    # (p = 2), compressed in memory.  The block starts as [0]: reads E 0-1, 1-2, SM 2-6; the thread decodes
    # 1-2 and 2-3 (one unit of charge), ends at 3 < 6 + 1: not compute-dominant.  Task 1 in front: the thread
    # decodes its chunks 0-1 and 1-2, then task 0's 2-3 and 3-4: no charge, so it goes to position 0.
    tasks = [Task(0, **MISSING), Task(1, **STATE_C)]
    p = [5.0, 2.0]
    costs = Costs(u=4.0, v=1.0, c=1.0, r=0.0, L=1, K=2)
    blocks = sch.build_blocks(tasks, p, costs)
    assert blocks == [[1, 0]]
    tl = sch.simulate(tasks, p, costs, blocks)
    assert find(tl, sch.E_READ, 0, 0) == (0.0, 1.0) and find(tl, sch.E_READ, 0, 1) == (1.0, 2.0)
    assert find(tl, sch.SM_READ, 0) == (2.0, 6.0)
    assert [find(tl, sch.DECOMPRESS, 1, i) for i in (0, 1)] == [(0.0, 1.0), (1.0, 2.0)]
    assert [find(tl, sch.DECOMPRESS, 0, i) for i in (0, 1)] == [(2.0, 3.0), (3.0, 4.0)]
    assert find(tl, sch.RECOVER, 1) == (2.0, 2.0) and find(tl, sch.EXECUTE, 1) == (2.0, 4.0)
    assert find(tl, sch.RECOVER, 0) == (6.0, 6.0) and find(tl, sch.EXECUTE, 0) == (6.0, 11.0)
    assert tl.makespan == 11.0 and tl.charge == 0.0 and tl.io_end == 6.0 and tl.worker_end == [4.0]
    assert tl.makespan == sch.lower_bounds(tasks, p, costs)["Z"]          # it is optimal here
    check_timeline(tasks, p, costs, blocks, tl)


def test_hand_worked_compute_dominant_block_closes_early():
    # As above with c = 3: the lone base decodes 1-4 and 4-7, 7 - 6 >= 1: compute-dominant, the block closes
    # with the base alone and the Type-II task forms the last block.  At run time the thread is free at 0 and
    # only task 1's chunks are ready, so work conservation runs one of them first: 0-3, then task 0's
    # (ready since 1 and 2) 3-6 and 6-9, then task 1's second 9-12.
    tasks = [Task(0, **MISSING), Task(1, **STATE_C)]
    p = [5.0, 2.0]
    costs = Costs(u=4.0, v=1.0, c=3.0, r=0.0, L=1, K=2)
    blocks = sch.build_blocks(tasks, p, costs)
    assert blocks == [[0], [1]]
    tl = sch.simulate(tasks, p, costs, blocks)
    assert [find(tl, sch.DECOMPRESS, 1, i) for i in (0, 1)] == [(0.0, 3.0), (9.0, 12.0)]
    assert [find(tl, sch.DECOMPRESS, 0, i) for i in (0, 1)] == [(3.0, 6.0), (6.0, 9.0)]
    assert find(tl, sch.EXECUTE, 0) == (9.0, 14.0) and find(tl, sch.EXECUTE, 1) == (14.0, 16.0)
    assert tl.makespan == 16.0 and tl.charge == 0.0
    check_timeline(tasks, p, costs, blocks, tl)


def test_hand_worked_fallback_position_and_recovery_delay():
    # L = 1, K = 2, u = 4, v = 1, c = 0.5, r = 0.25.  Task 0: expert 0 (p = 5) nothing cached; task 1:
    # expert 1 (p = 2) SM cached.  Base alone: decodes 1-1.5 and 2-2.5, charge 1.5.  Task 1 in front or behind
    # adds two more E-chunk reads the thread has to wait for (charge 2.5 either way), so the fallback puts it
    # behind the base.  Reads: E 0-1, 1-2 (task 0), 2-3, 3-4 (task 1), SM 4-8.
    tasks = [Task(0, **MISSING), Task(1, **STATE_S)]
    p = [5.0, 2.0]
    costs = Costs(u=4.0, v=1.0, c=0.5, r=0.25, L=1, K=2)
    blocks = sch.build_blocks(tasks, p, costs)
    assert blocks == [[0, 1]]
    tl = sch.simulate(tasks, p, costs, blocks)
    assert [find(tl, sch.DECOMPRESS, 0, i) for i in (0, 1)] == [(1.0, 1.5), (2.0, 2.5)]
    assert [find(tl, sch.DECOMPRESS, 1, i) for i in (0, 1)] == [(3.0, 3.5), (4.0, 4.5)]
    assert tl.charge == 2.5
    assert find(tl, sch.RECOVER, 1) == (4.5, 4.75) and find(tl, sch.EXECUTE, 1) == (4.75, 6.75)
    assert find(tl, sch.RECOVER, 0) == (8.0, 8.25) and find(tl, sch.EXECUTE, 0) == (8.25, 13.25)
    assert tl.makespan == 13.25
    check_timeline(tasks, p, costs, blocks, tl)


def test_hand_worked_two_threads_and_two_tensors():
    # L = 2, K = 2, u = 2, v = 0.5, c = 1, r = 0.  Expert 0 (p = 3) has two tensors with E-chunks cached
    # (tasks 0, 1: Type-I); expert 1 (p = 1) has one compressed tensor (task 2).  Base task 0: SM 0-2, threads
    # decode 0-1 each, F = (1, 1), 1 - 2 < 0.5: not dominant.  Task 2 at position 0: threads decode task 2
    # 0-1, task 0 1-2: no charge, block [2, 0], F = (2, 2), I/O 2: still not dominant (0 < 0.5).  Next from
    # U is task 1 (Type-I): position 0 is free of charge: block [1, 2, 0]; reads SM(1) 0-2, SM(0) 2-4; threads:
    # task 1 0-1 both, task 2 1-2 both, task 0 2-3 both.  GPU: task 1 recovered at 2; task 2 at 2, expert 1
    # runs 2-3; task 0 at 4, expert 0 runs 4-7.
    tasks = [Task(0, **STATE_E), Task(0, **STATE_E), Task(1, **STATE_C)]
    p = [3.0, 1.0]
    costs = Costs(u=2.0, v=0.5, c=1.0, r=0.0, L=2, K=2)
    blocks = sch.build_blocks(tasks, p, costs)
    assert blocks == [[1, 2, 0]]
    tl = sch.simulate(tasks, p, costs, blocks)
    assert find(tl, sch.SM_READ, 1) == (0.0, 2.0) and find(tl, sch.SM_READ, 0) == (2.0, 4.0)
    assert sorted(find(tl, sch.DECOMPRESS, 1, i) for i in (0, 1)) == [(0.0, 1.0), (0.0, 1.0)]
    assert sorted(find(tl, sch.DECOMPRESS, 2, i) for i in (0, 1)) == [(1.0, 2.0), (1.0, 2.0)]
    assert sorted(find(tl, sch.DECOMPRESS, 0, i) for i in (0, 1)) == [(2.0, 3.0), (2.0, 3.0)]
    assert find(tl, sch.EXECUTE, 1) == (2.0, 3.0) and find(tl, sch.EXECUTE, 0) == (4.0, 7.0)
    assert tl.makespan == 7.0 and tl.worker_end == [3.0, 3.0]
    check_timeline(tasks, p, costs, blocks, tl)


def test_hand_worked_every_thread_has_its_own_lag_threshold():
    # L = 2, K = 2, u = 2, v = 1, c = 3.5.  Base: expert 0 (p = 2), E-chunks cached: SM 0-2, both threads decode
    # 0-3.5.  The earliest thread lags the I/O thread by 1.5 >= 1 v, the second one by 1.5 < 2 v: not
    # compute-dominant, so the compressed task of expert 1 (p = 1) is drawn in; in front it costs no idle time.
    tasks = [Task(0, **STATE_E), Task(1, **STATE_C)]
    p = [2.0, 1.0]
    costs = Costs(u=2.0, v=1.0, c=3.5, r=0.0, L=2, K=2)
    assert not sch.compute_dominant(sch.simulate(tasks, p, costs, [[0]]), costs)
    assert sch.compute_dominant(sch.simulate(tasks, p, costs, [[1, 0]]), costs)      # lags 5 and 5
    blocks = sch.build_blocks(tasks, p, costs)
    assert blocks == [[1, 0]]
    tl = sch.simulate(tasks, p, costs, blocks)
    assert sorted(find(tl, sch.DECOMPRESS, 0, i) for i in (0, 1)) == [(3.5, 7.0), (3.5, 7.0)]
    assert find(tl, sch.EXECUTE, 1) == (3.5, 4.5) and find(tl, sch.EXECUTE, 0) == (7.0, 9.0)
    assert tl.makespan == 9.0


# ---------------------------------------------------------------- closed forms

@pytest.mark.parametrize("L,K,n_tensors,k", [(1, 4, 3, 2), (3, 4, 2, 3), (4, 2, 1, 5), (2, 8, 3, 1)])
def test_all_compressed_equal_experts_closed_form(L, K, n_tensors, k):
    # Nothing to read: the threads decode k*n*K chunks back to back; every expert's execution (p each) follows
    # its own last chunk, and the GPU is a single queue.
    c, r, pe = 1.0, 0.0, 0.125
    tasks = [Task(n, **STATE_C) for n in range(k) for _ in range(n_tensors)]
    p = [pe] * k
    costs = Costs(u=9.0, v=1.0, c=c, r=r, L=L, K=K)
    blocks = sch.build_blocks(tasks, p, costs)
    assert blocks == [list(range(len(tasks)))]            # no Type-I task: one block in sorted order
    tl = sch.simulate(tasks, p, costs, blocks)
    assert tl.charge == 0.0 and tl.io_end == 0.0
    assert tl.makespan == math.ceil(k * n_tensors * K / L) * c + pe
    check_timeline(tasks, p, costs, blocks, tl)


def test_all_full_experts_cost_only_their_execution():
    tasks = [Task(n, **STATE_F) for n in range(4) for _ in range(3)]
    p = [0.5, 2.0, 1.0, 0.25]
    costs = Costs(u=1.0, v=0.25, c=1.0, r=1.0, L=2, K=4)
    blocks = sch.build_blocks(tasks, p, costs)
    assert [tasks[j].expert for j in blocks[0]] == [1, 1, 1, 2, 2, 2, 0, 0, 0, 3, 3, 3]    # by tokens
    tl = sch.simulate(tasks, p, costs, blocks)
    assert tl.makespan == sum(p)
    assert [e.task for e in tl.events] == [1, 2, 0, 3]


def test_io_bound_requests_finish_one_chunk_after_the_last_read():
    # Everything must be read and decoding is cheap (c < v, L >= 1): the I/O thread is the bottleneck; with one
    # block the E-chunks come first, so the last operation chain is the base's SM-chunk read, its recovery and
    # its execution.
    k, n, K = 3, 2, 4
    tasks = [Task(e, **MISSING) for e in range(k) for _ in range(n)]
    p = [0.5] * k
    costs = Costs(u=2.0, v=0.5, c=0.125, r=0.25, L=2, K=K)
    blocks = sch.build_blocks(tasks, p, costs)
    assert len(blocks) == 1 and sorted(blocks[0]) == list(range(k * n))
    tl = sch.simulate(tasks, p, costs, blocks)
    assert tl.io_end == k * n * (K * 0.5 + 2.0)
    assert tl.makespan == tl.io_end + 0.25 + 0.5
    check_timeline(tasks, p, costs, blocks, tl)


# ---------------------------------------------------------------- random instances

def random_instance(rng, max_ops):
    while True:
        K = rng.choice([1, 2])
        L = rng.choice([1, 2, 3])
        n_exp = rng.choice([1, 2, 3])
        tasks = []
        for e in range(n_exp):
            st = rng.choice(STATES)
            tasks += [Task(e, **st) for _ in range(rng.choice([1, 1, 2]))]
        unit = [0.25, 0.5, 1.0, 1.5, 2.0, 3.0]
        costs = Costs(u=rng.choice(unit), v=rng.choice(unit[:4]), c=rng.choice(unit), r=rng.choice([0.0, 0.0, 0.25]), L=L, K=K)
        p = [rng.choice(unit) for _ in range(n_exp)]
        if len(ops_of(tasks, p, costs)) <= max_ops:
            return tasks, p, costs


def test_random_instances_are_valid_and_respect_the_lower_bounds():
    rng = random.Random(20260121)
    for _ in range(300):
        tasks, p, costs = random_instance(rng, 40)
        blocks = sch.build_blocks(tasks, p, costs)
        assert sorted(j for B in blocks for j in B) == list(range(len(tasks)))
        tl = sch.simulate(tasks, p, costs, blocks)
        check_timeline(tasks, p, costs, blocks, tl)
        for name, bound in sch.lower_bounds(tasks, p, costs).items():
            assert tl.makespan >= bound - 1e-12, name
        one = [j for j in range(len(tasks)) if sch.is_type_one(tasks[j])]
        if one:                                          # every block but a trailing Type-II one has a base
            first = blocks[0]
            assert any(j in one for j in first)


def test_against_the_optimum_on_tiny_instances():
    # Sec. 3.3's theorem: ALG <= (3 - 1/L) OPT; and nothing beats the optimum, the lower bounds included.
    rng = random.Random(7)
    worst = 0.0
    for _ in range(120):
        tasks, p, costs = random_instance(rng, 11)
        blocks = sch.build_blocks(tasks, p, costs)
        alg = sch.simulate(tasks, p, costs, blocks).makespan
        opt = optimum(tasks, p, costs, alg + 1e-9)
        assert opt <= alg + 1e-9
        for name, bound in sch.lower_bounds(tasks, p, costs).items():
            assert opt >= bound - 1e-12, name
        if opt > 0:
            assert alg <= (3.0 - 1.0 / costs.L) * opt + 1e-12
            worst = max(worst, alg / opt)
    assert 1.0 <= worst < 2.0                          # observed: well inside the bound


def test_priority_order_matters_to_the_simulation():
    # The same requests under two block lists give different timelines: the simulator reads the order.
    tasks = [Task(0, **MISSING), Task(1, **MISSING)]
    p = [1.0, 1.0]
    costs = Costs(u=2.0, v=1.0, c=1.0, r=0.0, L=1, K=1)
    a = sch.simulate(tasks, p, costs, [[0, 1]])
    b = sch.simulate(tasks, p, costs, [[0], [1]])
    # one block: E(0) 0-1, E(1) 1-2, SM(0) 2-4, SM(1) 4-6; two blocks: E(0) 0-1, SM(0) 1-3, E(1) 3-4, SM(1) 4-6
    assert find(a, sch.SM_READ, 0) == (2.0, 4.0) and find(b, sch.SM_READ, 0) == (1.0, 3.0)
    assert find(a, sch.EXECUTE, 0) == (4.0, 5.0) and find(b, sch.EXECUTE, 0) == (3.0, 4.0)
    assert a.makespan == b.makespan == 7.0
