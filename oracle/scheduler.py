"""Reference implementation of ZipMoE's cache-affinity scheduling (arXiv 2601.21198, Sec. 3.3, App. A, App. B).

TEST INFRASTRUCTURE ONLY: plain, slow Python in float64; the product library never imports it and it
shares no code with the library.

What it follows
  Sec. 3.3 "DAG Representation"  one reconstruction task per tensor; its operations are K E-chunk reads
                 (each rho*u/K), one SM-chunk read (u), K decompressions (each c, one per E-chunk, ready
                 once that E-chunk is in memory), a recovery on the GPU stream once all K decompressions
                 and the SM-chunk are there, and, per expert, an execution of length p_n once all of the
                 expert's tensors are recovered.  Which reads a task needs depends on its compression
                 state (F: nothing at all, C: decompress only, S: E-chunk reads, E: SM-chunk read,
                 missing: both).
  Sec. 3.3 "Task Partition"      Type-I = tasks that must read their SM-chunk, Type-II = the others; each
                 class sorted by non-increasing p of the task's expert, tensors of an expert kept together.
  Sec. 3.3 "Block Construction", App. A Alg. 1 and its definition of a compute-dominant block.
  App. A         execution: one I/O thread, L decompression threads and one GPU stream each take the first
                 available operation in the priority order of the blocks (work-conserving list scheduling).
  App. B         the charged (idle) time before a decompression on its thread; the lower bounds
                 OPT >= max(I, C/L, P, Z).

Readings where the paper leaves a choice:
  * The I/O thread has no precedence constraints, so it runs its reads back to back: block after block,
    inside a block all E-chunk reads in task order, then all SM-chunk reads in task order.
  * A free decompression thread takes the first decompression, in (block, task position, chunk) order,
    whose E-chunk has arrived; if none has, it waits for the earliest arrival.  Among threads that are
    free at the same time the lowest-numbered one is used.
  * The GPU stream takes, in the same priority order, recoveries and expert executions; an expert's
    execution has the priority of the expert's last task in the order.  The recovery has its own cost r
    (the paper's analysis has none: r = 0 gives its model).
  * The insertion test of Alg. 1 (a position that adds no idle time on any thread): the total charged time of App. B (sum over decompressions of
    the idle gap before it on its thread), with the blocks built so far in front, must not grow.
  * A block is compute-dominant when, with the worker completion times sorted increasingly as
    F(1) <= ... <= F(L), F(l) - F_io >= l * rho*u/K for every l in 1..min(L, K)  (Sec. 3.3's wording;
    App. A's formula has the same right-hand side).
  * The fallback position is right after the last Type-II task of the block whose expert has at least as
    many tokens (after the last such Type-I task if the block has no Type-II task; the end of the block if
    there is no such task at all).
  * Type-II tasks that are left when no Type-I task remains form one last block in their sorted order.

Pins (tests/test_scheduler_oracle.py): timelines worked by hand, an independent validity checker
(precedence, exclusive resources, durations, work conservation), the lower bounds of App. B, the optimum by
exhaustive search on tiny instances together with the factor 3 - 1/L of Sec. 3.3, closed forms for the
all-F, all-C and I/O-bound cases.  Nothing is unpinned.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple

E_READ, SM_READ, DECOMPRESS, RECOVER, EXECUTE = range(5)
IO, WORKER, GPU = range(3)


@dataclass(frozen=True)
class Task:
    """One tensor-level reconstruction task."""
    expert: int
    needs_sm: bool          # the SM-chunk is not in memory: Type-I
    needs_e: bool           # the E-chunks are not in memory
    needs_decode: bool = True   # False: the tensor is held in full, nothing to reconstruct


@dataclass(frozen=True)
class Costs:
    u: float                # read delay of one SM-chunk
    v: float                # read delay of one E-chunk (rho * u / K)
    c: float                # decompression delay of one E-chunk
    r: float                # recovery delay of one tensor on the GPU stream
    L: int                  # decompression threads
    K: int                  # E-chunks per tensor


@dataclass(frozen=True)
class Event:
    kind: int
    task: int               # task index; for EXECUTE the expert id
    chunk: int              # E-chunk index for E_READ / DECOMPRESS, else 0
    resource: int           # IO, WORKER or GPU
    unit: int               # which decompression thread; 0 for the others
    start: float
    end: float


@dataclass
class Timeline:
    events: List[Event]
    makespan: float
    io_end: float
    worker_end: List[float]
    charge: float           # total idle time in front of decompressions on their threads (App. B)


def is_type_one(t: Task) -> bool:
    return t.needs_decode and t.needs_sm


def simulate(tasks: Sequence[Task], p: Sequence[float], costs: Costs, blocks: Sequence[Sequence[int]]) -> Timeline:
    """Run the operations of the tasks named in `blocks` (lists of task indices, highest priority first)."""
    K, L = costs.K, costs.L
    events: List[Event] = []
    order = [j for B in blocks for j in B]

    # I/O thread
    t = 0.0
    e_at: Dict[Tuple[int, int], float] = {}
    sm_at: Dict[int, float] = {}
    for B in blocks:
        for j in B:
            if tasks[j].needs_decode and tasks[j].needs_e:
                for i in range(K):
                    events.append(Event(E_READ, j, i, IO, 0, t, t + costs.v))
                    t = t + costs.v
                    e_at[(j, i)] = t
        for j in B:
            if tasks[j].needs_decode and tasks[j].needs_sm:
                events.append(Event(SM_READ, j, 0, IO, 0, t, t + costs.u))
                t = t + costs.u
                sm_at[j] = t
    io_end = t

    # decompression threads
    pending = [(j, i) for j in order if tasks[j].needs_decode for i in range(K)]
    free = [0.0] * L
    charge = 0.0
    decoded_at: Dict[int, float] = {}
    while pending:
        w = min(range(L), key=lambda x: (free[x], x))
        now = free[w]
        pick = next((op for op in pending if e_at.get(op, 0.0) <= now), None)
        if pick is None:
            now = min(e_at.get(op, 0.0) for op in pending)
            pick = next(op for op in pending if e_at.get(op, 0.0) <= now)
        pending.remove(pick)
        charge += now - free[w]
        events.append(Event(DECOMPRESS, pick[0], pick[1], WORKER, w, now, now + costs.c))
        free[w] = now + costs.c
        decoded_at[pick[0]] = max(decoded_at.get(pick[0], 0.0), free[w])

    # GPU stream: (priority, kind, id); an execution ranks right after the expert's last task
    last_pos: Dict[int, int] = {}
    for pos, j in enumerate(order):
        last_pos[tasks[j].expert] = pos
    ops = []
    for pos, j in enumerate(order):
        if tasks[j].needs_decode:
            ops.append((pos, 0, RECOVER, j))
    for n, pos in last_pos.items():
        ops.append((pos, 1, EXECUTE, n))
    ops.sort()
    recovered_at: Dict[int, float] = {j: 0.0 for j in order if not tasks[j].needs_decode}
    members: Dict[int, List[int]] = {}
    for j in order:
        members.setdefault(tasks[j].expert, []).append(j)

    def ready_time(op):
        _, _, kind, x = op
        if kind == RECOVER:
            return max(decoded_at[x], sm_at.get(x, 0.0))
        if all(j in recovered_at for j in members[x]):
            return max([recovered_at[j] for j in members[x]] + [0.0])
        return None                                    # a recovery of this expert is still to be placed

    gpu = 0.0
    while ops:
        known = [(op, ready_time(op)) for op in ops]
        known = [(op, rt) for op, rt in known if rt is not None]
        now = gpu
        pick = next((op for op, rt in known if rt <= now), None)
        if pick is None:
            now = min(rt for _, rt in known)
            pick = next(op for op, rt in known if rt <= now)
        ops.remove(pick)
        _, _, kind, x = pick
        dur = costs.r if kind == RECOVER else p[x]
        events.append(Event(kind, x, 0, GPU, 0, now, now + dur))
        gpu = now + dur
        if kind == RECOVER:
            recovered_at[x] = gpu
    return Timeline(events, gpu, io_end, free, charge)


def compute_dominant(tl: Timeline, costs: Costs) -> bool:
    """App. A, definition of a compute-dominant block (with Sec. 3.3's reading of the index l)."""
    ends = sorted(tl.worker_end)
    return all(ends[l - 1] - tl.io_end >= l * costs.v for l in range(1, min(costs.L, costs.K) + 1))


def sorted_classes(tasks: Sequence[Task], p: Sequence[float]) -> Tuple[List[int], List[int]]:
    """Sec. 3.3 "Task Partition": the two priority sequences."""
    key = lambda j: (-p[tasks[j].expert], tasks[j].expert, j)
    one = sorted((j for j in range(len(tasks)) if is_type_one(tasks[j])), key=key)
    two = sorted((j for j in range(len(tasks)) if not is_type_one(tasks[j])), key=key)
    return one, two


def build_blocks(tasks: Sequence[Task], p: Sequence[float], costs: Costs) -> List[List[int]]:
    """App. A Alg. 1."""
    sigma1, sigma2 = sorted_classes(tasks, p)
    blocks: List[List[int]] = []
    while sigma1:
        B = [sigma1.pop(0)]
        while sigma1 or sigma2:
            now = simulate(tasks, p, costs, blocks + [B])
            if compute_dominant(now, costs):
                break
            j = sigma2.pop(0) if sigma2 else sigma1.pop(0)
            slack = 1e-12 * (1.0 + now.charge)
            placed = False
            for pos in range(len(B) + 1):
                cand = B[:pos] + [j] + B[pos:]
                if simulate(tasks, p, costs, blocks + [cand]).charge <= now.charge + slack:
                    B, placed = cand, True
                    break
            if not placed:
                pj = p[tasks[j].expert]
                has_two = any(not is_type_one(tasks[i]) for i in B)
                at = len(B)
                for pos in range(len(B) - 1, -1, -1):
                    i = B[pos]
                    if (not is_type_one(tasks[i])) == has_two and p[tasks[i].expert] >= pj:
                        at = pos + 1
                        break
                B = B[:at] + [j] + B[at:]
        blocks.append(B)
    if sigma2:
        blocks.append(list(sigma2))
    return blocks


def lower_bounds(tasks: Sequence[Task], p: Sequence[float], costs: Costs) -> Dict[str, float]:
    """App. B, the lemma on OPT: total I/O, total decompression over L threads, total execution, and the
    longest critical path of one task (with the recovery delay added where a task has one)."""
    K, L = costs.K, costs.L
    io = comp = 0.0
    z = 0.0
    for t in tasks:
        if not t.needs_decode:
            z = max(z, p[t.expert])
            continue
        io += (K * costs.v if t.needs_e else 0.0) + (costs.u if t.needs_sm else 0.0)
        comp += K * costs.c
        rounds = -(-K // min(K, L))
        path = (K * costs.v if t.needs_e else 0.0)
        path = max(path + costs.c, costs.v + rounds * costs.c) if t.needs_e else rounds * costs.c
        path = max(path, (K * costs.v if t.needs_e else 0.0) + (costs.u if t.needs_sm else 0.0))
        z = max(z, path + costs.r + p[t.expert])
    execs = sum(p[n] for n in {t.expert for t in tasks})
    return {"I": io, "C/L": comp / L, "P": execs, "Z": z}
