"""Reference implementation of ZipMoE's cache-pool planning (arXiv 2601.21198, Sec. 3.4, App. C, App. D).

TEST INFRASTRUCTURE ONLY: plain, slow, float64 Python; the product library never imports it and it
shares no code with the library.

What it follows
  App. D        modified iterative proportional fitting: rank-based inclusion probabilities f_i
                (sum = k) -> weights w_i with P(S) proportional to prod_{i in S} w_i over k-subsets,
                and selection probabilities q_i = w_i / (1 + w_i).
  App. C Alg. 2 probability of exactly h selections inside a rank interval (Poisson binomial).
  App. C Alg. 3 makespan estimate of a sparse layer for a hit pattern (h_F, h_C, h_S, h_E).
  App. C Alg. 4 grid search over memory ratios of the pools, expected makespan under the hit-pattern
                distribution of Sec. 3.4, conditioned on exactly k selections.

Pins (tests/test_planner_oracle.py): enumeration of all k-subsets on small N, the binomial special case,
probabilities that sum to one, hand-computed makespans.  Nothing is unpinned.
"""
from __future__ import annotations

import itertools
import math
from typing import List, Sequence, Tuple

POOLS = ("F", "C", "S", "E")


def elementary_symmetric(w: Sequence[float], n: int) -> float:
    """R(n, C) of App. D: the sum over all n-subsets of C of the product of their weights, written as the
    definition says (every subset is visited)."""
    return float(sum(math.prod(c) for c in itertools.combinations(w, n)))


def inclusion_from_weights(w: Sequence[float], k: int) -> List[float]:
    """f_i implied by weights w under P(S) ~ prod w over k-subsets: w_i R(k-1, N minus i) / R(k, N)."""
    total = elementary_symmetric(w, k)
    out = []
    for i in range(len(w)):
        rest = list(w[:i]) + list(w[i + 1:])
        out.append(w[i] * elementary_symmetric(rest, k - 1) / total)
    return out


def selection_probabilities(f: Sequence[float], k: int, iters: int = 5000, tol: float = 1e-12) -> Tuple[List[float], int]:
    """Modified iterative proportional fitting (App. D): start at w = f, multiply w_i by f_i / f_i(w) until
    the implied inclusion probabilities match; returns (q, iterations used)."""
    w = [float(x) for x in f]
    used = 0
    for used in range(1, iters + 1):
        cur = inclusion_from_weights(w, k)
        if max(abs(a - b) for a, b in zip(cur, f)) < tol:
            break
        w = [wi * fi / ci if ci > 0 else 0.0 for wi, fi, ci in zip(w, f, cur)]
    return [wi / (1.0 + wi) for wi in w], used


def hit_distribution(q: Sequence[float]) -> List[float]:
    """Alg. 2: Phi(h) = probability that exactly h of the independent selections with probabilities q occur."""
    phi = [0.0] * (len(q) + 1)
    phi[0] = 1.0
    for qr in q:
        for h in range(len(q), 0, -1):
            phi[h] = phi[h] * (1.0 - qr) + phi[h - 1] * qr
        phi[0] = phi[0] * (1.0 - qr)
    return phi


def makespan(k: int, h: Sequence[int], c: float, v: float, u: float, L: int, K: int, n: int) -> float:
    """Alg. 3: h = (h_F, h_C, h_S, h_E); c: decompression delay of one E-chunk, v: read delay of one
    E-chunk, u: read delay of one SM-chunk, L threads, K shards per tensor, n tensors per expert."""
    hF, hC, hS, hE = h
    n_sm = n * (k - hF - hC - hS)
    n_e = n * K * (k - hF - hC - hE)
    t_io = n_sm * u + n_e * v
    n_d = n * K * (k - hF)
    t_decomp = (n_e * v + n_d * c) / L
    return max(t_io, t_decomp)


def expected_makespan(q: Sequence[float], slots: Sequence[int], k: int, c: float, v: float, u: float,
                      L: int, K: int, n: int) -> float:
    """Inner part of Alg. 4: pools occupy consecutive rank intervals of sizes slots = (S_F, S_C, S_S, S_E),
    the remaining ranks form the miss pool M; the cost is the makespan of every hit pattern weighted by
    Phi_M(k_rem) / Phi_N(k) * prod_p Phi_p(h_p)."""
    at = 0
    phis = []
    for s in slots:
        phis.append(hit_distribution(q[at: at + s]))
        at += s
    phi_m = hit_distribution(q[at:])
    phi_n = hit_distribution(q)
    cost = 0.0
    for hF in range(slots[0] + 1):
        for hC in range(slots[1] + 1):
            for hS in range(slots[2] + 1):
                for hE in range(slots[3] + 1):
                    k_rem = k - hF - hC - hS - hE
                    if k_rem < 0:
                        break
                    if k_rem >= len(phi_m):
                        continue                       # more misses than there are ranks outside the pools
                    p = phi_m[k_rem] / phi_n[k] * phis[0][hF] * phis[1][hC] * phis[2][hS] * phis[3][hE]
                    cost += makespan(k, (hF, hC, hS, hE), c, v, u, L, K, n) * p
    return cost


def slots_for_ratios(ratios: Sequence[float], memory: float, bytes_per_expert: Sequence[float], n_experts: int) -> List[int]:
    """How many experts each pool holds: floor(ratio * memory / bytes of one expert in that pool's form),
    and no more ranks than are left after the pools before it."""
    left = n_experts
    out = []
    for r, b in zip(ratios, bytes_per_expert):
        s = int(math.floor(r * memory / b + 1e-9)) if r > 0 else 0
        s = min(s, left)
        left -= s
        out.append(s)
    return out


def plan_pools(f: Sequence[float], k: int, c: float, v: float, u: float, L: int, K: int, n: int,
               memory: float, bytes_per_expert: Sequence[float], grid: int, active: Sequence[bool]):
    """Alg. 4.  f: rank-based inclusion probabilities (rank 1 first); grid: number of steps the unit of
    memory is cut into (step length 1/grid); active[p]: whether pool p may get memory.  Ratios are visited
    in lexicographic order of (F, C, S, E) grid counts; a later configuration replaces the best one only if
    its cost is strictly smaller.  Returns (ratios, slots, cost)."""
    q, _ = selection_probabilities(f, k)
    best = None
    for gF in range(grid + 1):
        for gC in range(grid + 1 - gF):
            for gS in range(grid + 1 - gF - gC):
                gE = grid - gF - gC - gS
                g = (gF, gC, gS, gE)
                if any(x > 0 and not a for x, a in zip(g, active)):
                    continue
                ratios = [x / grid for x in g]
                slots = slots_for_ratios(ratios, memory, bytes_per_expert, len(f))
                cost = expected_makespan(q, slots, k, c, v, u, L, K, n)
                if best is None or cost < best[2]:
                    best = (ratios, slots, cost)
    return best
