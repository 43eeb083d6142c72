"""Seeded synthetic inputs: bf16 expert weights and routing draws.

This module holds no codec arithmetic.  It only produces tensors (as uint16
arrays holding bf16 bit patterns) and expert selections with the shapes, value
distributions and routing skew of the workloads; it is the one module that both
the reference codec's tests and the GPU path's tests import.

The tensors stand in for the expert weights of the MoE models evaluated in
ZipMoE (arXiv 2601.21198, Sec. 5: DeepSeekV2-Lite, Qwen1.5-MoE,
Switch-Large-128), which are not available offline: SwiGLU experts of three
matrices, bf16, zero-mean Gaussian entries whose exponent field has about 2.5
to 2.7 bits of entropy, as Fig. 2 of the paper reports for the real models.
Routing draws stand in for the skewed rank-popularity the paper describes in
Sec. 3.4.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np

MATRIX_NAMES = ("gate", "up", "down")


def bf16_round(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns, round to nearest, ties to even."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_to_float(w: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(w, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(*key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(list(key))))


@dataclass(frozen=True)
class Workload:
    """One benchmark configuration."""
    name: str
    ident: int                 # enters every seed
    n_layers: int
    n_experts: int
    hidden: int
    intermediate: int
    top_k: int
    chunk_values: int
    routing: str               # "all", "zipf" or "uniform"
    zipf_s: float = 0.0
    n_calls: int = 1           # calls per layer the workload is defined over
    single_matrix: Tuple[int, int] = (0, 0)   # config 1 only: one plain matrix

    def shapes(self) -> List[Tuple[int, int]]:
        if self.single_matrix != (0, 0):
            return [self.single_matrix]
        h, i = self.hidden, self.intermediate
        return [(i, h), (i, h), (h, i)]        # gate, up: [I, H]; down: [H, I]; row-major

    def values_per_expert(self) -> int:
        return sum(r * c for r, c in self.shapes())


CFG1 = Workload("cfg1-matrix-256x512", 1, 1, 1, 0, 0, 1, 4096, "all", single_matrix=(256, 512))
CFG2 = Workload("cfg2-expert-2048x1408-outliers", 2, 1, 1, 2048, 1408, 1, 16384, "all")
CFG3 = Workload("cfg3-layer-64x(2048,1024)-top8-zipf1.1", 3, 1, 64, 2048, 1024, 8, 16384, "zipf", 1.1, 100)
CFG4 = Workload("cfg4-layer-8x(4096,14336)-top2-uniform", 4, 1, 8, 4096, 14336, 2, 16384, "uniform", 0.0, 1000)
CFG5 = Workload("cfg5-model-24x60x(2048,1408)-top4-zipf1.2", 5, 24, 60, 2048, 1408, 4, 16384, "zipf", 1.2, 256)
WORKLOADS = {w.name.split("-")[0]: w for w in (CFG1, CFG2, CFG3, CFG4, CFG5)}


def expert_std(wl: Workload, layer: int, expert: int) -> float:
    """Standard deviation of the Gaussian body of one expert's entries."""
    if wl.ident in (1, 2):
        return 0.02
    if wl.ident == 3:      # per-expert std ~ U[0.01, 0.04]
        return float(_rng(wl.ident, 1000, expert).uniform(0.01, 0.04))
    if wl.ident == 4:
        return 0.015
    if wl.ident == 5:      # per-layer std ~ U[0.01, 0.05]
        return float(_rng(wl.ident, 1000, layer).uniform(0.01, 0.05))
    raise ValueError(wl.name)


def expert_matrix(wl: Workload, layer: int, expert: int, matrix: int) -> np.ndarray:
    """bf16 bit patterns (uint16, shape [rows, cols]) of one expert matrix."""
    rows, cols = wl.shapes()[matrix]
    if wl.ident == 1:
        rng = np.random.Generator(np.random.PCG64(0))          # "seed 0"
    else:
        rng = _rng(wl.ident, layer, expert, matrix)
    x = rng.standard_normal((rows, cols), dtype=np.float32)
    x *= np.float32(expert_std(wl, layer, expert))
    if wl.ident == 2:      # 1 % of the entries replaced by draws from N(0, 0.2^2)
        mask = rng.random((rows, cols), dtype=np.float32) < np.float32(0.01)
        wide = rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(0.2)
        x = np.where(mask, wide, x)
    if wl.ident == 4:      # every output row scaled by a LogNormal(0, 0.3) draw
        scale = rng.lognormal(0.0, 0.3, size=(rows, 1)).astype(np.float32)
        x *= scale
    return bf16_round(x)


def expert_tensors(wl: Workload, layer: int, expert: int) -> List[np.ndarray]:
    return [expert_matrix(wl, layer, expert, m) for m in range(len(wl.shapes()))]


def route(wl: Workload, layer: int, call: int) -> np.ndarray:
    """The distinct expert ids (int32, length top_k) one call decodes."""
    if wl.routing == "all":
        return np.arange(wl.n_experts, dtype=np.int32)[: wl.top_k]
    rng = _rng(wl.ident, 2000, layer, call)
    if wl.routing == "uniform":
        return rng.choice(wl.n_experts, size=wl.top_k, replace=False).astype(np.int32)
    # zipf: popularity rank r (1-based) has weight r^-s; ranks map to expert ids through a
    # fixed per-layer permutation; k distinct experts are drawn without replacement
    perm = _rng(wl.ident, 3000, layer).permutation(wl.n_experts)
    p = np.arange(1, wl.n_experts + 1, dtype=np.float64) ** (-wl.zipf_s)
    p /= p.sum()
    ranks = rng.choice(wl.n_experts, size=wl.top_k, replace=False, p=p)
    return perm[ranks].astype(np.int32)


# ---- small adversarial tensors for edge cases -------------------------------------------

def special_tensor(kind: str, n: int, seed: int = 0) -> np.ndarray:
    """uint16 bf16 patterns of length n with awkward exponent statistics."""
    rng = _rng(77, seed, n)
    if kind == "all_equal":
        return np.full(n, 0x3C00, np.uint16)
    if kind == "two_exponents":
        w = np.where(np.arange(n) % 2 == 0, 0x3C00, 0x3C80).astype(np.uint16)
        return w | rng.integers(0, 128, n, dtype=np.uint16)
    if kind == "uniform_u16":
        return rng.integers(0, 65536, n, dtype=np.uint16)
    if kind == "rare_last":
        w = bf16_round(rng.standard_normal(n, dtype=np.float32) * np.float32(0.02))
        if n:
            w[-1] = 0x7F81      # a NaN pattern: exponent 255 appears once, at the end
        return w
    if kind == "gauss":
        return bf16_round(rng.standard_normal(n, dtype=np.float32) * np.float32(0.02))
    if kind == "wide":          # some forty distinct exponents with long tails: log-normal magnitudes
        mag = np.exp(rng.normal(0.0, 3.0, n)).astype(np.float32)
        return bf16_round(mag * rng.choice(np.array([-1.0, 1.0], np.float32), n))
    if kind == "many_long":     # one exponent half of the time, the other 255 equally rare: with a limit above 8 bits
        e = np.where(rng.random(n) < 0.5, 0x70, rng.integers(0, 256, n)).astype(np.uint16)   # there are many codes of 9 bits
        return (e << 7) | rng.integers(0, 128, n, dtype=np.uint16) | (rng.integers(0, 2, n, dtype=np.uint16) << 15)
    raise ValueError(kind)
