"""Seeded synthetic MoE routing workloads (inputs only).

This module is shared by the CPU oracle's tests and by the HIP path's tests and
benchmark.  It only *draws inputs* -- hidden states X, routing ids K, gate
weights W and per-expert stand-in scales -- and holds none of the method's
arithmetic: no offsets, no placement, no reduction.  (The count matrix of synthetic
peer ranks, an INPUT of the several-sources plan, is tallied here with numpy's bincount.)

Shapes follow the paper's notation (Section 5.1): T tokens, hidden size H,
routing degree k, E experts spread over R rank regions (E_r = E / R experts
per region).  The paper's kernel benchmarks use synthetic routing on
DeepSeek-/Qwen-shaped layers (Section 6.1); the five named configurations below
are such layers.

Generator: numpy ``default_rng(seed)`` (PCG64); draw order is fixed as
X, K, logits, scales.  bf16 tensors are carried as ``uint16`` bit patterns
(numpy has no bf16); they are fp32 draws rounded to nearest-even.  Routing ids
are kept in draw order, never sorted.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional

import numpy as np

DTYPE_BF16 = 0
DTYPE_F32 = 1


@dataclass(frozen=True)
class Config:
    name: str
    T: int
    H: int
    k: int
    E: int
    R: int
    dtype: int = DTYPE_BF16          # storage type of X / window / expert_out / Y
    routing: str = "uniform"         # uniform | zipf | group_limited
    zipf_s: float = 1.2
    n_groups: int = 8                # group_limited only
    groups_per_token: int = 4        # group_limited only
    scale: str = "uniform"           # stand-in expert: "index" -> e+1, "uniform" -> U(0.5, 1.5)
    seed: int = 0

    @property
    def N(self) -> int:
        return self.T * self.k

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == DTYPE_BF16 else 4

    @property
    def payload_bytes(self) -> int:
        """Algorithmic payload bytes of one dispatch + one combine."""
        return 2 * self.T * self.H * self.elem_bytes * (1 + self.k)

    def with_(self, **kw) -> "Config":
        return replace(self, **kw)


CONFIGS: Dict[str, Config] = {
    "tiny": Config("tiny", T=16, H=128, k=2, E=8, R=2, dtype=DTYPE_F32, scale="index"),
    "decode": Config("decode", T=128, H=7168, k=8, E=256, R=32),
    "prefill": Config("prefill", T=4096, H=7168, k=8, E=256, R=32),
    "skewed": Config("skewed", T=16384, H=7168, k=8, E=256, R=32, routing="zipf"),
    "wide": Config("wide", T=32768, H=4096, k=8, E=128, R=16, routing="group_limited",
                   n_groups=8, groups_per_token=4),
}


@dataclass
class Workload:
    cfg: Config
    X: np.ndarray          # [T, H]  uint16 (bf16 bits) or float32
    K: np.ndarray          # [T, k]  int32
    W: np.ndarray          # [T, k]  float32
    scale: np.ndarray      # [E]     float32 (stand-in expert multiplier)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Storage conversion for generated data: fp32 -> bf16 bit pattern, nearest-even.

    Inputs are finite draws, so no NaN handling is needed here.
    """
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _draw_hidden(rng: np.random.Generator, T: int, H: int, dtype: int) -> np.ndarray:
    out = np.empty((T, H), dtype=np.uint16 if dtype == DTYPE_BF16 else np.float32)
    step = max(1, (1 << 24) // max(H, 1))          # bound the fp32 temporary
    for t0 in range(0, T, step):
        blk = rng.standard_normal((min(step, T - t0), H), dtype=np.float32)
        out[t0:t0 + blk.shape[0]] = f32_to_bf16_bits(blk) if dtype == DTYPE_BF16 else blk
    return out


def _topk_uniform(rng, T, k, E):
    # k distinct ids per token, uniformly: the first k entries of a random permutation
    keys = rng.random((T, E))
    return np.argsort(keys, axis=1, kind="stable")[:, :k].astype(np.int32)


def _topk_zipf(rng, T, k, E, s):
    # sampling without replacement from p_rank ~ rank^-s over a seeded expert permutation,
    # via Gumbel-top-k on log p (same law as sequential draws; ids kept in draw order)
    perm = rng.permutation(E)
    p = np.arange(1, E + 1, dtype=np.float64) ** (-s)
    logp = np.empty(E)
    logp[perm] = np.log(p / p.sum())
    g = rng.gumbel(size=(T, E))
    order = np.argsort(-(logp[None, :] + g), axis=1, kind="stable")
    return order[:, :k].astype(np.int32)


def _topk_group_limited(rng, T, k, E, n_groups, groups_per_token):
    per_group = E // n_groups
    gsel = np.argsort(rng.random((T, n_groups)), axis=1, kind="stable")[:, :groups_per_token]
    cand = groups_per_token * per_group
    pick = np.argsort(rng.random((T, cand)), axis=1, kind="stable")[:, :k]
    grp = np.take_along_axis(gsel, pick // per_group, axis=1)
    return (grp * per_group + pick % per_group).astype(np.int32)


def make(cfg: Config, seed: Optional[int] = None) -> Workload:
    """Draw one workload for ``cfg`` (seed defaults to ``cfg.seed``)."""
    rng = np.random.default_rng(cfg.seed if seed is None else seed)
    T, H, k, E = cfg.T, cfg.H, cfg.k, cfg.E
    X = _draw_hidden(rng, T, H, cfg.dtype)
    K = draw_routing(cfg, rng)
    logits = rng.standard_normal((T, k))
    w = np.exp(logits - logits.max(axis=1, keepdims=True)) if T else logits
    W = (w / w.sum(axis=1, keepdims=True)).astype(np.float32) if T else np.zeros((0, k), np.float32)
    if cfg.scale == "index":
        scale = np.arange(1, E + 1, dtype=np.float32)
    else:
        scale = rng.uniform(0.5, 1.5, size=E).astype(np.float32)
    return Workload(cfg, X, np.ascontiguousarray(K.reshape(T, k)), np.ascontiguousarray(W), scale)


def draw_routing(cfg: Config, rng: np.random.Generator) -> np.ndarray:
    """Routing ids [T,k] of ``cfg``'s routing law from ``rng`` (no hidden states are drawn)."""
    T, k, E = cfg.T, cfg.k, cfg.E
    if cfg.routing == "uniform":
        return _topk_uniform(rng, T, k, E)
    if cfg.routing == "zipf":
        return _topk_zipf(rng, T, k, E, cfg.zipf_s)
    if cfg.routing == "group_limited":
        return _topk_group_limited(rng, T, k, E, cfg.n_groups, cfg.groups_per_token)
    raise ValueError(cfg.routing)


def source_count_matrix(cfg: Config, sources: int, seed: int = 1000) -> np.ndarray:
    """Gathered count matrix M[R,E] (int32) for a run as one of several source ranks: rows 0..sources-1
    hold the per-expert branch counts of an independent draw of ``cfg``'s routing (every source rank routes
    T tokens like this one), the remaining rows are zero.  Input synthesis only: counting the ids of a
    synthetic peer is what the count exchange would deliver, not a step of the method under test."""
    M = np.zeros((cfg.R, cfg.E), np.int32)
    for r in range(min(sources, cfg.R)):
        K = draw_routing(cfg, np.random.default_rng(seed + r))
        M[r] = np.bincount(K.reshape(-1), minlength=cfg.E)
    return M


def random_routing(rng: np.random.Generator, T: int, k: int, E: int, *, distinct: bool = False,
                   p_masked: float = 0.0, p_invalid: float = 0.0) -> np.ndarray:
    """Adversarial routing for edge-case tests: ids may repeat inside a token, some
    slots may be masked (-1) or out of range (E + something, or < -1)."""
    if distinct and k <= E:
        K = _topk_uniform(rng, T, k, E)
    else:
        K = rng.integers(0, E, size=(T, k), dtype=np.int32)
    if p_masked > 0:
        K = np.where(rng.random((T, k)) < p_masked, np.int32(-1), K)
    if p_invalid > 0:
        bad = rng.random((T, k)) < p_invalid
        junk = np.where(rng.random((T, k)) < 0.5, E + rng.integers(0, 5, size=(T, k)),
                        -2 - rng.integers(0, 5, size=(T, k)))
        K = np.where(bad, junk, K)
    return np.ascontiguousarray(K.astype(np.int32))
