"""Seeded synthetic inputs for the verification hot path (trees, Q/K/V, needles).

This module only draws numbers and lays them out.  It contains none of the
method's arithmetic (no attention, no softmax, no scoring, no selection), so
both the CPU oracle's tests and the HIP path's tests / benchmark can take
their inputs from here without sharing any computation.

Layouts (row-major, last index fastest):
  q         [T, Hq, d]        tree-token queries
  k_prefix  [Hkv, L, d]       target-model cached keys   (v_prefix likewise)
  k_tree    [Hkv, T, d]       keys of the tree tokens    (v_tree likewise)
  parent    [T] int32         parent[i] < i, -1 marks a root
  draft_k   [Ld, Hd, L, d]    draft-model cache          (draft_v likewise)

bf16 tensors are drawn in fp32, rounded once to nearest-even bf16, and both
the 16-bit patterns and the exactly equal fp32 values are returned, so every
consumer sees the same numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

# --------------------------------------------------------------------------
# bf16 <-> fp32 bit conversions (round to nearest even), pure integer work
# --------------------------------------------------------------------------


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(x: np.ndarray, dtype: str) -> np.ndarray:
    """Return x as fp32 values that are exactly representable in `dtype`."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(x))
    if dtype == "f32":
        return x
    raise ValueError(f"unknown dtype {dtype!r}")


# --------------------------------------------------------------------------
# draft trees (parent-index arrays in topological order)
# --------------------------------------------------------------------------


def tree_depths(parent: np.ndarray) -> np.ndarray:
    """Depth of each node, roots have depth 0 (pure index chasing)."""
    parent = np.asarray(parent)
    depth = np.zeros(len(parent), dtype=np.int32)
    for i, p in enumerate(parent):
        depth[i] = 0 if p < 0 else depth[p] + 1
    return depth


def random_parent_tree(n: int, max_depth: int, rng: np.random.Generator) -> np.ndarray:
    """Node 0 is the root; parent[i] uniform in [0, i), redrawn until the
    node's depth is at most `max_depth` (root depth 0)."""
    parent = np.full(n, -1, dtype=np.int32)
    depth = np.zeros(n, dtype=np.int32)
    for i in range(1, n):
        while True:
            p = int(rng.integers(0, i))
            if depth[p] + 1 <= max_depth:
                break
        parent[i] = p
        depth[i] = depth[p] + 1
    return parent


def eagle_style_tree(n: int, max_depth: int, rng: np.random.Generator,
                     root_fanout=(4, 8), inner_fanout=(1, 3)) -> np.ndarray:
    """Top-heavy tree in breadth-first order, truncated at n nodes.

    The root gets U{root_fanout} children, every deeper node U{inner_fanout}
    children, nodes at `max_depth` get none.  If the frontier dies out before
    n nodes exist, the remaining nodes are attached to seeded random nodes
    whose depth allows a child, which keeps parent[i] < i.
    """
    parent = [-1]
    depth = [0]
    frontier = [0]
    while frontier and len(parent) < n:
        nxt = []
        for node in frontier:
            if depth[node] >= max_depth:
                continue
            lo, hi = root_fanout if node == 0 else inner_fanout
            for _ in range(int(rng.integers(lo, hi + 1))):
                if len(parent) >= n:
                    break
                parent.append(node)
                depth.append(depth[node] + 1)
                nxt.append(len(parent) - 1)
        frontier = nxt
    while len(parent) < n:
        cand = [i for i in range(len(parent)) if depth[i] < max_depth]
        p = cand[int(rng.integers(0, len(cand)))]
        parent.append(p)
        depth.append(depth[p] + 1)
    return np.asarray(parent, dtype=np.int32)


def wide_tree(n: int, max_depth: int, rng: np.random.Generator) -> np.ndarray:
    """Wide shallow tree: breadth-first, every level roughly equally full."""
    parent = np.full(n, -1, dtype=np.int32)
    depth = np.zeros(n, dtype=np.int32)
    per_level = max(1, (n - 1 + max_depth - 1) // max_depth)
    level_start = 0
    level_end = 1
    i = 1
    for lvl in range(1, max_depth + 1):
        cnt = min(per_level, n - i)
        for _ in range(cnt):
            p = int(rng.integers(level_start, level_end))
            parent[i] = p
            depth[i] = depth[p] + 1
            i += 1
        level_start, level_end = level_end, i
        if i >= n:
            break
    return parent


def chain_tree(n: int) -> np.ndarray:
    """parent[i] = i - 1: a single path (the causal special case)."""
    return np.arange(-1, n - 1, dtype=np.int32)


# --------------------------------------------------------------------------
# workloads
# --------------------------------------------------------------------------


@dataclass
class Workload:
    name: str
    dtype: str                # "f32" | "bf16"
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    prefix_len: int
    chunk_size: int
    top_k: int
    parent: np.ndarray        # int32 [T]
    score_row: int
    needle_chunks: List[int]
    # fp32 arrays holding values exactly representable in `dtype`
    q: np.ndarray
    k_prefix: np.ndarray
    v_prefix: np.ndarray
    k_tree: np.ndarray
    v_tree: np.ndarray
    draft_k: Optional[np.ndarray] = None
    draft_v: Optional[np.ndarray] = None
    meta: Dict = field(default_factory=dict)

    @property
    def n_tree(self) -> int:
        return int(len(self.parent))

    @property
    def n_chunks(self) -> int:
        return (self.prefix_len + self.chunk_size - 1) // self.chunk_size


def _normal(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    return (rng.standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float32)


def plant_needles(k_prefix: np.ndarray, q: np.ndarray, row: int, chunks, chunk_size: int,
                  shift: float) -> None:
    """Shift every key of the given chunks toward the mean query direction.

    For KV head g the direction is the normalised mean of the G query vectors
    of that group at tree row `row`; `shift` is the length of the added vector.
    In place on k_prefix [Hkv, L, d].
    """
    n_kv, plen, _ = k_prefix.shape
    group = q.shape[1] // n_kv
    for g in range(n_kv):
        u = q[row, g * group:(g + 1) * group, :].astype(np.float64).mean(axis=0)
        nrm = float(np.sqrt((u * u).sum()))
        if nrm == 0.0:
            continue
        u = (u / nrm * shift).astype(np.float32)
        for c in chunks:
            lo, hi = c * chunk_size, min((c + 1) * chunk_size, plen)
            k_prefix[g, lo:hi, :] += u


def make_workload(name: str, *, seed: int, dtype: str, n_q_heads: int, n_kv_heads: int,
                  head_dim: int, prefix_len: int, parent: np.ndarray, chunk_size: int,
                  top_k: int, n_needles: int, score_row: int = 0, value_std: Optional[float] = None,
                  needle_shift_sigmas: float = 3.0, draft_layers: int = 0,
                  draft_kv_heads: Optional[int] = None, draft_head_dim: Optional[int] = None) -> Workload:
    """Draw one layer's inputs.  value_std None means 1/sqrt(head_dim)."""
    rng = np.random.default_rng(seed)
    std = (1.0 / np.sqrt(head_dim)) if value_std is None else float(value_std)
    n_tree = len(parent)
    q = _normal(rng, (n_tree, n_q_heads, head_dim), std)
    k_prefix = _normal(rng, (n_kv_heads, prefix_len, head_dim), std)
    v_prefix = _normal(rng, (n_kv_heads, prefix_len, head_dim), std)
    k_tree = _normal(rng, (n_kv_heads, n_tree, head_dim), std)
    v_tree = _normal(rng, (n_kv_heads, n_tree, head_dim), std)
    n_chunks = (prefix_len + chunk_size - 1) // chunk_size
    full_chunks = prefix_len // chunk_size          # needles never sit in a ragged tail chunk
    needles: List[int] = []
    n_needles = min(n_needles, full_chunks)
    if n_needles > 0:
        needles = sorted(int(c) for c in rng.choice(full_chunks, size=n_needles, replace=False))
        # queries are quantised first so the direction is the one both sides see
        qq = quantize(q, dtype)
        plant_needles(k_prefix, qq, score_row, needles, chunk_size, needle_shift_sigmas * std)
    wl = Workload(
        name=name, dtype=dtype, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, head_dim=head_dim,
        prefix_len=prefix_len, chunk_size=chunk_size, top_k=top_k,
        parent=np.asarray(parent, dtype=np.int32), score_row=score_row, needle_chunks=needles,
        q=quantize(q, dtype), k_prefix=quantize(k_prefix, dtype), v_prefix=quantize(v_prefix, dtype),
        k_tree=quantize(k_tree, dtype), v_tree=quantize(v_tree, dtype),
        meta={"seed": seed, "value_std": std, "n_chunks": n_chunks},
    )
    if draft_layers > 0:
        hd = draft_kv_heads or n_kv_heads
        dd = draft_head_dim or head_dim
        wl.draft_k = quantize(_normal(rng, (draft_layers, hd, prefix_len, dd), std), dtype)
        wl.draft_v = quantize(_normal(rng, (draft_layers, hd, prefix_len, dd), std), dtype)
    return wl


def config_seed(config: int, item: int = 0) -> int:
    return 1000 * config + item


def config_tree(config: int, variant: str = "") -> np.ndarray:
    """The draft tree of a numbered configuration (seeded, layer-independent)."""
    rng = np.random.default_rng(config_seed(config, 999))
    if config == 1:
        return random_parent_tree(8, 4, rng)
    if config in (2, 3, 4):
        # one 60-node tree shape for all Llama-shaped configurations
        return eagle_style_tree(60, 6, np.random.default_rng(config_seed(2, 999)))
    if config == 5:
        if variant == "chain":
            return chain_tree(16)
        return wide_tree(128, 4, rng)
    raise ValueError(config)


def config_workload(config: int, *, item: int = 0, variant: str = "", sharp: bool = False,
                    prefix_len: Optional[int] = None) -> Workload:
    """The five numbered configurations (one layer each; `item` picks the layer).

    1  toy: fp32, Hq=4, Hkv=1, d=64, L=512, T=8 random tree, B=32, k=4, 2 needles
    2  bf16, Hq=32, Hkv=8, d=128, L=2048, 60-node tree, B=32, k=32, 4 needles
    3  as 2 at L=8192, plus a 1-layer draft cache of 8 KV heads to gather from
    4  as 2 at L=16384 (32 layers = items 0..31), 8 needles
    5  stress: L=32768-37, B=64, k=16; variant "wide" (128 nodes) or "chain" (16)
    `sharp` draws unit-variance values so the softmax is far from uniform.
    """
    std = 1.0 if sharp else None
    seed = config_seed(config, item) + (500 if sharp else 0)
    if config == 1:
        return make_workload("toy", seed=seed, dtype="f32", n_q_heads=4, n_kv_heads=1, head_dim=64,
                             prefix_len=prefix_len or 512, parent=config_tree(1), chunk_size=32,
                             top_k=4, n_needles=2, value_std=std)
    if config in (2, 3, 4):
        plen = prefix_len or {2: 2048, 3: 8192, 4: 16384}[config]
        return make_workload(f"llama8b_L{plen}", seed=seed, dtype="bf16", n_q_heads=32, n_kv_heads=8,
                             head_dim=128, prefix_len=plen, parent=config_tree(config), chunk_size=32,
                             top_k=32, n_needles={2: 4, 3: 4, 4: 8}[config], value_std=std,
                             draft_layers=1 if config == 3 else 0)
    if config == 5:
        variant = variant or "wide"
        plen = prefix_len or (32768 - 37)
        return make_workload(f"stress_{variant}", seed=seed + (1 if variant == "chain" else 0),
                             dtype="bf16", n_q_heads=32, n_kv_heads=8, head_dim=128, prefix_len=plen,
                             parent=config_tree(5, variant), chunk_size=64, top_k=16, n_needles=4,
                             value_std=std)
    raise ValueError(config)
