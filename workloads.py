"""Seeded synthetic inputs for the tree-attention hot path.

This module only *draws inputs*: tree shapes (parent array, segment lengths,
trained flags) and tensor values.  It holds none of the method's arithmetic
(no DFS, no masks, no positions, no weights), so both the CPU oracle and the
HIP library can be fed from it without sharing any logic.

The trees stand in for the agentic rollout trees the paper trains on
(Section "Speedup and Correctness on real-world agentic trajectories": sparse,
unbalanced trees with overlap ratios of 28%..89%) and for its synthetic
overlap sweep; neither data set is available, so shapes are imitated.

Tree RNG: splitmix64 (public-domain generator by S. Vigna), so the same draws
can be reproduced in any language.  Tensor values: torch CPU generator.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

_MASK64 = (1 << 64) - 1


class SplitMix64:
    def __init__(self, seed: int):
        self.state = seed & _MASK64

    def u64(self) -> int:
        self.state = (self.state + 0x9E3779B97F4A7C15) & _MASK64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
        return z ^ (z >> 31)

    def randint(self, a: int, b: int) -> int:
        """Uniform-ish integer in [a, b] (plain modulo)."""
        return a + self.u64() % (b - a + 1)

    def unif(self) -> float:
        return (self.u64() >> 11) * (2.0 ** -53)


@dataclass
class Tree:
    """A trajectory tree (or forest) in *input* numbering.

    parent[n] = -1 marks a root; siblings are ordered by ascending node id.
    """
    parent: np.ndarray            # int32 [n_nodes]
    seg_len: np.ndarray           # int32 [n_nodes]
    trained: np.ndarray           # uint8 [n_nodes]
    name: str = ""

    @property
    def n_nodes(self) -> int:
        return int(self.parent.shape[0])

    @property
    def n_tokens(self) -> int:
        return int(self.seg_len.sum())


def _mk(parent, seg_len, trained, name) -> Tree:
    return Tree(np.asarray(parent, dtype=np.int32), np.asarray(seg_len, dtype=np.int32),
                np.asarray(trained, dtype=np.uint8), name)


# --------------------------------------------------------------------------
# The five benchmark configurations
# --------------------------------------------------------------------------

def tree_cfg1() -> Tree:
    """Three-leaf tree with the topology of the paper's Fig. 1/2 (n0 -> {n1 -> {n3, n4}, n2})."""
    #        root  A   A1  A2  B
    parent = [-1, 0, 1, 1, 0]
    seg = [64, 48, 32, 40, 56]
    trained = [0, 1, 0, 1, 0]      # alternate nodes; the root is prompt
    return _mk(parent, seg, trained, "cfg1-worked-tree")


def tree_cfg2(seed: int = 117) -> Tree:
    """Depth-4 random tree, fan-out U{2,3,4}, segments U[128,1024]."""
    rng = SplitMix64(seed)
    parent: List[int] = []
    seg: List[int] = []

    def rec(par: int, level: int) -> None:
        me = len(parent)
        parent.append(par)
        seg.append(rng.randint(128, 1024))
        if level < 4:
            fan = rng.randint(2, 4)
            for _ in range(fan):
                rec(me, level + 1)

    rec(-1, 1)
    trained = [1 if rng.unif() < 0.5 else 0 for _ in parent]
    return _mk(parent, seg, trained, f"cfg2-random-depth4-seed{seed}")


def tree_cfg3() -> Tree:
    """Agentic fan-out: 8K shared prefix -> 16 x (2K -> 2 x 1K)."""
    parent = [-1]
    seg = [8192]
    trained = [0]
    for _ in range(16):
        b = len(parent)
        parent.append(0); seg.append(2048); trained.append(1)
        for _ in range(2):
            parent.append(b); seg.append(1024); trained.append(1)
    return _mk(parent, seg, trained, "cfg3-agentic-fanout")


def tree_cfg4(seed: int = 195) -> Tree:
    """Deep context-management chain: 32-node spine with dead-end side chains."""
    rng = SplitMix64(seed)
    parent: List[int] = []
    seg: List[int] = []
    prev = -1
    for s in range(32):
        me = len(parent)
        parent.append(prev)
        seg.append(rng.randint(1024, 4096))
        if s < 31 and rng.unif() < 0.25:
            cnt = rng.randint(1, 3)
            p = me
            for _ in range(cnt):
                c = len(parent)
                parent.append(p)
                seg.append(rng.randint(1024, 4096))
                p = c
        prev = me
    trained = [n & 1 for n in range(len(parent))]
    return _mk(parent, seg, trained, f"cfg4-deep-chain-seed{seed}")


def tree_cfg5(seed: int = 1) -> Tree:
    """Large two-level fan-out-8 tree (the tree that gets partitioned)."""
    rng = SplitMix64(seed)
    parent = [-1]
    seg = [32768]
    for _ in range(8):
        b = len(parent)
        parent.append(0); seg.append(rng.randint(2048, 8192))
        for _ in range(8):
            parent.append(b); seg.append(rng.randint(2048, 8192))
    trained = [0] + [1] * (len(parent) - 1)
    return _mk(parent, seg, trained, f"cfg5-large-tree-seed{seed}")


@dataclass
class PartitionStep:
    """One partition step: a query chunk (its own small tree) behind a cached prefix."""
    chunk: Tree
    n_prefix: int
    prefix_visible: np.ndarray    # uint8 [n_prefix]; 1 = ancestor of the chunk root
    name: str = ""


def step_cfg5(seed: int = 1, n_chunk: int = 32768, n_prefix: int = 65536,
              variant: str = "b", lo: int = 2048, hi: int = 8192,
              root_visible: int = 32768) -> PartitionStep:
    """Config-5 timed unit: a 32K-token chunk (one node + children, truncated to exactly
    n_chunk tokens) attending to 64K cached prefix keys.  Variant "a": whole prefix visible;
    variant "b": first root_visible keys visible, then alternating visible/masked runs."""
    rng = SplitMix64(seed)
    parent = [-1]
    seg = [rng.randint(lo, hi)]
    total = seg[0]
    while total < n_chunk:
        ln = min(rng.randint(lo, hi), n_chunk - total)
        parent.append(0); seg.append(ln); total += ln
    chunk = _mk(parent, seg, [1] * len(parent), f"cfg5-step-chunk-seed{seed}")
    vis = np.ones(n_prefix, dtype=np.uint8)
    if variant == "b":
        pos = min(root_visible, n_prefix)
        flag = 1
        while pos < n_prefix:
            ln = min(rng.randint(lo, hi), n_prefix - pos)
            vis[pos:pos + ln] = flag
            flag ^= 1
            pos += ln
    return PartitionStep(chunk, n_prefix, vis, f"cfg5-step-{variant}")


@dataclass
class AttnDims:
    hq: int
    hkv: int
    d: int
    dtype: str          # "bf16" | "fp32"
    std: float          # Q/K/V/dO ~ std * N(0,1)
    vocab: int = 0
    logit_std: float = 1.0
    logit_dtype: str = "fp32"


DIMS = {
    1: AttnDims(4, 4, 64, "fp32", 1.0, 1024, 1.0, "fp32"),
    2: AttnDims(32, 8, 128, "bf16", 0.5, 32768, 2.0, "bf16"),
    3: AttnDims(64, 8, 128, "bf16", 0.5, 151936, 2.0, "bf16"),
    4: AttnDims(32, 8, 128, "bf16", 0.5),
    5: AttnDims(64, 8, 128, "bf16", 0.5),
}


def tree_config(cfg: int) -> Tree:
    return {1: tree_cfg1, 2: tree_cfg2, 3: tree_cfg3, 4: tree_cfg4, 5: tree_cfg5}[cfg]()


# --------------------------------------------------------------------------
# Small / exhaustive trees for tests
# --------------------------------------------------------------------------

def all_parent_arrays(n_nodes: int):
    """Every parent array with parent[0] = -1 and parent[i] in [-1, i): all labelled
    increasing forests on n_nodes nodes (covers every rooted ordered tree shape)."""
    def rec(prefix):
        if len(prefix) == n_nodes:
            yield list(prefix)
            return
        i = len(prefix)
        for p in range(-1, i):
            yield from rec(prefix + [p])
    yield from rec([-1])


def random_tree(seed: int, n_nodes: int, lo: int = 1, hi: int = 16, n_roots: int = 1,
                shuffle: bool = True, p_zero: float = 0.0) -> Tree:
    """Random recursive tree/forest; node ids optionally shuffled so that input numbering
    is not DFS order.  Segment lengths U[lo, hi], zero with probability p_zero."""
    rng = SplitMix64(seed)
    parent = []
    for i in range(n_nodes):
        if i < n_roots:
            parent.append(-1)
        else:
            parent.append(rng.randint(0, i - 1))
    seg = [0 if rng.unif() < p_zero else rng.randint(lo, hi) for _ in range(n_nodes)]
    trained = [1 if rng.unif() < 0.5 else 0 for _ in range(n_nodes)]
    if shuffle:
        perm = list(range(n_nodes))
        for i in range(n_nodes - 1, 0, -1):      # Fisher-Yates
            j = rng.randint(0, i)
            perm[i], perm[j] = perm[j], perm[i]
        # perm[old] = new id
        new_parent = [0] * n_nodes
        new_seg = [0] * n_nodes
        new_tr = [0] * n_nodes
        for old in range(n_nodes):
            new = perm[old]
            new_parent[new] = -1 if parent[old] < 0 else perm[parent[old]]
            new_seg[new] = seg[old]
            new_tr[new] = trained[old]
        parent, seg, trained = new_parent, new_seg, new_tr
    return _mk(parent, seg, trained, f"random-seed{seed}-n{n_nodes}")


def chain_tree(lengths) -> Tree:
    n = len(lengths)
    return _mk([-1] + list(range(n - 1)), lengths, [1] * n, "chain")


def forest_of_chains(lengths) -> Tree:
    n = len(lengths)
    return _mk([-1] * n, lengths, [1] * n, "forest-of-chains")


# --------------------------------------------------------------------------
# Tensor values
# --------------------------------------------------------------------------

def _torch():
    import torch
    return torch


def randn(shape, seed: int, std: float = 1.0, dtype: str = "fp32"):
    """CPU torch tensor ~ std*N(0,1); drawn in fp32, then rounded to `dtype`."""
    torch = _torch()
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    x = torch.randn(shape, generator=g, dtype=torch.float32) * std
    if dtype == "bf16":
        x = x.to(torch.bfloat16)
    return x


def attn_inputs(n_q: int, n_k: int, dims: AttnDims, seed: int):
    """Q, dO: [n_q, hq, d]; K, V: [n_k, hkv, d] in the config's dtype (CPU torch tensors).
    Inputs are in DFS token order already (values are i.i.d., so order carries no meaning)."""
    q = randn((n_q, dims.hq, dims.d), seed * 1000 + 1, dims.std, dims.dtype)
    k = randn((n_k, dims.hkv, dims.d), seed * 1000 + 2, dims.std, dims.dtype)
    v = randn((n_k, dims.hkv, dims.d), seed * 1000 + 3, dims.std, dims.dtype)
    do = randn((n_q, dims.hq, dims.d), seed * 1000 + 4, dims.std, dims.dtype)
    return q, k, v, do


def loss_inputs(n_rows: int, vocab: int, seed: int, std: float = 1.0, dtype: str = "fp32"):
    """logits [n_rows, vocab] ~ std*N(0,1) in `dtype`; target ids uniform in [0, vocab)."""
    torch = _torch()
    logits = randn((n_rows, vocab), seed * 1000 + 5, std, dtype)
    g = torch.Generator(device="cpu")
    g.manual_seed(seed * 1000 + 6)
    target = torch.randint(0, vocab, (n_rows,), generator=g, dtype=torch.int32)
    return logits, target
