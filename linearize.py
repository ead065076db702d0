"""Linearised per-branch layout of a tree: the baseline the paper compares against (Section
"Derivation", X_base / Eq. 7: every root-to-leaf path written out in full, shared prefixes
repeated; Section "Evaluation Setups": linearised branches + sequence packing).

Benchmark helper (not part of the library): bench.py uses it to run the *same* library on the K-chain forest, so that the only
difference from the tree run is the redundancy."""
from __future__ import annotations

import numpy as np

from paper_2511_00413_amd import TreeMeta


def branch_token_lists(meta: TreeMeta):
    """DFS token indices of every root-to-leaf path (leaves in DFS order)."""
    n = meta.n_nodes
    has_child = np.zeros(n, dtype=bool)
    has_child[meta.node_parent[meta.node_parent >= 0]] = True
    out = []
    for leaf in np.nonzero(~has_child)[0]:
        chain = []
        a = int(leaf)
        while a >= 0:
            chain.append(a)
            a = int(meta.node_parent[a])
        chain.reverse()
        out.append(np.concatenate([np.arange(meta.node_start[c], meta.node_end[c], dtype=np.int64)
                                   for c in chain]))
    return out


def linearized_forest(meta: TreeMeta):
    """Returns (gather_index [N_lin], parent [K], seg_len [K]): gathering the tree's tokens with
    gather_index gives the packed forest of K independent chains."""
    paths = branch_token_lists(meta)
    idx = np.concatenate(paths) if paths else np.zeros(0, dtype=np.int64)
    parent = np.full(len(paths), -1, dtype=np.int32)
    seg = np.asarray([len(p) for p in paths], dtype=np.int32)
    return idx, parent, seg


def visible_pairs(meta: TreeMeta) -> int:
    """Number of (query, key) pairs the mask lets through: key j is seen by kend[j] - j queries."""
    P = meta.n_prefix
    own = meta.kend[P:].astype(np.int64) - np.arange(P, P + meta.n_tokens, dtype=np.int64)
    pre = np.where(meta.kend[:P] > 0, meta.n_tokens, 0).astype(np.int64)
    return int(own.sum() + pre.sum())
