"""CPU ORACLE (test infrastructure only) -- tree metadata straight from the paper's definitions.

Everything here is integer work on small trees and is written with plain Python loops so it can
be checked against the paper by eye.  Citations name the paper's sections/equations.
"""
from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np

INT32_MAX = 2**31 - 1


def _children(parent) -> (List[List[int]], List[int]):
    n = len(parent)
    kids: List[List[int]] = [[] for _ in range(n)]
    roots: List[int] = []
    for i in range(n):                       # ascending id => siblings keep input order
        p = int(parent[i])
        if p < 0:
            roots.append(i)
        else:
            kids[p].append(i)
    return kids, roots


def dfs_meta(parent, seg_len, trained=None, root_pos_offset=None) -> Dict[str, object]:
    """DFS pre-order serialisation and per-node / per-token metadata.

    Eq. 8 (X_DFS): a node's tokens, then each child's serialisation in child order.
    Section "Derivation": K = number of root-to-leaf paths (one per leaf), g_n = number of paths
    through node n.  Eq. 9: pos(t) = total length of strict ancestors + offset within the node
    (roots start at root_pos_offset, eq. pos_offset_child).  Eq. 4: weight = g_t / K, zero for
    tokens of untrained (input) nodes (Fig. 1 caption: only model output is trained).

    All per-node outputs are indexed by DFS rank (position of the node in pre-order).
    """
    parent = [int(x) for x in parent]
    seg_len = [int(x) for x in seg_len]
    n = len(parent)
    trained = [1] * n if trained is None else [int(x) for x in trained]
    kids, roots = _children(parent)
    if root_pos_offset is None:
        root_pos_offset = [0] * len(roots)
    root_pos_offset = [int(x) for x in root_pos_offset]

    order: List[int] = []                    # order[rank] = input id

    def visit(i: int) -> None:
        order.append(i)
        for c in kids[i]:
            visit(c)

    import sys
    sys.setrecursionlimit(max(10000, 4 * n + 100))
    for r in roots:
        visit(r)
    assert len(order) == n, "parent array is not a forest"
    rank = [0] * n
    for rk, i in enumerate(order):
        rank[i] = rk

    node_start = [0] * n
    node_end = [0] * n
    pos = 0
    for rk, i in enumerate(order):
        node_start[rk] = pos
        pos += seg_len[i]
        node_end[rk] = pos
    n_tokens = pos

    # leaves under each node; subtree end = end of the last descendant in pre-order
    def leaves(i: int) -> int:
        return 1 if not kids[i] else sum(leaves(c) for c in kids[i])

    def last_desc(i: int) -> int:
        return i if not kids[i] else last_desc(kids[i][-1])

    node_g = [leaves(order[rk]) for rk in range(n)]
    K = sum(leaves(r) for r in roots)
    subtree_end = [node_end[rank[last_desc(order[rk])]] for rk in range(n)]
    node_parent = [-1 if parent[order[rk]] < 0 else rank[parent[order[rk]]] for rk in range(n)]

    # Eq. 9 by its literal statement: sum over strict ancestors
    node_pos0 = [0] * n
    for rk in range(n):
        i = order[rk]
        total = 0
        a = parent[i]
        top = i
        while a >= 0:
            total += seg_len[a]
            top = a
            a = parent[a]
        node_pos0[rk] = total + root_pos_offset[roots.index(top)]

    tok_node = np.zeros(n_tokens, dtype=np.int32)
    tok_pos = np.zeros(n_tokens, dtype=np.int32)
    tok_pred = np.zeros(n_tokens, dtype=np.int32)
    tok_weight = np.zeros(n_tokens, dtype=np.float32)
    for rk in range(n):
        i = order[rk]
        # the token whose logits predict this node's first token: last token of the nearest
        # ancestor that holds any token; none for a branch that starts here
        a = parent[i]
        while a >= 0 and seg_len[a] == 0:
            a = parent[a]
        pred0 = -1 if a < 0 else node_end[rank[a]] - 1
        w = np.float32(trained[i]) * (np.float32(node_g[rk]) / np.float32(K))
        for j in range(seg_len[i]):
            t = node_start[rk] + j
            tok_node[t] = rk
            tok_pos[t] = node_pos0[rk] + j
            tok_pred[t] = pred0 if j == 0 else t - 1
            tok_weight[t] = w

    return dict(
        n_nodes=n, n_tokens=n_tokens, K=K,
        dfs_order=np.asarray(order, dtype=np.int32),
        node_start=np.asarray(node_start, dtype=np.int32),
        node_end=np.asarray(node_end, dtype=np.int32),
        subtree_end=np.asarray(subtree_end, dtype=np.int32),
        node_g=np.asarray(node_g, dtype=np.int32),
        node_parent=np.asarray(node_parent, dtype=np.int32),
        node_pos0=np.asarray(node_pos0, dtype=np.int32),
        tok_node=tok_node, tok_pos=tok_pos, tok_pred=tok_pred, tok_weight=tok_weight,
        tok_trained=np.asarray([trained[order[rk]] for rk in tok_node], dtype=np.uint8),
    )


def paths(meta) -> List[np.ndarray]:
    """Token index list of every root-to-leaf branch (one per leaf, in DFS order of the leaves):
    the concatenation of the token ranges of the nodes on the path ("Derivation": each path spells
    a trajectory by concatenating its nodes' segments)."""
    n = meta["n_nodes"]
    par = meta["node_parent"]
    has_child = np.zeros(n, dtype=bool)
    for rk in range(n):
        if par[rk] >= 0:
            has_child[par[rk]] = True
    out = []
    for rk in range(n):
        if has_child[rk]:
            continue
        chain = []
        a = rk
        while a >= 0:
            chain.append(a)
            a = int(par[a])
        chain.reverse()
        idx = [np.arange(meta["node_start"][a], meta["node_end"][a], dtype=np.int32) for a in chain]
        out.append(np.concatenate(idx) if idx else np.zeros(0, dtype=np.int32))
    return out


def row_branch(meta, t: int) -> np.ndarray:
    """Tokens of the root-to-t sequence (t last): ancestor nodes in full, own node up to t."""
    rk = int(meta["tok_node"][t])
    par = meta["node_parent"]
    chain = []
    a = int(par[rk])
    while a >= 0:
        chain.append(a)
        a = int(par[a])
    chain.reverse()
    idx = [np.arange(meta["node_start"][a], meta["node_end"][a], dtype=np.int32) for a in chain]
    idx.append(np.arange(meta["node_start"][rk], t + 1, dtype=np.int32))
    return np.concatenate(idx)


def kend(meta, n_prefix: int = 0, prefix_visible=None) -> np.ndarray:
    """Per-key upper visibility bound on the unified key axis [prefix ; own]:
    key j is visible to query i (global index i + n_prefix) iff j <= i + n_prefix < kend[j].
    Own keys: n_prefix + end of the key's node's subtree.  Prefix keys (Appendix "Ancestor-Aware
    Attention Bias"): ancestors are visible to every query, non-ancestors to none."""
    own = meta["subtree_end"][meta["tok_node"]].astype(np.int64) + n_prefix
    pre = np.full(n_prefix, INT32_MAX, dtype=np.int64)
    if prefix_visible is not None:
        pre = np.where(np.asarray(prefix_visible) != 0, INT32_MAX, 0).astype(np.int64)
    return np.concatenate([pre, own]).astype(np.int32)


def tile_minmax(kend_arr, n_prefix: int, tile_n: int):
    """min/max of kend over key tiles; prefix and own regions are tiled separately, each from its
    own first key."""
    mins, maxs = [], []
    for lo, hi in ((0, n_prefix), (n_prefix, len(kend_arr))):
        for s in range(lo, hi, tile_n):
            blk = kend_arr[s:min(s + tile_n, hi)]
            mins.append(int(blk.min()))
            maxs.append(int(blk.max()))
    return np.asarray(mins, dtype=np.int32), np.asarray(maxs, dtype=np.int32)


# ---- three statements of the mask (all N x N bool, tiny N only) ---------------------------------

def mask_from_kend(kend_arr, n_prefix: int = 0) -> np.ndarray:
    nk = len(kend_arr)
    nq = nk - n_prefix
    m = np.zeros((nq, nk), dtype=bool)
    for i in range(nq):
        for j in range(nk):
            m[i, j] = (j <= i + n_prefix) and (i + n_prefix < kend_arr[j])
    return m


def mask_common_path(meta) -> np.ndarray:
    """Section "Attention Mask": i attends j iff j <= i and the nodes of i and j lie on a common
    root-to-leaf path."""
    n = meta["n_tokens"]
    node_sets = []
    par = meta["node_parent"]
    nn = meta["n_nodes"]
    has_child = [False] * nn
    for rk in range(nn):
        if par[rk] >= 0:
            has_child[par[rk]] = True
    for rk in range(nn):
        if not has_child[rk]:
            s = set()
            a = rk
            while a >= 0:
                s.add(a)
                a = int(par[a])
            node_sets.append(s)
    m = np.zeros((n, n), dtype=bool)
    tn = meta["tok_node"]
    for i in range(n):
        for j in range(i + 1):
            m[i, j] = any((int(tn[i]) in s) and (int(tn[j]) in s) for s in node_sets)
    return m


def mask_chunks(meta) -> np.ndarray:
    """Appendix "Tree Attention Mask via FlashMask": a token has full access to the chunk of every
    strict ancestor of its node and causal access inside its own chunk.  Stated at node level first
    (which chunks a chunk may look at), then expanded to tokens."""
    nn, n = meta["n_nodes"], meta["n_tokens"]
    par = np.asarray(meta["node_parent"])
    tn = np.asarray(meta["tok_node"])
    # strict_anc[c, a]: a is a strict ancestor of c (nodes are in pre-order, so parents come first)
    strict_anc = np.zeros((nn, nn), dtype=bool)
    for c in range(nn):
        if par[c] >= 0:
            strict_anc[c] = strict_anc[par[c]]
            strict_anc[c, par[c]] = True
    tok = np.arange(n)
    ancestor_chunk = strict_anc[tn[:, None], tn[None, :]]                       # all of an ancestor's tokens
    own_chunk_causal = (tn[:, None] == tn[None, :]) & (tok[None, :] <= tok[:, None])
    return ancestor_chunk | own_chunk_causal


def por(n_tree: int, n_base: int) -> float:
    """Potential Overlap Ratio, Eq. 12."""
    return 1.0 - n_tree / n_base


WEIGHT_PATH_SUM, WEIGHT_UNIFORM, WEIGHT_PATH_TOKEN_MEAN = 0, 1, 2


def path_weights(meta, scheme: int = WEIGHT_PATH_SUM, path_weight=None, advantage=None) -> np.ndarray:
    """General per-token loss weights ("Derivation", last paragraph): with path weights w_k a token's
    weight is the sum of w_k over the root-to-leaf paths that contain it, lambda_t = sum_{k: t in p_k} w_k;
    untrained tokens get 0 (only model output is trained, Fig. 1); a per-token advantage (policy-gradient
    objective, l_t = -A_t log p) multiplies in.  Written as the definition: one pass over every path.

    scheme WEIGHT_PATH_SUM         w_k = path_weight[k], paths in DFS order of their leaves
           WEIGHT_UNIFORM          lambda_t = 1 for every unique token (the paper's example of another objective)
           WEIGHT_PATH_TOKEN_MEAN  w_k = 1 / (K * number of trained tokens on path k): every branch's loss is
                                   its token mean, branches averaged (w_k = 0 for a branch without trained tokens)
    Arithmetic: sums in fp64, one rounding to fp32, then the fp32 product with the advantage."""
    n = meta["n_tokens"]
    trained = np.asarray(meta["tok_trained"]) != 0
    pl = paths(meta)
    K = len(pl)
    if scheme == WEIGHT_UNIFORM:
        lam = np.ones(n, dtype=np.float64)
    else:
        if scheme == WEIGHT_PATH_SUM:
            w = np.asarray(path_weight, dtype=np.float32).astype(np.float64)
            assert len(w) == K
        elif scheme == WEIGHT_PATH_TOKEN_MEAN:
            w = np.zeros(K)
            for k, p in enumerate(pl):
                cnt = int(trained[p].sum())
                w[k] = 1.0 / (float(K) * cnt) if cnt else 0.0
        else:
            raise ValueError("unknown scheme")
        lam = np.zeros(n, dtype=np.float64)
        for k, p in enumerate(pl):
            for t in p:
                lam[t] += w[k]
    lam = np.where(trained, lam, 0.0).astype(np.float32)
    if advantage is not None:
        lam = lam * np.asarray(advantage, dtype=np.float32)
    return lam.astype(np.float32)
