"""Oracle for tree partitioning and partition-boundary ("gateway") bookkeeping.

TEST INFRASTRUCTURE ONLY: plain Python, small trees, no relation to the HIP library's code.

What is fixed by the paper and what is not:

* Section "Redundancy-Free Tree Partitioning", paragraph "Partitioning": a partition is a connected
  subtree, cuts fall on node boundaries, a partition holds at most C tokens, the partitions form a
  tree (one parent partition each) and the goal is as few partitions as possible.  The paper hands
  that optimisation to a bin-packing solver; which feasible assignment comes out is NOT unique, so
  `check_partitions` states what every valid answer satisfies and `greedy_partitions` is one
  deterministic stand-in whose rule is written out below (and is what the library must reproduce
  node for node).
* Appendix "Zero-Overhead Partition Boundaries": given the assignment, everything at a boundary is
  determined: the cached slice (the parent partition's own cache followed by its own DFS sequence
  up to the end of the cut node n_c), the ancestor-aware bias (visible = tokens of the nodes on the
  path from the parent partition's root to n_c, plus what was visible in the parent's own cache)
  and the position offset (parent's offset + depth-based position of n_c's first token inside the
  parent + |T_nc|).  `gateways` follows those three definitions literally.

Reading taken where the appendix is loose: it calls the parent's own cached part "fully visible,
already ancestor-filtered".  A cached slice physically still contains the masked sibling tokens, so
the flags of the parent's slice are carried over unchanged (a masked token stays masked for every
descendant partition); otherwise a grandchild partition would attend to a great-uncle's tokens and
the per-branch equivalence of Eq. 6 would break.
"""
from typing import Dict, List, Sequence

import numpy as np


def _kids(parent: Sequence[int]):
    kids = [[] for _ in parent]
    roots = []
    for i, p in enumerate(parent):
        (roots if p < 0 else kids[p]).append(i)          # ascending input id
    return kids, roots


def greedy_partitions(parent: Sequence[int], seg_len: Sequence[int], cap: int) -> List[List[int]]:
    """Stand-in packer.  Rule: partitions are opened in first-in-first-out order of their root
    nodes (the tree's roots first, in ascending id).  A partition takes its root unconditionally,
    then walks depth-first, children in ascending id: a child joins if the partition's running
    token count plus the child's own length stays within `cap`; otherwise the edge to it is cut and
    the child is queued as the root of a later partition.  The running count includes everything
    added so far, also below earlier siblings.  Returns node lists in the partition's DFS order."""
    kids, roots = _kids(parent)
    pending = list(roots)
    parts: List[List[int]] = []

    def grow(part: List[int], size: int, node: int) -> int:
        part.append(node)
        size += int(seg_len[node])
        for c in kids[node]:
            if size + int(seg_len[c]) <= cap:
                size = grow(part, size, c)
            else:
                pending.append(c)
        return size

    while pending:
        part: List[int] = []
        grow(part, 0, pending.pop(0))
        parts.append(part)
    return parts


def check_partitions(parent: Sequence[int], seg_len: Sequence[int], cap: int, parts: List[List[int]]) -> None:
    """Raises AssertionError unless `parts` is a valid partitioning in the sense of Section
    "Redundancy-Free Tree Partitioning": every node in exactly one partition; each partition a
    connected subtree listed root first with every other node after its parent; at most `cap`
    tokens unless it is a single node that is longer than `cap` by itself (a node cannot be split);
    partitions listed parents first (the partition of a root's parent node comes earlier)."""
    n = len(parent)
    seen = [-1] * n
    for pi, part in enumerate(parts):
        assert len(part) > 0, "empty partition"
        for nid in part:
            assert 0 <= nid < n and seen[nid] < 0, f"node {nid} assigned twice or out of range"
            seen[nid] = pi
    assert all(s >= 0 for s in seen), "node without a partition"
    for pi, part in enumerate(parts):
        where = {nid: k for k, nid in enumerate(part)}
        root = part[0]
        for nid in part[1:]:
            p = parent[nid]
            assert p in where and where[p] < where[nid], f"partition {pi} is not a connected subtree at node {nid}"
        p = parent[root]
        assert p < 0 or seen[p] < pi, f"partition {pi} comes before the partition of its root's parent"
        tokens = sum(int(seg_len[nid]) for nid in part)
        assert tokens <= cap or len(part) == 1, f"partition {pi} holds {tokens} > {cap} tokens"


def min_partitions_bruteforce(parent: Sequence[int], seg_len: Sequence[int], cap: int) -> int:
    """Fewest partitions over ALL valid cut sets (each non-root edge is cut or kept), for tiny
    trees.  Every node must fit (`seg_len <= cap`)."""
    n = len(parent)
    edges = [i for i in range(n) if parent[i] >= 0]
    n_roots = n - len(edges)
    best = n
    for bits in range(1 << len(edges)):
        cut = {e for k, e in enumerate(edges) if bits >> k & 1}
        comp_tokens: Dict[int, int] = {}
        for i in range(n):
            top = i
            while parent[top] >= 0 and top not in cut:
                top = parent[top]
            comp_tokens[top] = comp_tokens.get(top, 0) + int(seg_len[i])
        if all(t <= cap for t in comp_tokens.values()):
            best = min(best, n_roots + len(cut))
    return best


def gateways(parent: Sequence[int], seg_len: Sequence[int], parts: List[List[int]]) -> List[Dict[str, object]]:
    """Boundary bookkeeping for a valid partitioning, partitions in the given (parents first) order.

    Token indices are positions in the WHOLE tree's DFS serialisation (Eq. 8, children in ascending
    id).  Per partition:
      root, parent_part, cut_node   cut_node = parent of the root (n_c), -1 for a top partition
      own_tok        whole-tree indices of the partition's tokens, in the partition's DFS order
      prefix_tok     whole-tree indices of the cached slice, in slice order
      prefix_visible 1 where the ancestor-aware bias is 0, 0 where it is -inf
      pos_offset     depth-based position of the partition's first token
    """
    kids, roots = _kids(parent)
    n = len(parent)
    # whole-tree DFS token range of every node
    start = [0] * n
    t = 0
    stack = list(reversed(roots))
    while stack:
        i = stack.pop()
        start[i] = t
        t += int(seg_len[i])
        stack.extend(reversed(kids[i]))
    node_tok = lambda i: list(range(start[i], start[i] + int(seg_len[i])))

    part_of = {}
    for pi, part in enumerate(parts):
        for nid in part:
            part_of[nid] = pi

    out: List[Dict[str, object]] = []
    for pi, part in enumerate(parts):
        root = part[0]
        n_c = int(parent[root])
        own = [tok for nid in part for tok in node_tok(nid)]
        if n_c < 0:
            rec = dict(root=root, parent_part=-1, cut_node=-1, prefix_tok=[], prefix_visible=[], pos_offset=0)
        else:
            P = out[part_of[n_c]]
            p_nodes = parts[part_of[n_c]]
            # token range [s, e) of each node in P's own DFS sequence
            s_loc, e_loc, run = {}, {}, 0
            for nid in p_nodes:
                s_loc[nid] = run
                run += int(seg_len[nid])
                e_loc[nid] = run
            # path(P.root, n_c): parent chain of n_c inside P
            path = [n_c]
            while path[-1] != P["root"]:
                path.append(int(parent[path[-1]]))
            anc = set()
            for nid in path:
                anc.update(range(s_loc[nid], e_loc[nid]))
            past_len = len(P["prefix_tok"])
            e_nc = e_loc[n_c]
            prefix_tok = list(P["prefix_tok"]) + list(P["own_tok"][:e_nc])
            prefix_visible = list(P["prefix_visible"]) + [1 if j in anc else 0 for j in range(e_nc)]
            assert len(prefix_tok) == past_len + e_nc
            # depth-based position of n_c's first token within P = lengths of its strict ancestors in P
            pos_nc = sum(int(seg_len[nid]) for nid in path[1:])
            rec = dict(root=root, parent_part=part_of[n_c], cut_node=n_c, prefix_tok=prefix_tok,
                       prefix_visible=prefix_visible, pos_offset=int(P["pos_offset"]) + pos_nc + int(seg_len[n_c]))
        rec["own_tok"] = own
        rec["nodes"] = list(part)
        out.append(rec)
    for rec in out:
        for key in ("own_tok", "prefix_tok"):
            rec[key] = np.asarray(rec[key], dtype=np.int32)
        rec["prefix_visible"] = np.asarray(rec["prefix_visible"], dtype=np.uint8)
    return out
