"""Pins for oracle/partition.py: the appendix's worked boundary cases, the boundary bookkeeping
against facts of the WHOLE tree that know nothing about partitions (ancestor sets, depth-based
positions, the tree mask), the packer against closed forms and brute force, and planted mistakes
that the validity checker must catch."""
import numpy as np
import pytest

import workloads as W
from oracle import meta as M
from oracle import partition as P


def _whole(parent, seg):
    m = M.dfs_meta(parent, seg)
    rank = {int(nid): rk for rk, nid in enumerate(m["dfs_order"])}
    return m, rank


def test_sibling_in_cached_slice_is_masked():
    """Appendix "Ancestor-Aware Attention Bias": the parent partition's DFS sequence is
    [a, b, c1, c2] with c1, c2 siblings and the cut below c2; the slice holds c1's tokens and the
    child must not see them.  Appendix "Depth-Based Position Offset": the offset counts ancestors
    only, so it differs from the slice length."""
    #          a    b   c1  c2   x (child of c2, own partition)
    parent = [-1,   0,   1,  1,  3]
    seg =    [ 3,   2,   4,  5,  6]
    parts = [[0, 1, 2, 3], [4]]
    P.check_partitions(parent, seg, 14, parts)
    gw = P.gateways(parent, seg, parts)
    top, child = gw
    assert top["parent_part"] == -1 and len(top["prefix_tok"]) == 0 and top["pos_offset"] == 0
    assert child["cut_node"] == 3 and child["parent_part"] == 0
    assert list(child["prefix_tok"]) == list(range(14))                 # a b c1 c2, contiguous here
    assert list(child["prefix_visible"]) == [1] * 3 + [1] * 2 + [0] * 4 + [1] * 5
    assert child["pos_offset"] == 3 + 2 + 5
    assert child["pos_offset"] != len(child["prefix_tok"])
    assert list(child["own_tok"]) == list(range(14, 20))


def test_cut_at_first_sibling_excludes_later_sibling():
    """The slice ends at the end of the cut node: with the cut below c1, c2 is not cached at all,
    and the offset equals the slice length (no sibling in between)."""
    parent = [-1, 0, 1, 1, 2]
    seg = [3, 2, 4, 5, 6]
    parts = [[0, 1, 2, 3], [4]]
    child = P.gateways(parent, seg, parts)[1]
    assert list(child["prefix_tok"]) == list(range(9))
    assert list(child["prefix_visible"]) == [1] * 9
    assert child["pos_offset"] == 9 == len(child["prefix_tok"])
    # whole-tree DFS is a b c1 x c2: x's tokens sit between c1 and c2
    assert list(child["own_tok"]) == list(range(9, 15))


def test_masked_tokens_stay_masked_two_levels_down():
    """A grandchild partition's slice = the child's slice + the child's own prefix; what was masked
    for the child stays masked for the grandchild."""
    #          a   c1  c2   x(c2)  y(x)
    parent = [-1,  0,  0,   2,     3]
    seg =    [ 2,  3,  4,   5,     1]
    parts = [[0, 1, 2], [3], [4]]
    gw = P.gateways(parent, seg, parts)
    assert list(gw[1]["prefix_visible"]) == [1, 1, 0, 0, 0, 1, 1, 1, 1]
    assert list(gw[2]["prefix_visible"]) == [1, 1, 0, 0, 0, 1, 1, 1, 1] + [1] * 5
    assert gw[2]["pos_offset"] == 2 + 4 + 5
    assert gw[2]["parent_part"] == 1


@pytest.mark.parametrize("seed", range(12))
def test_boundaries_agree_with_whole_tree(seed):
    """Against the whole tree, which knows nothing about partitions: the visible part of a slice is
    exactly the ancestor tokens of the partition's root; the offset is the depth-based position
    (Eq. 9) of its first token; every token is owned once; and the partition's combined mask (own
    tree mask behind the biased slice) equals the whole tree's mask on the same (query, key) pairs."""
    tree = W.random_tree(900 + seed, n_nodes=4 + seed, lo=1, hi=9, n_roots=1 + seed % 2, p_zero=0.15)
    parent, seg = list(tree.parent), list(tree.seg_len)
    whole, rank = _whole(parent, seg)
    full_mask = M.mask_common_path(whole)
    cap = 6 + 3 * (seed % 4)
    parts = P.greedy_partitions(parent, seg, cap)
    P.check_partitions(parent, seg, cap, parts)
    gw = P.gateways(parent, seg, parts)
    owned = np.concatenate([g["own_tok"] for g in gw])
    assert sorted(owned.tolist()) == list(range(whole["n_tokens"]))
    for part, g in zip(parts, gw):
        # ancestors of the root through the whole tree's parent chain
        anc_tok = []
        a = parent[g["root"]]
        chain = []
        while a >= 0:
            chain.append(a)
            a = parent[a]
        for a in reversed(chain):
            anc_tok.extend(range(whole["node_start"][rank[a]], whole["node_end"][rank[a]]))
        vis = g["prefix_visible"].astype(bool)
        assert g["prefix_tok"][vis].tolist() == anc_tok
        assert g["pos_offset"] == len(anc_tok) == int(whole["node_pos0"][rank[g["root"]]])
        assert len(set(g["prefix_tok"].tolist())) == len(g["prefix_tok"])
        # the partition as a local tree
        local = {nid: i for i, nid in enumerate(part)}
        lparent = [-1 if nid == part[0] else local[parent[nid]] for nid in part]
        lmeta = M.dfs_meta(lparent, [seg[nid] for nid in part], root_pos_offset=[g["pos_offset"]])
        assert [part[i] for i in lmeta["dfs_order"]] == part            # listed in its own DFS order
        assert np.array_equal(lmeta["tok_pos"], whole["tok_pos"][g["own_tok"]])
        ke = M.kend(lmeta, n_prefix=len(g["prefix_tok"]), prefix_visible=g["prefix_visible"])
        combined = M.mask_from_kend(ke, n_prefix=len(g["prefix_tok"]))
        keys = np.concatenate([g["prefix_tok"], g["own_tok"]]).astype(np.int64)
        assert np.array_equal(combined, full_mask[np.ix_(g["own_tok"], keys)])
        # and nothing outside [slice ; own] is visible to these queries
        other = np.setdiff1d(np.arange(whole["n_tokens"]), keys)
        assert not full_mask[np.ix_(g["own_tok"], other)].any()


def test_packer_closed_forms():
    # a chain of n equal nodes: ceil(n / floor(cap / L)) partitions, cut every m nodes
    n, L = 11, 5
    parent = [-1] + list(range(n - 1))
    seg = [L] * n
    for cap in (5, 9, 10, 14, 15, 27, 55, 60):
        parts = P.greedy_partitions(parent, seg, cap)
        m = cap // L
        assert [len(p) for p in parts] == [m] * (n // m) + ([n % m] if n % m else [])
        assert parts[0] == list(range(min(m, n)))
    # a star: the root takes children in ascending id while they fit, the rest are singletons
    parent = [-1] + [0] * 6
    seg = [4, 3, 3, 9, 3, 1, 2]
    parts = P.greedy_partitions(parent, seg, 12)
    assert parts == [[0, 1, 2, 5], [3], [4], [6]]            # 4+3+3=10, 9 no, 3 no, +1=11, 2 no
    # capacity at least the whole forest: one partition per root
    tree = W.random_tree(5, n_nodes=20, lo=1, hi=9, n_roots=3)
    parts = P.greedy_partitions(list(tree.parent), list(tree.seg_len), sum(tree.seg_len))
    assert len(parts) == 3 and sorted(x for p in parts for x in p) == list(range(20))
    # a node longer than the capacity is a partition by itself
    parts = P.greedy_partitions([-1, 0, 1], [3, 50, 2], 10)
    assert parts == [[0], [1], [2]]
    P.check_partitions([-1, 0, 1], [3, 50, 2], 10, parts)
    # zero-length nodes always fit
    parts = P.greedy_partitions([-1, 0, 0, 1], [10, 0, 0, 0], 10)
    assert parts == [[0, 1, 3, 2]]


@pytest.mark.parametrize("seed", range(10))
def test_packer_valid_and_bounded(seed):
    tree = W.random_tree(300 + seed, n_nodes=9, lo=1, hi=8, shuffle=bool(seed % 2))
    parent, seg = list(tree.parent), list(tree.seg_len)
    cap = max(seg) + seed % 5
    parts = P.greedy_partitions(parent, seg, cap)
    P.check_partitions(parent, seg, cap, parts)
    best = P.min_partitions_bruteforce(parent, seg, cap)
    assert -(-sum(seg) // cap) <= best <= len(parts)


def test_packer_optimal_on_chains():
    for n, cap in ((7, 10), (8, 13), (5, 4)):
        parent = [-1] + list(range(n - 1))
        seg = [4] * n
        assert len(P.greedy_partitions(parent, seg, cap)) == P.min_partitions_bruteforce(parent, seg, cap)


def test_checker_catches_planted_mistakes():
    parent = [-1, 0, 0, 1, 1, 2]
    seg = [4, 4, 4, 4, 4, 4]
    good = [[0, 1, 3], [2, 5], [4]]
    P.check_partitions(parent, seg, 12, good)
    bad = {
        "a node twice": [[0, 1, 3], [2, 5], [4, 3]],
        "a node missing": [[0, 1, 3], [2, 5]],
        "not connected": [[0, 1, 5], [2], [3], [4]],
        "child before parent inside a partition": [[0, 3, 1], [2, 5], [4]],
        "over capacity": [[0, 1, 3, 4], [2, 5]],
        "child partition before its parent": [[2, 5], [0, 1, 3], [4]],
    }
    for what, parts in bad.items():
        with pytest.raises(AssertionError):
            P.check_partitions(parent, seg, 12, parts)
            pytest.fail(what)
