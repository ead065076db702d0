"""Pins for oracle/meta.py: the worked tree, the three statements of the mask on every small tree,
per-path positions, the integer form of the loss identity, printed paper numbers."""
import itertools

import numpy as np
import pytest

import workloads as W
from oracle import meta as M
from tt_testutil import read_golden


def test_worked_tree_golden():
    g = read_golden("worked_tree.txt")
    m = M.dfs_meta(g["parent"], g["seg_len"])
    assert list(m["dfs_order"]) == [0, 1, 2, 3, 4]
    for key in ("node_start", "node_end", "subtree_end", "node_pos0", "node_g"):
        assert list(m[key]) == g[key], key
    assert m["K"] == g["K"][0]
    w = m["tok_weight"]
    for rk in range(5):
        seg = w[m["node_start"][rk]:m["node_end"][rk]]
        assert np.all(seg == np.float32(g["weight"][rk]))
    pl = M.paths(m)
    assert [len(p) for p in pl] == g["path_len"]
    assert m["n_tokens"] == g["n_tree"][0] and sum(len(p) for p in pl) == g["n_base"][0]
    ke = M.kend(m)
    assert int((ke - np.arange(m["n_tokens"])).sum()) == g["pairs_tree"][0]
    assert sum(len(p) * (len(p) + 1) // 2 for p in pl) == g["pairs_base"][0]
    assert abs(M.por(g["n_tree"][0], g["n_base"][0]) - (1 - 240 / 416)) < 1e-15
    # config 1 of the workload module is this tree
    t = W.tree_cfg1()
    assert list(t.parent) == g["parent"] and list(t.seg_len) == g["seg_len"]


def test_six_token_golden():
    g = read_golden("six_token_tree.txt")
    m = M.dfs_meta(g["parent"], g["seg_len"])
    assert list(M.kend(m)) == g["kend"]
    assert list(m["tok_pos"]) == g["pos"]
    mask = M.mask_from_kend(M.kend(m))
    for i in range(6):
        assert list(np.nonzero(mask[i])[0]) == g[f"row{i}"]
    # n3 (token 3) and n2 (token 5) mutually blocked
    assert not mask[5, 3] and not mask[3, 5]
    assert np.array_equal(mask, M.mask_common_path(m))
    assert np.array_equal(mask, M.mask_chunks(m))


def test_paper_numbers():
    g = read_golden("paper_numbers.txt")
    assert abs(M.por(g["por_n_tree"][0], g["por_n_base"][0]) - g["por_value"][0]) < 5e-4


def _check_tree(parent, seg):
    m = M.dfs_meta(parent, seg)
    n = m["n_tokens"]
    ke = M.kend(m)
    a = M.mask_from_kend(ke)
    b = M.mask_common_path(m)
    c = M.mask_chunks(m)
    assert np.array_equal(a, b), (parent, seg)
    assert np.array_equal(a, c), (parent, seg)
    assert all(a[i, i] for i in range(n))            # no empty row
    pl = M.paths(m)
    assert len(pl) == m["K"]
    roots = [i for i, p in enumerate(parent) if p < 0]
    for p in pl:
        # positions along a path are 0..L-1 (Eq. 9) and every path row sees exactly its own prefix
        assert list(m["tok_pos"][p]) == list(range(len(p)))
        for r, t in enumerate(p):
            assert list(np.nonzero(a[t])[0]) == sorted(p[:r + 1])
            assert m["tok_pred"][t] == (p[r - 1] if r > 0 else -1)
    # integer loss identity (Eq. 2): tokens counted over paths == sum of g over tokens
    g_tok = m["node_g"][m["tok_node"]]
    assert sum(len(p) for p in pl) == int(g_tok.sum())
    # every token lies on g paths
    cnt = np.zeros(n, dtype=np.int64)
    for p in pl:
        cnt[p] += 1
    assert np.array_equal(cnt, g_tok)
    # DFS: nodes' ranges tile [0, n) in order, subtree range is contiguous and nested
    assert m["node_start"][0] == 0 and m["node_end"][-1] == n
    assert np.all(m["node_start"][1:] == m["node_end"][:-1])
    for rk in range(m["n_nodes"]):
        pr = m["node_parent"][rk]
        if pr >= 0:
            assert pr < rk and m["subtree_end"][rk] <= m["subtree_end"][pr]


def test_masks_exhaustive_small_trees():
    count = 0
    for n in (1, 2, 3, 4):
        for parent in W.all_parent_arrays(n):
            for seg in itertools.product((1, 2, 3), repeat=n):
                _check_tree(parent, list(seg))
                count += 1
    for parent in W.all_parent_arrays(5):
        for seg in itertools.product((1, 2), repeat=5):
            _check_tree(parent, list(seg))
            count += 1
    assert count > 5000


def test_zero_length_segments_and_shuffled_ids():
    for seed in range(40):
        t = W.random_tree(seed, n_nodes=2 + seed % 9, lo=1, hi=5, n_roots=1 + seed % 3,
                          shuffle=True, p_zero=0.25)
        m = M.dfs_meta(t.parent, t.seg_len, t.trained)
        n = m["n_tokens"]
        if n == 0:
            continue
        a = M.mask_from_kend(M.kend(m))
        assert np.array_equal(a, M.mask_common_path(m))
        assert np.array_equal(a, M.mask_chunks(m))
        pl = M.paths(m)
        assert len(pl) == m["K"]
        for p in pl:
            assert list(m["tok_pos"][p]) == list(range(len(p)))
            for r, tk in enumerate(p):
                assert m["tok_pred"][tk] == (p[r - 1] if r > 0 else -1)
        # weight = trained * g / K, read through dfs_order
        for rk in range(m["n_nodes"]):
            w = np.float32(t.trained[m["dfs_order"][rk]]) * (np.float32(m["node_g"][rk]) / np.float32(m["K"]))
            assert np.all(m["tok_weight"][m["node_start"][rk]:m["node_end"][rk]] == w)


def test_chain_and_forest_reduce_to_causal():
    m = M.dfs_meta(*[getattr(W.chain_tree([3, 4, 2]), k) for k in ("parent", "seg_len")])
    assert np.array_equal(M.mask_from_kend(M.kend(m)), np.tril(np.ones((9, 9), dtype=bool)))
    assert list(m["tok_pos"]) == list(range(9)) and m["K"] == 1
    f = W.forest_of_chains([3, 2, 4])
    m = M.dfs_meta(f.parent, f.seg_len)
    want = np.zeros((9, 9), dtype=bool)
    for lo, hi in ((0, 3), (3, 5), (5, 9)):
        want[lo:hi, lo:hi] = np.tril(np.ones((hi - lo, hi - lo), dtype=bool))
    assert np.array_equal(M.mask_from_kend(M.kend(m)), want)
    assert list(m["tok_pos"]) == [0, 1, 2, 0, 1, 0, 1, 2, 3] and m["K"] == 3


def test_partition_prefix_examples():
    # Appendix "Ancestor-Aware Attention Bias": parent partition DFS is [a, b, c1, c2], the cut node
    # is c2; the gateway slice holds c1's tokens, which the child partition must not see.
    la, lb, lc1, lc2 = 3, 2, 4, 2
    vis = np.array([1] * la + [1] * lb + [0] * lc1 + [1] * lc2, dtype=np.uint8)
    child = W.chain_tree([3])
    m = M.dfs_meta(child.parent, child.seg_len, root_pos_offset=[la + lb + lc2])
    P = len(vis)
    ke = M.kend(m, P, vis)
    mask = M.mask_from_kend(ke, P)
    for i in range(3):
        assert list(np.nonzero(mask[i])[0]) == [0, 1, 2, 3, 4, 9, 10] + list(range(P, P + i + 1))
    # Appendix "Depth-Based Position Offset": pos_offset counts ancestors only, not the sibling c1,
    # so it differs from past_len
    assert list(m["tok_pos"]) == [7, 8, 9] and m["tok_pos"][0] != P
    # whole-tree view gives the same positions for those tokens
    whole = M.dfs_meta([-1, 0, 1, 1, 3], [la, lb, lc1, lc2, 3])
    assert list(whole["tok_pos"][-3:]) == [7, 8, 9]
    # tile summaries: prefix and own regions tiled separately
    mn, mx = M.tile_minmax(ke, P, 4)
    assert len(mn) == 3 + 1
    assert list(mn) == [M.INT32_MAX, 0, 0, P + 3] and list(mx) == [M.INT32_MAX, M.INT32_MAX, M.INT32_MAX, P + 3]


def test_benchmark_tree_sizes():
    # sizes the generators must reproduce (cross-check of the workload recipes)
    want = {1: (5, 240, 3), 2: (30, 16406, 20), 3: (49, 73728, 32), 4: (49, 131091, 8), 5: (73, 400937, 64)}
    for c, (nn, nt, k) in want.items():
        t = W.tree_config(c)
        m = M.dfs_meta(t.parent, t.seg_len, t.trained)
        assert (m["n_nodes"], m["n_tokens"], m["K"]) == (nn, nt, k)
    s = W.step_cfg5()
    assert s.chunk.n_tokens == 32768 and len(s.prefix_visible) == 65536
