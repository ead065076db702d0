"""tt_tree_partition_plan (host C++) against the oracle: the same packing node for node, the
boundary bookkeeping and every flattened array bit-exact, plus what holds for any valid answer."""
import numpy as np
import pytest

import paper_2511_00413_amd as T
import workloads as W
from oracle import meta as M
from oracle import partition as P


def _compare(parent, seg, cap):
    parent, seg = [int(x) for x in parent], [int(x) for x in seg]
    got = T.tree_partition_plan(parent, seg, cap)
    parts = P.greedy_partitions(parent, seg, cap)
    P.check_partitions(parent, seg, cap, parts)
    gw = P.gateways(parent, seg, parts)
    assert got.n_parts == len(parts) and got.n_tokens == sum(seg)
    lib_parts = [got.part_nodes[got.part_node_off[p]:got.part_node_off[p + 1]].tolist() for p in range(got.n_parts)]
    assert lib_parts == parts
    P.check_partitions(parent, seg, cap, lib_parts)               # valid whatever the packer
    for p, g in enumerate(gw):
        for nid in parts[p]:
            assert got.part_of_node[nid] == p
        assert got.part_parent[p] == g["parent_part"] and got.part_cut_node[p] == g["cut_node"]
        assert got.part_pos_offset[p] == g["pos_offset"]
        own = got.own_tok[got.part_tok_off[p]:got.part_tok_off[p + 1]]
        pre = slice(got.part_prefix_off[p], got.part_prefix_off[p + 1])
        assert np.array_equal(own, g["own_tok"])
        assert np.array_equal(got.prefix_tok[pre], g["prefix_tok"])
        assert np.array_equal(got.prefix_visible[pre], g["prefix_visible"])
        run = lambda t: int(t[0]) if len(t) and np.array_equal(t, t[0] + np.arange(len(t))) else -1
        assert got.part_own_start[p] == run(g["own_tok"]) and got.part_prefix_start[p] == run(g["prefix_tok"])
        # bounds and tile summaries = the oracle's metadata of the partition taken as a local tree
        local = {nid: i for i, nid in enumerate(parts[p])}
        lparent = [-1 if nid == parts[p][0] else local[parent[nid]] for nid in parts[p]]
        lmeta = M.dfs_meta(lparent, [seg[nid] for nid in parts[p]])
        n_pre = len(g["prefix_tok"])
        ke = M.kend(lmeta, n_pre, g["prefix_visible"])
        k0 = got.part_prefix_off[p] + got.part_tok_off[p]
        assert np.array_equal(got.kend[k0:k0 + len(ke)], ke)
        tiles = slice(got.part_ktile_off[p], got.part_ktile_off[p + 1])
        if len(ke):
            mn, mx = M.tile_minmax(ke, n_pre, T.KTILE)
            assert np.array_equal(got.kt_min[tiles], mn) and np.array_equal(got.kt_max[tiles], mx)
        else:
            assert tiles.start == tiles.stop
    sz = T.tree_partition_sizes(parent, seg, cap)
    assert sz["n_parts"] == got.n_parts and sz["sum_prefix"] == len(got.prefix_tok) == got.part_prefix_off[-1]
    assert sz["sum_ktiles"] == len(got.kt_min) == got.part_ktile_off[-1]
    assert sz["max_part_tokens"] == max(len(g["own_tok"]) for g in gw)
    assert sz["max_prefix"] == max(len(g["prefix_tok"]) for g in gw)
    return got


@pytest.mark.parametrize("seed", range(40))
def test_random_trees(seed):
    t = W.random_tree(500 + seed, n_nodes=2 + seed, lo=1, hi=150, n_roots=1 + seed % 3, p_zero=0.1,
                      shuffle=bool(seed % 2))
    for cap in (150, 260, 1000):
        _compare(t.parent, t.seg_len, cap)


def test_exhaustive_small_trees():
    import itertools
    for n in (1, 2, 3, 4):
        for parent in W.all_parent_arrays(n):
            for seg in itertools.product((0, 2, 3), repeat=n):
                for cap in (1, 3, 5, 100):
                    _compare(parent, list(seg), cap)


def test_deep_chain_and_wide_star():
    n = 3000
    _compare([-1] + list(range(n - 1)), [7] * n, 500)         # no recursion: a 3000-deep chain
    _compare([-1] + [0] * (n - 1), [5] * n, 64)               # 3000 children, most of them cut off


@pytest.mark.parametrize("cfg,cap", [(2, 4096), (3, 16384), (4, 32768), (5, 65536)])
def test_benchmark_trees(cfg, cap):
    t = W.tree_config(cfg)
    got = T.tree_partition_plan(t.parent, t.seg_len, cap)
    parts = [got.part_nodes[got.part_node_off[p]:got.part_node_off[p + 1]].tolist() for p in range(got.n_parts)]
    P.check_partitions(list(t.parent), list(t.seg_len), cap, parts)
    assert sorted(got.own_tok.tolist()) == list(range(got.n_tokens))
    whole = T.tree_build_meta(t.parent, t.seg_len, t.trained)
    for p in range(got.n_parts):
        own = got.own_tok[got.part_tok_off[p]:got.part_tok_off[p + 1]]
        if len(own):                      # offset = Eq. 9 position of the partition's first token
            assert got.part_pos_offset[p] == whole.tok_pos[own[0]]
        pre = slice(got.part_prefix_off[p], got.part_prefix_off[p + 1])
        assert int(got.prefix_visible[pre].sum()) == got.part_pos_offset[p]


def test_errors():
    with pytest.raises(T.TreeTrainError) as e:
        T.tree_partition_plan([-1, 0], [3, 4], 0)
    assert e.value.status == -2
    with pytest.raises(T.TreeTrainError) as e:
        T.tree_partition_plan([1, 0], [3, 4], 10)             # a cycle, no root
    assert e.value.status == -3
    with pytest.raises(T.TreeTrainError) as e:
        T.tree_partition_plan([-1, 0], [3, -4], 10)
    assert e.value.status == -2
    empty = T.tree_partition_plan([], [], 10)
    assert empty.n_parts == 0 and empty.n_tokens == 0
