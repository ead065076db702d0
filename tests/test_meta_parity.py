"""tt_tree_build_meta (host C++) against the oracle: bit-exact ids, ranges, positions, weights,
visibility bounds and tile summaries."""
import itertools

import numpy as np
import pytest

import paper_2511_00413_amd as T
import workloads as W
from oracle import meta as M

KEYS = ("dfs_order", "node_start", "node_end", "subtree_end", "node_parent", "node_g",
        "tok_node", "tok_pos", "tok_pred", "tok_weight")


def _compare(tree_args, n_prefix=0, prefix_visible=None, root_pos_offset=None):
    parent, seg, trained = tree_args
    got = T.tree_build_meta(parent, seg, trained, root_pos_offset=root_pos_offset, n_prefix=n_prefix,
                            prefix_visible=prefix_visible)
    want = M.dfs_meta(parent, seg, trained, root_pos_offset=root_pos_offset)
    assert got.n_tokens == want["n_tokens"] and got.n_leaves == want["K"]
    for k in KEYS:
        a, b = getattr(got, k), want[k]
        assert a.dtype == b.dtype and np.array_equal(a, b), k
    ke = M.kend(want, n_prefix, prefix_visible)
    assert np.array_equal(got.kend, ke)
    if len(ke):
        mn, mx = M.tile_minmax(ke, n_prefix, T.KTILE)
        assert np.array_equal(got.ktile_kend_min, mn) and np.array_equal(got.ktile_kend_max, mx)
    return got


def test_exhaustive_small_trees():
    for n in (1, 2, 3, 4):
        for parent in W.all_parent_arrays(n):
            for seg in itertools.product((0, 1, 3), repeat=n):
                _compare((parent, list(seg), None))


@pytest.mark.parametrize("seed", range(30))
def test_random_trees_shuffled_ids(seed):
    t = W.random_tree(seed, n_nodes=1 + seed * 3, lo=1, hi=200, n_roots=1 + seed % 4, p_zero=0.1)
    nroots = int((t.parent < 0).sum())
    offs = [(seed * 7 + 13 * r) % 50 for r in range(nroots)]
    P = (seed % 3) * 100 + (seed % 2) * 7
    vis = (np.arange(P) // 13 % 2).astype(np.uint8) if seed % 4 == 1 else None
    _compare((t.parent, t.seg_len, t.trained), n_prefix=P, prefix_visible=vis, root_pos_offset=offs)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_benchmark_configs(cfg):
    t = W.tree_config(cfg)
    _compare((t.parent, t.seg_len, t.trained))


def test_partition_step():
    s = W.step_cfg5(n_chunk=4096, n_prefix=8192 + 5, lo=200, hi=900, root_visible=3000)
    _compare((s.chunk.parent, s.chunk.seg_len, s.chunk.trained), n_prefix=s.n_prefix,
             prefix_visible=s.prefix_visible, root_pos_offset=[int(s.prefix_visible.sum())])


def test_global_g_override():
    # a partition whose leaf is a cut node: weights use the whole tree's g and K
    whole = M.dfs_meta([-1, 0, 0, 1, 1], [4, 3, 2, 5, 6])
    part = T.tree_build_meta([-1, 0, 0], [4, 3, 2], g_override=[3, 2, 1], K_override=3)
    assert np.array_equal(part.node_g, [3, 2, 1])
    assert np.array_equal(part.tok_weight, whole["tok_weight"][:9])
    with pytest.raises(T.TreeTrainError):
        T.tree_build_meta([-1], [1], g_override=[1], K_override=0)
