"""The benchmark's own arithmetic (no GPU): the pair count that defines the useful flops of the headline, and the
linearized per-branch forest the speedup is measured against (Section "Derivation", Eq. 7; "Metrics", Eq. 12),
checked against the oracle's dense mask and its branch enumeration."""
import os
import subprocess
import sys

import numpy as np
import pytest

import linearize
import paper_2511_00413_amd as T
import workloads as W
from oracle import meta as M
from tt_testutil import ROOT


def _meta(tree, **kw):
    return T.tree_build_meta(tree.parent, tree.seg_len, tree.trained, **kw)


@pytest.mark.parametrize("seed", range(12))
def test_visible_pairs_is_the_number_of_ones_in_the_dense_mask(seed):
    t = W.random_tree(500 + seed, n_nodes=2 + 2 * seed, lo=1, hi=12, n_roots=1 + seed % 3, p_zero=0.2)
    m = _meta(t)
    om = M.dfs_meta(t.parent, t.seg_len, t.trained)
    dense = M.mask_common_path(om)            # "key and query lie on a common root-to-leaf path", token by token
    assert linearize.visible_pairs(m) == int(np.asarray(dense).sum())


def test_visible_pairs_with_a_prefix():
    """Visible prefix keys are seen by every query of the chunk, hidden ones by none."""
    t = W.random_tree(41, n_nodes=5, lo=3, hi=20)
    vis = np.array([1, 1, 0, 1, 0, 0, 1], dtype=np.uint8)
    own = linearize.visible_pairs(_meta(t))
    m = _meta(t, n_prefix=len(vis), prefix_visible=vis, root_pos_offset=[int(vis.sum())])
    assert linearize.visible_pairs(m) == own + int(vis.sum()) * m.n_tokens


@pytest.mark.parametrize("seed", range(8))
def test_linearized_forest_is_every_root_to_leaf_path(seed):
    t = W.random_tree(600 + seed, n_nodes=3 + 3 * seed, lo=1, hi=30, n_roots=1 + seed % 2, p_zero=0.15)
    m = _meta(t)
    om = M.dfs_meta(t.parent, t.seg_len, t.trained)
    idx, parent, seg = linearize.linearized_forest(m)
    paths = M.paths(om)                                   # the oracle's branches: lists of DFS token indices
    assert len(seg) == len(paths) == m.n_leaves and np.all(parent == -1)
    assert sorted(tuple(int(x) for x in p) for p in paths) == sorted(
        tuple(int(x) for x in idx[o:o + n]) for o, n in zip(np.concatenate([[0], np.cumsum(seg)[:-1]]), seg))
    # every chain is causal attention over its own tokens: L (L + 1) / 2 pairs each
    lm = T.tree_build_meta(parent, seg, np.ones(len(seg), dtype=np.uint8))
    assert linearize.visible_pairs(lm) == int(sum(int(n) * (int(n) + 1) // 2 for n in seg))
    # token redundancy (Eq. 12's bound): N_lin / N
    assert len(idx) == int(sum(len(p) for p in paths)) >= m.n_tokens


def test_benchmark_table_numbers():
    """The counts the benchmark's ratios are built from, for the headline configuration."""
    t = W.tree_config(2)
    m = _meta(t)
    idx, parent, seg = linearize.linearized_forest(m)
    assert (m.n_tokens, len(seg), len(idx)) == (16406, 20, 43656)
    pairs = linearize.visible_pairs(m)
    lm = T.tree_build_meta(parent, seg, np.ones(len(seg), dtype=np.uint8))
    assert pairs == 28627950 and linearize.visible_pairs(lm) == 50209128
    assert abs(len(idx) / m.n_tokens - 2.661) < 1e-3 and abs(50209128 / pairs - 1.754) < 1e-3


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
