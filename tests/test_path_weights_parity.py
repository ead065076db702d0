"""tt_tree_path_weights (host C++) against the oracle's path-by-path definition."""
import numpy as np
import pytest

import paper_2511_00413_amd as T
import workloads as W
from oracle import meta as M


def _ulp_close(a, b, ulps=1):
    np.testing.assert_array_max_ulp(a, b, maxulp=ulps)


@pytest.mark.parametrize("seed", range(25))
def test_random_trees(seed):
    t = W.random_tree(700 + seed, n_nodes=1 + 3 * seed, lo=1, hi=40, n_roots=1 + seed % 3, p_zero=0.1)
    m = M.dfs_meta(t.parent, t.seg_len, t.trained)
    rng = np.random.default_rng(seed)
    K, n = m["K"], m["n_tokens"]
    w = rng.uniform(0.01, 3.0, K).astype(np.float32)
    adv = rng.normal(size=n).astype(np.float32)
    got, leaf = T.tree_path_weights(t.parent, t.seg_len, t.trained, path_weight=w)
    _ulp_close(got, M.path_weights(m, M.WEIGHT_PATH_SUM, w))
    # path k ends in the k-th leaf of the DFS order
    has_child = np.zeros(m["n_nodes"], bool)
    has_child[m["node_parent"][m["node_parent"] >= 0]] = True
    assert np.array_equal(leaf, m["dfs_order"][~has_child])
    got, _ = T.tree_path_weights(t.parent, t.seg_len, t.trained, path_weight=w, advantage=adv)
    want = M.path_weights(m, M.WEIGHT_PATH_SUM, w, advantage=adv)
    assert np.allclose(got, want, rtol=3e-7, atol=0)          # 1 ulp of lambda, then the same fp32 product
    got, _ = T.tree_path_weights(t.parent, t.seg_len, t.trained, scheme=T.WEIGHT_PATH_TOKEN_MEAN)
    _ulp_close(got, M.path_weights(m, M.WEIGHT_PATH_TOKEN_MEAN))
    got, _ = T.tree_path_weights(t.parent, t.seg_len, t.trained, scheme=T.WEIGHT_UNIFORM)
    assert np.array_equal(got, M.path_weights(m, M.WEIGHT_UNIFORM))
    # dyadic path weights: every partial sum is exact, so any summation order gives the same bits
    wd = (rng.integers(1, 64, K) / 64.0).astype(np.float32)
    got, _ = T.tree_path_weights(t.parent, t.seg_len, t.trained, path_weight=wd)
    assert np.array_equal(got, M.path_weights(m, M.WEIGHT_PATH_SUM, wd))


@pytest.mark.parametrize("cfg", [2, 3, 4])
def test_benchmark_trees_equal_weights(cfg):
    t = W.tree_config(cfg)
    meta = T.tree_build_meta(t.parent, t.seg_len, t.trained)
    K = meta.n_leaves
    got, leaf = T.tree_path_weights(t.parent, t.seg_len, t.trained, path_weight=np.full(K, 1.0 / K, np.float32))
    assert len(leaf) == K
    if K & (K - 1) == 0:
        assert np.array_equal(got, meta.tok_weight)           # the special case of Eq. 4, exact for K = 2^m
    else:
        assert np.allclose(got, meta.tok_weight, rtol=3e-7, atol=0)


def test_deep_chain_and_errors():
    n = 5000
    w, leaf = T.tree_path_weights([-1] + list(range(n - 1)), [2] * n, scheme=T.WEIGHT_PATH_TOKEN_MEAN)
    assert leaf.tolist() == [n - 1] and np.allclose(w, 1.0 / (2 * n), rtol=1e-7)
    with pytest.raises(T.TreeTrainError) as e:
        T.tree_path_weights([-1, 0], [1, 1], scheme=7)
    assert e.value.status == -8
    with pytest.raises(T.TreeTrainError) as e:
        T.tree_path_weights([-1, 0], [1, 1])                  # path-sum scheme without path weights
    assert e.value.status == -1
    with pytest.raises(ValueError):
        T.tree_path_weights([-1, 0, 0], [1, 1, 1], path_weight=[1.0])
    w, leaf = T.tree_path_weights([], [], scheme=T.WEIGHT_UNIFORM)
    assert len(w) == 0 and len(leaf) == 0
