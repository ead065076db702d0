"""Pins for oracle/meta.py:path_weights ("Derivation", general path weights): the weighted-sum
identity against the double sum over branches, the special cases the paper names, closed forms."""
import numpy as np
import pytest

import workloads as W
from oracle import meta as M


def _branch_loss(meta, w, ell, adv=None):
    """sum_k w_k sum_{t in p_k} trained_t * A_t * l_t, every branch walked on its own (fp64)."""
    tr = meta["tok_trained"].astype(np.float64)
    a = np.ones(meta["n_tokens"]) if adv is None else np.asarray(adv, dtype=np.float64)
    total = 0.0
    for k, p in enumerate(M.paths(meta)):
        total += w[k] * sum(tr[t] * a[t] * ell[t] for t in p)
    return total


@pytest.mark.parametrize("seed", range(10))
def test_weighted_sum_equals_branch_double_sum(seed):
    t = W.random_tree(40 + seed, n_nodes=3 + 2 * seed, lo=1, hi=7, n_roots=1 + seed % 2, p_zero=0.1)
    m = M.dfs_meta(t.parent, t.seg_len, t.trained)
    rng = np.random.default_rng(seed)
    K = m["K"]
    w = rng.uniform(0.1, 2.0, K).astype(np.float32)
    ell = rng.uniform(0.5, 3.0, m["n_tokens"])
    adv = rng.normal(size=m["n_tokens"]).astype(np.float32)
    lam = M.path_weights(m, M.WEIGHT_PATH_SUM, w)
    assert lam.dtype == np.float32
    want = _branch_loss(m, w.astype(np.float64), ell)
    assert abs(float((lam.astype(np.float64) * ell).sum()) - want) <= 1e-6 * abs(want) + 1e-9
    lam_a = M.path_weights(m, M.WEIGHT_PATH_SUM, w, advantage=adv)
    want_a = _branch_loss(m, w.astype(np.float64), ell, adv)
    assert abs(float((lam_a.astype(np.float64) * ell).sum()) - want_a) <= 1e-5 * (abs(want_a) + 1.0)
    # per-branch token mean, branches averaged
    lam_m = M.path_weights(m, M.WEIGHT_PATH_TOKEN_MEAN)
    tr = m["tok_trained"].astype(np.float64)
    want_m = 0.0
    for p in M.paths(m):
        cnt = tr[p].sum()
        if cnt:
            want_m += (tr[p] * ell[p]).sum() / cnt
    want_m /= K
    assert abs(float((lam_m.astype(np.float64) * ell).sum()) - want_m) <= 1e-6 * abs(want_m) + 1e-9


def test_equal_path_weights_are_g_over_k():
    """w_k = 1/K is the special case of Eq. 4; with K a power of two everything is exact."""
    t = W.tree_config(3)                      # K = 32
    m = M.dfs_meta(t.parent, t.seg_len, t.trained)
    assert m["K"] == 32
    lam = M.path_weights(m, M.WEIGHT_PATH_SUM, np.full(32, 1.0 / 32, dtype=np.float32))
    assert np.array_equal(lam, m["tok_weight"])
    # the worked tree (K = 3): equal up to the rounding of 1/3
    t = W.tree_cfg1()
    m = M.dfs_meta(t.parent, t.seg_len, t.trained)
    lam = M.path_weights(m, M.WEIGHT_PATH_SUM, np.full(3, 1.0 / 3, dtype=np.float32))
    assert np.allclose(lam, m["tok_weight"], rtol=2e-7, atol=0)


def test_worked_tree_by_hand():
    """root 64 -> A 48 -> {B 32, C 40}; root -> D 56.  Leaves in DFS order: B, C, D."""
    t = W.tree_cfg1()
    m = M.dfs_meta(t.parent, t.seg_len, [1] * 5)
    lam = M.path_weights(m, M.WEIGHT_PATH_SUM, np.asarray([0.5, 0.25, 2.0], dtype=np.float32))
    seg = lambda rk: lam[m["node_start"][rk]:m["node_end"][rk]]
    assert np.all(seg(0) == 2.75) and np.all(seg(1) == 0.75)           # root: all three, A: B and C
    assert np.all(seg(2) == 0.5) and np.all(seg(3) == 0.25) and np.all(seg(4) == 2.0)
    # token mean: branch lengths 64+48+32 = 144, 64+48+40 = 152, 64+56 = 120; K = 3
    lam = M.path_weights(m, M.WEIGHT_PATH_TOKEN_MEAN).astype(np.float64)
    wb, wc, wd = 1 / (3 * 144), 1 / (3 * 152), 1 / (3 * 120)
    for rk, want in ((0, wb + wc + wd), (1, wb + wc), (2, wb), (3, wc), (4, wd)):
        assert np.allclose(seg_of(lam, m, rk), want, rtol=1e-7)
    # each branch's weights sum to 1/K over its tokens -> total = 1
    assert abs(lam.sum() - (144 * wb + 152 * wc + 120 * wd)) < 1e-6
    # uniform: every unique trained token counts once
    m2 = M.dfs_meta(t.parent, t.seg_len, [1, 0, 1, 1, 0])
    lam = M.path_weights(m2, M.WEIGHT_UNIFORM)
    assert lam.sum() == 64 + 32 + 40 and set(np.unique(lam)) == {0.0, 1.0}
    assert np.array_equal(lam != 0, m2["tok_trained"] != 0)


def seg_of(lam, m, rk):
    return lam[m["node_start"][rk]:m["node_end"][rk]]


def test_chain_and_untrained():
    m = M.dfs_meta([-1, 0, 1], [4, 5, 6], [0, 1, 1])
    lam = M.path_weights(m, M.WEIGHT_PATH_TOKEN_MEAN)
    assert np.all(lam[:4] == 0) and np.allclose(lam[4:], 1 / 11, rtol=1e-7)      # one branch, 11 trained tokens
    lam = M.path_weights(m, M.WEIGHT_PATH_SUM, [3.0], advantage=np.arange(15, dtype=np.float32))
    assert np.array_equal(lam, np.where(np.arange(15) >= 4, 3.0 * np.arange(15), 0).astype(np.float32))
    # a branch with no trained token gets no weight (and divides by nothing)
    m = M.dfs_meta([-1, 0, 0], [2, 3, 4], [0, 0, 1])
    lam = M.path_weights(m, M.WEIGHT_PATH_TOKEN_MEAN)
    assert np.all(lam[:5] == 0) and np.allclose(lam[5:], 1 / (2 * 4))
