"""Pins for oracle/rope.py: closed forms, orthogonality, the relative-position property that defines
RoPE, an independent complex-number formulation, and the tree property of Eq. 9's positions."""
import numpy as np

import workloads as W
from oracle import meta as M
from oracle import rope as R


def test_two_dimensional_head_is_a_plane_rotation():
    # d = 2: one frequency, base^0 = 1, so the vector turns by `pos` radians
    x = np.array([[[1.0, 0.0]], [[0.0, 1.0]], [[2.0, -3.0]]])
    y = R.rope(x, [1, 2, 0])
    assert np.allclose(y[0, 0], [np.cos(1.0), np.sin(1.0)], atol=1e-15)
    assert np.allclose(y[1, 0], [-np.sin(2.0), np.cos(2.0)], atol=1e-15)
    assert np.array_equal(y[2, 0], [2.0, -3.0])              # position 0: identity


def test_frequencies_follow_the_geometric_ladder():
    # unit vector in pair i at position 1 turns by base^(-2i/d)
    d, base = 8, 10000.0
    for i in range(d // 2):
        x = np.zeros((1, 1, d))
        x[0, 0, i] = 1.0
        y = R.rope(x, [1], base=base)
        a = base ** (-2.0 * i / d)
        want = np.zeros(d)
        want[i], want[i + d // 2] = np.cos(a), np.sin(a)
        assert np.allclose(y[0, 0], want, atol=1e-15)


def test_orthogonal_and_inverse():
    rng = np.random.default_rng(0)
    x = rng.normal(size=(9, 3, 16))
    pos = rng.integers(0, 100000, size=9)
    y = R.rope(x, pos)
    half = 8
    assert np.allclose(x[..., :half] ** 2 + x[..., half:] ** 2, y[..., :half] ** 2 + y[..., half:] ** 2, rtol=1e-12)
    assert np.allclose(R.rope(y, pos, inverse=True), x, atol=1e-10)


def test_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(1)
    q, k = rng.normal(size=(1, 1, 32)), rng.normal(size=(1, 1, 32))
    def score(m, n):
        return float((R.rope(q, [m], base=1e4) * R.rope(k, [n], base=1e4)).sum())
    assert abs(score(17, 5) - score(1012, 1000)) <= 1e-9
    assert abs(score(3, 3) - float((q * k).sum())) <= 1e-12
    assert abs(score(17, 5) - score(5, 17)) > 1e-3           # and the sign of the offset matters


def test_against_complex_multiplication():
    # independent formulation: pair (x[i], x[i + d/2]) as a complex number times exp(j * angle)
    rng = np.random.default_rng(2)
    x = rng.normal(size=(5, 2, 12))
    pos = np.array([0, 1, 7, 4096, 123457])
    base = 5.0e5
    z = x[..., :6] + 1j * x[..., 6:]
    ang = pos[:, None] * base ** (-np.arange(6) / 6.0)
    w = z * np.exp(1j * ang)[:, None, :]
    want = np.concatenate([w.real, w.imag], axis=-1)
    assert np.allclose(R.rope(x, pos, base=base), want, atol=1e-9)


def test_same_depth_on_different_branches_rotates_alike():
    # Eq. 9: siblings restart at the parent's end position, so the first tokens of two sibling nodes
    # get the same rotation although they are far apart in the DFS sequence
    t = W.tree_cfg1()
    m = M.dfs_meta(t.parent, t.seg_len, t.trained)
    pos = m["tok_pos"]
    ns = m["node_start"]
    par = m["node_parent"]
    sib = [(a, b) for a in range(m["n_nodes"]) for b in range(a + 1, m["n_nodes"]) if par[a] == par[b] and par[a] >= 0]
    assert sib
    a, b = sib[0]
    assert pos[ns[a]] == pos[ns[b]] and ns[a] != ns[b]
    x = np.random.default_rng(3).normal(size=(1, 1, 8))
    xa = R.rope(x, [pos[ns[a]]])
    xb = R.rope(x, [pos[ns[b]]])
    assert np.array_equal(xa, xb)
