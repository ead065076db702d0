"""Pins for oracle/ssm.py.  The tree convolution against a library conv1d run on every branch's own
sequence (forward and, through autograd, backward), finite differences, and the cases the paper
describes: sibling tokens never leak into a child's window, a short parent passes its own parent's
tail on to the grandchildren."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import meta as M
from oracle import ssm as S


def _branch_conv(xb, w, b, act):
    """Library causal depthwise conv1d on one branch sequence xb [L, C] (torch, fp64)."""
    K = w.shape[1]
    z = torch.nn.functional.conv1d(torch.nn.functional.pad(xb.T[None], (K - 1, 0)), w[:, None, :], b, groups=w.shape[0])[0].T
    return torch.nn.functional.silu(z) if act == "silu" else z


@pytest.mark.parametrize("seed,K,act", [(0, 4, "silu"), (1, 3, "silu"), (2, 4, None), (3, 2, "silu"), (4, 5, "silu"), (5, 4, "silu")])
def test_equals_library_conv_on_every_branch(seed, K, act):
    t = W.random_tree(60 + seed, n_nodes=4 + 2 * seed, lo=1, hi=5, n_roots=1 + seed % 2, p_zero=0.2)
    m = M.dfs_meta(t.parent, t.seg_len)
    n, C = m["n_tokens"], 6
    rng = np.random.default_rng(seed)
    x, w, b, dy = rng.normal(size=(n, C)), rng.normal(size=(C, K)), rng.normal(size=C), rng.normal(size=(n, C))
    y, _ = S.tree_conv(x, w, b, m["tok_pred"], act)
    dx, dw, db = S.tree_conv_bwd(x, w, b, m["tok_pred"], dy, act)
    # every branch on its own; a token shared by g branches gets 1/g of its upstream gradient in each
    share = np.zeros(n)
    paths = [p for p in M.paths(m) if len(p)]
    for p in paths:
        share[p] += 1
    xt = torch.tensor(x, requires_grad=True)
    wt = torch.tensor(w, requires_grad=True)
    bt = torch.tensor(b, requires_grad=True)
    total = 0.0
    for p in paths:
        idx = torch.tensor(p, dtype=torch.long)
        yb = _branch_conv(xt[idx], wt, bt, act)
        assert np.allclose(yb.detach().numpy(), y[p], rtol=1e-12, atol=1e-12)
        total = total + (yb * torch.tensor(dy[p] / share[p][:, None])).sum()
    total.backward()
    assert np.allclose(xt.grad.numpy(), dx, rtol=1e-10, atol=1e-12)
    assert np.allclose(wt.grad.numpy(), dw, rtol=1e-10, atol=1e-12)
    assert np.allclose(bt.grad.numpy(), db, rtol=1e-10, atol=1e-12)


def test_finite_differences():
    m = M.dfs_meta([-1, 0, 0, 1], [2, 1, 3, 2])
    rng = np.random.default_rng(1)
    n, C, K = m["n_tokens"], 3, 4
    x, w, b, dy = rng.normal(size=(n, C)), rng.normal(size=(C, K)), rng.normal(size=C), rng.normal(size=(n, C))
    dx, dw, db = S.tree_conv_bwd(x, w, b, m["tok_pred"], dy)
    f = lambda x_, w_, b_: float((S.tree_conv(x_, w_, b_, m["tok_pred"])[0] * dy).sum())
    eps = 1e-6
    for arr, grad, which in ((x, dx, 0), (w, dw, 1), (b, db, 2)):
        for idx in np.ndindex(arr.shape):
            hi, lo = arr.copy(), arr.copy()
            hi[idx] += eps
            lo[idx] -= eps
            args_hi = [x, w, b]; args_lo = [x, w, b]
            args_hi[which], args_lo[which] = hi, lo
            assert abs((f(*args_hi) - f(*args_lo)) / (2 * eps) - grad[idx]) < 1e-6


def test_sibling_tokens_do_not_leak_and_parent_tail_does():
    """Figure "SSM causal convolution" (K = 3): n0 -> {n1 -> {n3, n4}, n2}.  In DFS order n2 follows
    n4; its window must hold n0's last two tokens, not n4's."""
    parent = [-1, 0, 0, 1, 1]
    seg = [3, 2, 2, 2, 2]
    m = M.dfs_meta(parent, seg)
    assert list(m["dfs_order"]) == [0, 1, 3, 4, 2]
    rng = np.random.default_rng(2)
    n, C, K = m["n_tokens"], 2, 3
    x, w = rng.normal(size=(n, C)), rng.normal(size=(C, K))
    rank = {int(i): rk for rk, i in enumerate(m["dfs_order"])}
    tok = lambda nid: np.arange(m["node_start"][rank[nid]], m["node_end"][rank[nid]])
    y, _ = S.tree_conv(x, w, None, m["tok_pred"], None)
    x2 = x.copy()
    x2[tok(4)] += 1.0                                           # the DFS-adjacent sibling branch
    x2[tok(3)] -= 1.0
    x2[tok(1)] *= 2.0
    y2, _ = S.tree_conv(x2, w, None, m["tok_pred"], None)
    assert np.array_equal(y2[tok(2)], y[tok(2)])
    # first token of n2 by hand: w[:,2]*x[n2[0]] + w[:,1]*x[n0[-1]] + w[:,0]*x[n0[-2]]
    t0, p = tok(2)[0], tok(0)
    assert np.allclose(y[t0], w[:, 2] * x[t0] + w[:, 1] * x[p[-1]] + w[:, 0] * x[p[-2]])
    x3 = x.copy()
    x3[p[-1]] += 1.0
    assert not np.allclose(S.tree_conv(x3, w, None, m["tok_pred"], None)[0][t0], y[t0])


def test_short_parent_passes_grandparent_tail_on():
    """Appendix "Tree-Correct Causal Convolution": the saved context is the tail of [parent context ;
    chunk], so a one-token parent hands its own parent's tokens on; a zero-length node hands
    everything on; the start of a branch is zero-padded."""
    m = M.dfs_meta([-1, 0, 1, 2], [3, 1, 0, 2])
    K, C = 4, 1
    x = np.arange(1, 7, dtype=np.float64)[:, None]              # tokens 1..6
    w = np.asarray([[1000.0, 100.0, 10.0, 1.0]])
    y, _ = S.tree_conv(x, w, None, m["tok_pred"], None)
    # sequence is 1 2 3 | 4 | (empty) | 5 6
    assert y[:, 0].tolist() == [1.0, 12.0, 123.0, 1234.0, 2345.0, 3456.0]
    # a second root starts from zero context
    m = M.dfs_meta([-1, -1], [2, 2])
    y, _ = S.tree_conv(np.asarray([[1.0], [2.0], [3.0], [4.0]]), w, None, m["tok_pred"], None)
    assert y[:, 0].tolist() == [1.0, 12.0, 3.0, 34.0]


# ---- gated delta rule with tree state routing ----

def _gdn_inputs(n, hk, hv, dk, dv, seed):
    rng = np.random.default_rng(seed)
    q = rng.normal(size=(n, hk, dk)); k = rng.normal(size=(n, hk, dk))
    q /= np.linalg.norm(q, axis=-1, keepdims=True); k /= np.linalg.norm(k, axis=-1, keepdims=True)
    v = rng.normal(size=(n, hv, dv))
    g = -rng.uniform(0.01, 0.5, size=(n, hv))
    beta = rng.uniform(0.1, 0.9, size=(n, hv))
    return q, k, v, g, beta


def _gdn_chain_library(q, k, v, g, beta, scale):
    """One sequence, written with library matrix routines in the chunk-free 'delta rule as a linear
    attention with a triangular solve' form: with decay products D_ij = exp(sum_{j<l<=i} g_l),
    u = (I + tril(diag(beta) (K K^T) * D, -1))^{-1} diag(beta) V  and  o = scale * tril((Q K^T) * D) u.
    A different route to the same numbers than the recurrence (whole sequence as one chunk, zero
    initial state)."""
    import scipy.linalg
    n = len(q)
    gc = np.cumsum(g)
    D = np.exp(gc[:, None] - gc[None, :])
    A = np.tril(beta[:, None] * (k @ k.T) * D, -1)
    u = scipy.linalg.solve_triangular(np.eye(n) + A, beta[:, None] * v, lower=True, unit_diagonal=True)
    return scale * (np.tril((q @ k.T) * D) @ u)


def test_gdn_chain_equals_triangular_solve_form():
    n, dk, dv = 37, 8, 5
    q, k, v, g, beta = _gdn_inputs(n, 1, 1, dk, dv, 0)
    tok_pred = np.arange(-1, n - 1)
    o = S.gdn_tree(q, k, v, g, beta, tok_pred, scale=0.7)
    want = _gdn_chain_library(q[:, 0], k[:, 0], v[:, 0], g[:, 0], beta[:, 0], 0.7)
    assert np.allclose(o[:, 0], want, rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("seed", range(6))
def test_gdn_tree_equals_every_branch_run_alone(seed):
    """Forward equivalence (Eq. 6) for the SSM layer: a token's output in the tree equals its output
    when its branch is run as a standalone sequence."""
    t = W.random_tree(70 + seed, n_nodes=5 + 2 * seed, lo=1, hi=6, n_roots=1 + seed % 2, p_zero=0.15)
    m = M.dfs_meta(t.parent, t.seg_len)
    n = m["n_tokens"]
    q, k, v, g, beta = _gdn_inputs(n, 2, 4, 6, 5, seed)
    o = S.gdn_tree(q, k, v, g, beta, m["tok_pred"])
    for p in M.paths(m):
        if not len(p):
            continue
        chain = np.arange(-1, len(p) - 1)
        ob = S.gdn_tree(q[p], k[p], v[p], g[p], beta[p], chain)
        assert np.allclose(ob, o[p], rtol=1e-11, atol=1e-13)
        for h in range(4):                      # and the library route on the same branch
            want = _gdn_chain_library(q[p, h // 2], k[p, h // 2], v[p, h], g[p, h], beta[p, h], 6 ** -0.5)
            assert np.allclose(o[p, h], want, rtol=1e-9, atol=1e-11)


def test_gdn_sibling_state_does_not_leak():
    """Figure "SSM state routing": n0 -> {n1 -> {n3, n4}, n2}; n2 must start from n0's state, so
    nothing in n1's subtree may influence it, while n0's tokens must."""
    m = M.dfs_meta([-1, 0, 0, 1, 1], [3, 2, 2, 2, 2])
    n = m["n_tokens"]
    q, k, v, g, beta = _gdn_inputs(n, 1, 1, 4, 3, 5)
    rank = {int(i): rk for rk, i in enumerate(m["dfs_order"])}
    tok = lambda nid: np.arange(m["node_start"][rank[nid]], m["node_end"][rank[nid]])
    o = S.gdn_tree(q, k, v, g, beta, m["tok_pred"])
    v2 = v.copy()
    for nid in (1, 3, 4):
        v2[tok(nid)] += 1.0
    o2 = S.gdn_tree(q, k, v2, g, beta, m["tok_pred"])
    assert np.array_equal(o2[tok(2)], o[tok(2)])
    v3 = v.copy()
    v3[tok(0)[-1]] += 1.0
    assert not np.allclose(S.gdn_tree(q, k, v3, g, beta, m["tok_pred"])[tok(2)], o[tok(2)])


def test_gdn_closed_forms():
    # beta = 0: nothing is ever written, outputs are zero
    q, k, v, g, beta = _gdn_inputs(9, 1, 2, 4, 3, 1)
    assert np.all(S.gdn_tree(q, k, v, g, 0 * beta, np.arange(-1, 8)) == 0)
    # one token, beta = 1: S = k v^T, o = scale (q.k) v
    o = S.gdn_tree(q[:1], k[:1], v[:1], g[:1], np.ones((1, 2)), [-1], scale=1.0)
    assert np.allclose(o[0], (q[0, 0] @ k[0, 0]) * v[0])
    # beta = 1, no decay, the same unit key twice: the second write replaces the first value
    kk = np.zeros((2, 1, 4)); kk[:, 0, 1] = 1.0
    o = S.gdn_tree(kk, kk, v[:2, :1], np.zeros((2, 1)), np.ones((2, 1)), [-1, 0], scale=1.0)
    assert np.allclose(o[1, 0], v[1, 0]) and np.allclose(o[0, 0], v[0, 0])
    # orthogonal keys, beta = 1: plain decayed linear attention  o_t = sum_j exp(sum_{j<l<=t} g_l) (q_t.k_j) v_j
    n = 4
    ko = np.eye(4)[:n][:, None, :]
    qq = np.random.default_rng(2).normal(size=(n, 1, 4))
    gg = -np.random.default_rng(3).uniform(0.1, 0.4, size=(n, 1))
    vv = v[:n, :1]
    o = S.gdn_tree(qq, ko, vv, gg, np.ones((n, 1)), np.arange(-1, n - 1), scale=1.0)
    for t_ in range(n):
        want = sum(np.exp(gg[j + 1:t_ + 1, 0].sum()) * (qq[t_, 0] @ ko[j, 0]) * vv[j, 0] for j in range(t_ + 1))
        assert np.allclose(o[t_, 0], want)


# ---- backward of the gated delta rule with tree state routing ----

def _torch_branch_gdn(q, k, v, g, beta, scale):
    """One standalone sequence with library tensors (autograd does the differentiation): q, k [L, Dk], v [L, Dv]."""
    S_ = torch.zeros((q.shape[1], v.shape[1]), dtype=torch.float64)
    outs = []
    for t in range(q.shape[0]):
        S_ = torch.exp(g[t]) * S_
        d = beta[t] * (v[t] - S_.T @ k[t])
        S_ = S_ + torch.outer(k[t], d)
        outs.append(scale * (S_.T @ q[t]))
    return torch.stack(outs)


@pytest.mark.parametrize("seed", range(4))
def test_gdn_bwd_equals_autograd_over_branches(seed):
    """Every branch run alone through autograd; a token shared by n branches gets 1/n of its upstream gradient
    in each, so the summed branch gradients are the tree's."""
    t = W.random_tree(75 + seed, n_nodes=4 + 2 * seed, lo=1, hi=5, n_roots=1 + seed % 2, p_zero=0.15)
    m = M.dfs_meta(t.parent, t.seg_len)
    n, hk, hv, dk, dv = m["n_tokens"], 1, 2, 5, 4
    q, k, v, g, beta = _gdn_inputs(n, hk, hv, dk, dv, seed)
    d_o = np.random.default_rng(seed + 50).normal(size=(n, hv, dv))
    dq, dkk, dvv, dg, dbeta = S.gdn_tree_bwd(q, k, v, g, beta, m["tok_pred"], d_o, scale=0.6)
    share = np.zeros(n)
    paths = [p for p in M.paths(m) if len(p)]
    for p in paths:
        share[p] += 1
    tq, tk, tv, tg, tb = (torch.tensor(x, requires_grad=True) for x in (q, k, v, g, beta))
    total = 0.0
    for p in paths:
        idx = torch.tensor(p, dtype=torch.long)
        for h in range(hv):
            ob = _torch_branch_gdn(tq[idx, 0], tk[idx, 0], tv[idx, h], tg[idx, h], tb[idx, h], 0.6)
            total = total + (ob * torch.tensor(d_o[p, h] / share[p][:, None])).sum()
    total.backward()
    for name, a, b in (("dq", dq, tq.grad), ("dk", dkk, tk.grad), ("dv", dvv, tv.grad), ("dg", dg, tg.grad), ("dbeta", dbeta, tb.grad)):
        assert np.allclose(a, b.numpy(), rtol=1e-9, atol=1e-11), name


def test_gdn_bwd_finite_differences():
    m = M.dfs_meta([-1, 0, 0], [2, 2, 1])
    n, hk, hv, dk, dv = m["n_tokens"], 1, 1, 3, 2
    q, k, v, g, beta = _gdn_inputs(n, hk, hv, dk, dv, 9)
    d_o = np.random.default_rng(1).normal(size=(n, hv, dv))
    grads = S.gdn_tree_bwd(q, k, v, g, beta, m["tok_pred"], d_o)
    args = [q, k, v, g, beta]
    f = lambda a: float((S.gdn_tree(*a, m["tok_pred"]) * d_o).sum())
    eps = 1e-6
    for which, grad in enumerate(grads):
        for idx in np.ndindex(args[which].shape):
            hi = [x.copy() for x in args]; lo = [x.copy() for x in args]
            hi[which][idx] += eps; lo[which][idx] -= eps
            assert abs((f(hi) - f(lo)) / (2 * eps) - grad[idx]) < 1e-6, (which, idx)


def test_gdn_bwd_gradients_add_at_a_branch_point():
    """Two children of one parent: the parent's gradients are the sum of what each child alone would send
    back plus the parent's own (linearity in d_o)."""
    m = M.dfs_meta([-1, 0, 0], [3, 2, 2])
    n = m["n_tokens"]
    q, k, v, g, beta = _gdn_inputs(n, 1, 1, 4, 3, 4)
    d_o = np.random.default_rng(2).normal(size=(n, 1, 3))
    full = S.gdn_tree_bwd(q, k, v, g, beta, m["tok_pred"], d_o)
    parts = []
    for sel in (slice(0, 3), slice(3, 5), slice(5, 7)):
        masked = np.zeros_like(d_o)
        masked[sel] = d_o[sel]
        parts.append(S.gdn_tree_bwd(q, k, v, g, beta, m["tok_pred"], masked))
    for i in range(5):
        assert np.allclose(full[i], parts[0][i] + parts[1][i] + parts[2][i], rtol=1e-12, atol=1e-14)
    # a child's upstream gradient never reaches its sibling
    only_c1 = parts[1]
    assert np.all(only_c1[2][5:7] == 0) and np.all(only_c1[0][5:7] == 0) and np.any(only_c1[2][0:3] != 0)
