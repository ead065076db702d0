"""Pins for the attention oracle (oracle/branch_attention.c via oracle/attention.py).

The per-branch oracle is tied to (a) the paper's mask statements through an independent dense
numpy implementation, (b) a library routine (torch scaled_dot_product_attention + autograd on
the CPU) for the chain / masked cases, (c) finite differences for the gradients, (d) closed forms.
"""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import attention as A
from oracle import meta as M
from tt_testutil import rel_l2


def _inputs(n, hq, hkv, d, seed):
    dims = W.AttnDims(hq, hkv, d, "fp32", 1.0)
    return W.attn_inputs(n, n, dims, seed)


def _torch_ref(mask, q, k, v, do, scale):
    """Library third opinion: torch SDPA under a boolean mask, gradients by autograd, fp64."""
    G = q.shape[1] // k.shape[1]
    qt = q.double().permute(1, 0, 2).clone().requires_grad_(True)          # [h, n, d]
    kt = k.double().permute(1, 0, 2).clone().requires_grad_(True)
    vt = v.double().permute(1, 0, 2).clone().requires_grad_(True)
    ke = kt.repeat_interleave(G, dim=0)
    ve = vt.repeat_interleave(G, dim=0)
    o = torch.nn.functional.scaled_dot_product_attention(
        qt[None], ke[None], ve[None], attn_mask=torch.from_numpy(mask)[None, None], scale=scale)[0]
    (o * do.double().permute(1, 0, 2)).sum().backward()
    s = scale * qt @ ke.transpose(1, 2)
    s = s.masked_fill(~torch.from_numpy(mask)[None], float("-inf"))
    lse = torch.logsumexp(s, dim=-1)
    return dict(o=o.permute(1, 0, 2).detach().numpy(), lse=lse.detach().numpy(),
                dq=qt.grad.permute(1, 0, 2).numpy(), dk=kt.grad.permute(1, 0, 2).numpy(),
                dv=vt.grad.permute(1, 0, 2).numpy())


@pytest.mark.parametrize("seed", range(6))
def test_branches_equal_dense_mask_and_torch(seed):
    t = W.random_tree(100 + seed, n_nodes=3 + seed, lo=1, hi=9, n_roots=1 + seed % 2, p_zero=0.1)
    m = M.dfs_meta(t.parent, t.seg_len)
    n = m["n_tokens"]
    hq, hkv, d = (4, 2, 8) if seed % 2 else (3, 3, 16)
    q, k, v, do = _inputs(n, hq, hkv, d, seed)
    scale = 0.37
    got = A.branches(m, q, k, v, do, scale=scale)
    mask = M.mask_chunks(m)                      # the appendix's literal mask construction
    ref = A.dense(mask, q, k, v, do, scale=scale)
    lib = _torch_ref(mask, q, k, v, do, scale)
    for key in ("o", "lse", "dq", "dk", "dv"):
        assert rel_l2(got[key], ref[key]) < 1e-12, key
        assert rel_l2(got[key], lib[key]) < 1e-12, key


def test_chain_is_textbook_causal_attention():
    t = W.chain_tree([5, 7, 4])
    m = M.dfs_meta(t.parent, t.seg_len)
    q, k, v, do = _inputs(16, 2, 1, 8, 3)
    got = A.branches(m, q, k, v, do)
    qt, kt, vt = (x.double().permute(1, 0, 2)[None] for x in (q, k, v))
    o = torch.nn.functional.scaled_dot_product_attention(qt, kt.expand(1, 2, 16, 8), vt.expand(1, 2, 16, 8),
                                                         is_causal=True)[0].permute(1, 0, 2).numpy()
    assert rel_l2(got["o"], o) < 1e-12


def test_forest_of_chains_is_block_diagonal():
    f = W.forest_of_chains([4, 6, 3])
    m = M.dfs_meta(f.parent, f.seg_len)
    q, k, v, do = _inputs(13, 2, 2, 8, 4)
    got = A.branches(m, q, k, v, do)
    lo = 0
    for ln in (4, 6, 3):
        sl = slice(lo, lo + ln)
        c = W.chain_tree([ln])
        sub = A.branches(M.dfs_meta(c.parent, c.seg_len), q[sl], k[sl], v[sl], do[sl])
        for key in ("o", "dq", "dk", "dv"):
            assert rel_l2(got[key][sl], sub[key]) < 1e-13
        assert rel_l2(got["lse"][:, sl], sub["lse"]) < 1e-13
        lo += ln


def test_finite_differences():
    t = W.tree_cfg1()
    small = W.Tree(t.parent, np.array([3, 2, 2, 3, 2], dtype=np.int32), t.trained)
    m = M.dfs_meta(small.parent, small.seg_len)
    n = m["n_tokens"]
    q, k, v, do = _inputs(n, 2, 1, 8, 7)
    base = A.branches(m, q, k, v, do, scale=0.5)

    def f(qq, kk, vv):
        return float((A.branches(m, qq, kk, vv, None, scale=0.5)["o"] * do.double().numpy()).sum())

    eps = 1e-3          # inputs are float32: step must survive the float32 rounding of x +- eps
    rng = np.random.default_rng(0)
    for name, x in (("dq", q), ("dk", k), ("dv", v)):
        for _ in range(12):
            i = tuple(int(rng.integers(0, s)) for s in x.shape)
            xp, xm = x.clone(), x.clone()
            xp[i] += eps
            xm[i] -= eps
            args_p = {"dq": (xp, k, v), "dk": (q, xp, v), "dv": (q, k, xp)}[name]
            args_m = {"dq": (xm, k, v), "dk": (q, xm, v), "dv": (q, k, xm)}[name]
            h = float(xp[i] - xm[i])
            fd = (f(*args_p) - f(*args_m)) / h
            assert abs(fd - base[name][i]) < 1e-5 * max(1.0, abs(fd)), (name, i, fd, base[name][i])


def test_closed_forms():
    t = W.tree_cfg1()
    small = W.Tree(t.parent, np.array([4, 3, 2, 3, 2], dtype=np.int32), t.trained)
    m = M.dfs_meta(small.parent, small.seg_len)
    n = m["n_tokens"]
    q, k, v, do = _inputs(n, 2, 2, 8, 9)
    # V constant => O constant (rows of P sum to one); dQ = dK = 0 then, because dP - D = 0
    vc = torch.ones_like(v) * 0.75
    r = A.branches(m, q, k, vc, do)
    assert np.allclose(r["o"], 0.75, atol=1e-14)
    assert np.abs(r["dq"]).max() < 1e-14 and np.abs(r["dk"]).max() < 1e-14
    # dV column sums: sum_j dV_j = sum_i dO_i (each row of P sums to one)
    r = A.branches(m, q, k, v, do)
    assert rel_l2(r["dv"].sum(axis=0), do.double().numpy().sum(axis=0)) < 1e-13
    # Q = 0 => uniform attention over the visible keys: LSE = log(count), count = position + 1
    r0 = A.branches(m, torch.zeros_like(q), k, v, None)
    assert np.allclose(r0["lse"], np.log(m["tok_pos"] + 1.0)[None, :], atol=1e-14)


def test_rows_matches_branches():
    t = W.random_tree(5, n_nodes=7, lo=2, hi=9)
    m = M.dfs_meta(t.parent, t.seg_len)
    n = m["n_tokens"]
    q, k, v, do = _inputs(n, 4, 2, 8, 11)
    full = A.branches(m, q, k, v, do)
    rows = [0, n // 3, n // 2, n - 1]
    keys = [0, 1, n // 2, n - 1]
    for kvh in (0, 1):
        s = A.rows(m, q, k, v, do, kvh, rows, keys)
        hs = slice(kvh * 2, kvh * 2 + 2)
        assert rel_l2(s["o"], full["o"][rows][:, hs]) < 1e-13
        assert rel_l2(s["lse"], full["lse"][hs][:, rows].T) < 1e-13
        assert rel_l2(s["dq"], full["dq"][rows][:, hs]) < 1e-12
        assert rel_l2(s["dk"], full["dk"][keys][:, kvh]) < 1e-12
        assert rel_l2(s["dv"], full["dv"][keys][:, kvh]) < 1e-12


def test_rows_restricted_to_a_query_subset():
    """complete_keys=False: with d_o zero outside the subset, the subset's contributions are the whole
    dK / dV (every term of Eq. 5's sum carries a factor dO_i); pinned against branches() on the masked d_o,
    and against the unrestricted rows() call on the same masked d_o."""
    t = W.random_tree(6, n_nodes=8, lo=2, hi=9)
    m = M.dfs_meta(t.parent, t.seg_len)
    n = m["n_tokens"]
    q, k, v, do = _inputs(n, 4, 2, 8, 12)
    subset = sorted({1, n // 4, n // 2, n - 2, n - 1})
    do_masked = torch.zeros_like(do)
    do_masked[subset] = do[subset]
    full = A.branches(m, q, k, v, do_masked)
    keys = [0, 1, n // 4, n - 1]
    for kvh in (0, 1):
        s = A.rows(m, q, k, v, do_masked, kvh, subset, keys, complete_keys=False)
        assert s["n_rows_evaluated"] == len(subset)
        assert rel_l2(s["dk"], full["dk"][keys][:, kvh]) < 1e-12
        assert rel_l2(s["dv"], full["dv"][keys][:, kvh]) < 1e-12
        c = A.rows(m, q, k, v, do_masked, kvh, subset, keys)
        assert rel_l2(s["dk"], c["dk"]) < 1e-12 and rel_l2(s["dv"], c["dv"]) < 1e-12
    # and it is NOT the whole gradient when d_o is not masked (the option really drops rows)
    s = A.rows(m, q, k, v, do, 0, subset, [0], complete_keys=False)
    assert rel_l2(s["dv"], A.branches(m, q, k, v, do)["dv"][[0]][:, 0]) > 1e-2


def test_fp32_variant_close_to_fp64():
    t = W.tree_cfg1()
    m = M.dfs_meta(t.parent, t.seg_len)
    q, k, v, do = _inputs(240, 4, 4, 64, 1)
    a = A.branches(m, q, k, v, do)
    b = A.branches(m, q, k, v, do, real="f32")
    for key in ("o", "lse", "dq", "dk", "dv"):
        assert rel_l2(b[key], a[key]) < 2e-6, key
