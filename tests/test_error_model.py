"""The per-row budgets of the attention parity tests (tt_testutil.dq_allowance / dk_allowance) are bounds on what the
rounding of the saved O does to dQ and dK rows.  Checked here on the CPU with dense fp64 attention over a small tree:
the backward is formed twice, with D_i = dO_i . O_i from the exact O and from O rounded to bf16, and the rows of the
difference must stay inside the budgets -- and reach a fair share of them, so that the budgets are not vacuous."""
import numpy as np
import torch

import workloads as W
from oracle import meta as M
from tt_testutil import dk_allowance, dq_allowance, row_err


def _dense_backward(q, k, v, do, vis, scale, o_for_d):
    """fp64, one head: returns o, lse, dq, dk with D formed from o_for_d (None: the exact O)."""
    s = scale * q @ k.T
    s = np.where(vis, s, -np.inf)
    m = s.max(axis=1, keepdims=True)
    p = np.exp(s - m)
    l = p.sum(axis=1, keepdims=True)
    p = p / l
    o = p @ v
    dd = (do * (o if o_for_d is None else o_for_d)).sum(axis=1, keepdims=True)
    ds = p * (do @ v.T - dd)
    return o, (m + np.log(l))[:, 0], scale * ds @ k, scale * ds.T @ q


def test_budgets_bound_the_effect_of_rounding_the_saved_o():
    t = W.random_tree(1100437, n_nodes=24, lo=1, hi=3, n_roots=3, p_zero=0.0)
    om = M.dfs_meta(t.parent, t.seg_len, t.trained)
    n, hq, hkv, d, scale = om["n_tokens"], 4, 2, 32, 32 ** -0.5
    g = torch.Generator().manual_seed(5)
    q, do = (torch.randn((n, hq, d), generator=g).to(torch.bfloat16).double().numpy() for _ in range(2))
    k, v = (torch.randn((n, hkv, d), generator=g).to(torch.bfloat16).double().numpy() for _ in range(2))
    vis = M.mask_chunks(om)
    o = np.zeros((n, hq, d)); lse = np.zeros((hq, n))
    dq = np.zeros((2, n, hq, d)); dk = np.zeros((2, n, hkv, d))
    for h in range(hq):
        kv = h // (hq // hkv)
        o[:, h], lse[h], dq[0, :, h], dkh = _dense_backward(q[:, h], k[:, kv], v[:, kv], do[:, h], vis, scale, None)
        dk[0, :, kv] += dkh
        o_rounded = torch.from_numpy(o[:, h]).to(torch.bfloat16).double().numpy()
        _, _, dq[1, :, h], dkh = _dense_backward(q[:, h], k[:, kv], v[:, kv], do[:, h], vis, scale, o_rounded)
        dk[1, :, kv] += dkh
    kmax = np.repeat(np.linalg.norm(k, axis=-1).max(axis=0), hq // hkv)
    bq = dq_allowance(do, o, kmax[None, :], scale, "bf16")
    bk = dk_allowance(q, k, lse, vis, do, o, scale, "bf16")
    eq = np.linalg.norm(dq[1] - dq[0], axis=-1)
    ek = np.linalg.norm(dk[1] - dk[0], axis=-1)
    assert (eq <= bq * (1 + 1e-9) + 1e-15).all() and (ek <= bk * (1 + 1e-9) + 1e-15).all()
    assert (eq / np.maximum(bq, 1e-30)).max() > 0.05 and (ek / np.maximum(bk, 1e-30)).max() > 0.05
    # with the budgets the rounding of O is invisible to the row metric; without them it is not
    assert row_err(dq[1], dq[0], budget=bq) == 0.0 and row_err(dk[1], dk[0], budget=bk) == 0.0
    assert row_err(dq[1], dq[0]) > 1e-3


def test_a_wrong_row_exceeds_its_budget():
    """A budget must not hide a wrong row: a row that misses one key is far outside it."""
    t = W.random_tree(1100096, n_nodes=9, lo=1, hi=3, n_roots=3, p_zero=0.0)
    om = M.dfs_meta(t.parent, t.seg_len, t.trained)
    n, d, scale = om["n_tokens"], 32, 32 ** -0.5
    g = torch.Generator().manual_seed(6)
    q, k, v, do = (torch.randn((n, d), generator=g).to(torch.bfloat16).double().numpy() for _ in range(4))
    vis = M.mask_chunks(om)
    o, lse, dq, dk = _dense_backward(q, k, v, do, vis, scale, None)
    i = int(np.argmax(vis.sum(axis=1) >= 2))                # first query that sees two keys
    wrong = vis.copy()
    wrong[i, np.nonzero(vis[i])[0][0]] = False              # drops its first key
    _, _, dq_w, dk_w = _dense_backward(q, k, v, do, wrong, scale, None)
    bq = dq_allowance(do[:, None], o[:, None], np.linalg.norm(k, axis=-1).max(), scale, "bf16")[:, 0]
    bk = dk_allowance(q[:, None], k[:, None], lse[None], vis, do[:, None], o[:, None], scale, "bf16")[:, 0]
    assert row_err(dq_w, dq, budget=bq) > 0.1 or row_err(dk_w, dk, budget=bk) > 0.1
