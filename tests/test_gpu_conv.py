"""GPU parity: tree-correct causal convolution (forward and backward) against the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_2511_00413_amd as T
import workloads as W
from oracle import meta as M
from oracle import ssm as S
from tt_testutil import rel_l2

pytestmark = pytest.mark.gpu


def _inputs(n, c, k, seed, dtype):
    g = torch.Generator().manual_seed(seed)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    x = torch.randn((n, c), generator=g).to(tdt)
    dy = torch.randn((n, c), generator=g).to(tdt)
    w = torch.randn((c, k), generator=g) * 0.5
    b = torch.randn(c, generator=g) * 0.1
    return x, dy, w, b


def _run_and_check(tok_pred, n, c, k, seed, dtype, silu=True, bias=True):
    x, dy, w, b = _inputs(n, c, k, seed, dtype)
    if not bias:
        b = None
    act = "silu" if silu else None
    want_y, _ = S.tree_conv(x, w, b, tok_pred, act)
    want_dx, want_dw, want_db = S.tree_conv_bwd(x, w, b, tok_pred, dy, act)
    pred_d = torch.from_numpy(np.asarray(tok_pred, dtype=np.int32)).cuda()
    xd, dyd, wd, bd = x.cuda(), dy.cuda(), w.cuda(), None if b is None else b.cuda()
    plan = T.tree_conv_plan(tok_pred, k)
    print(f"[case] tree conv n={n} C={c} K={k} {dtype} silu={silu} bias={bias}: {len(plan.fix_tok)} fix-up tokens", flush=True)
    y = T.tree_conv_fwd(xd, wd, bd, pred_d, silu=silu)
    dx, dw, db = T.tree_conv_bwd(xd, wd, bd, pred_d, dyd, plan, silu=silu, want_dbias=bias)
    torch.cuda.synchronize()
    tol = 4e-3 if dtype == "bf16" else 2e-6           # bf16: one rounding of the output (2^-9 relative)
    errs = dict(y=rel_l2(y.float().cpu().numpy(), want_y), dx=rel_l2(dx.float().cpu().numpy(), want_dx),
                dw=rel_l2(dw.cpu().numpy(), want_dw))
    if bias:
        errs["db"] = rel_l2(db.cpu().numpy(), want_db)
    print("   rel-L2:", {k_: f"{e:.2e}" for k_, e in errs.items()}, flush=True)
    assert errs["y"] <= tol and errs["dx"] <= tol
    assert errs["dw"] <= 1e-5 and errs.get("db", 0.0) <= 1e-5      # fp32 sums of exact products
    # element-wise on the fix-up rows and their neighbours (a wrong successor shows up there)
    rows = np.unique(np.clip(np.concatenate([plan.fix_tok, plan.fix_tok + 1, plan.fix_t, [0, n - 1]]), 0, n - 1))
    a, bq = dx.float().cpu().numpy()[rows], want_dx[rows]
    assert np.abs(a - bq).max() <= (3e-2 if dtype == "bf16" else 1e-4) * max(1.0, np.abs(bq).max())
    return y, dx, dw, db


@pytest.mark.parametrize("seed,k,dtype,c", [(0, 4, "bf16", 64), (1, 3, "bf16", 128), (2, 2, "fp32", 32), (3, 4, "fp32", 64),
                                             (4, 4, "bf16", 8), (5, 4, "fp32", 4)])
def test_random_trees_short_nodes(seed, k, dtype, c):
    """Nodes of 0..4 tokens: windows cross several nodes, branch points everywhere."""
    t = W.random_tree(950 + seed, n_nodes=40 + 10 * seed, lo=1, hi=4, n_roots=1 + seed % 2, p_zero=0.2)
    m = M.dfs_meta(t.parent, t.seg_len)
    _run_and_check(m["tok_pred"], m["n_tokens"], c, k, seed, dtype)


@pytest.mark.parametrize("silu,bias", [(False, True), (True, False), (False, False)])
def test_activation_and_bias_variants(silu, bias):
    t = W.random_tree(971, n_nodes=30, lo=1, hi=30)
    m = M.dfs_meta(t.parent, t.seg_len)
    _run_and_check(m["tok_pred"], m["n_tokens"], 128, 4, 7, "bf16", silu=silu, bias=bias)


def test_many_tiles_ragged_tail_and_reproducible():
    """Several thousand tokens (many token tiles, a ragged last one), a few hundred channels."""
    t = W.random_tree(981, n_nodes=60, lo=20, hi=200)
    m = M.dfs_meta(t.parent, t.seg_len)
    n = m["n_tokens"]
    assert n % 64 != 0
    y, dx, dw, db = _run_and_check(m["tok_pred"], n, 328, 4, 11, "bf16")
    y2, dx2, dw2, db2 = _run_and_check(m["tok_pred"], n, 328, 4, 11, "bf16")
    for a, b in ((y, y2), (dx, dx2), (dw, dw2), (db, db2)):
        assert torch.equal(a, b)


def test_strided_rows_and_chain():
    """x and dy as column slices of wider buffers; a plain chain equals a library causal conv1d."""
    n, c, k = 700, 64, 4
    tok_pred = np.arange(-1, n - 1, dtype=np.int32)
    x, dy, w, b = _inputs(n, 2 * c, k, 3, "bf16")
    xs, dys = x.cuda()[:, c:], dy.cuda()[:, :c]
    w, b = w[:c].contiguous(), b[:c].contiguous()
    pred_d = torch.from_numpy(tok_pred).cuda()
    plan = T.tree_conv_plan(tok_pred, k)
    assert len(plan.fix_tok) == 0
    print("[case] tree conv strided rows, chain", flush=True)
    y = T.tree_conv_fwd(xs, w.cuda(), b.cuda(), pred_d)
    dx, dw, db = T.tree_conv_bwd(xs, w.cuda(), b.cuda(), pred_d, dys, plan)
    torch.cuda.synchronize()
    xt = x[:, c:].double().requires_grad_(True)
    wt, bt = w.double().requires_grad_(True), b.double().requires_grad_(True)
    z = torch.nn.functional.conv1d(torch.nn.functional.pad(xt.T[None], (k - 1, 0)), wt[:, None, :], bt, groups=c)[0].T
    ref = torch.nn.functional.silu(z)
    (ref * dy[:, :c].double()).sum().backward()
    assert rel_l2(y.float().cpu().numpy(), ref.detach().numpy()) <= 4e-3
    assert rel_l2(dx.float().cpu().numpy(), xt.grad.numpy()) <= 4e-3
    assert rel_l2(dw.cpu().numpy(), wt.grad.numpy()) <= 1e-5 and rel_l2(db.cpu().numpy(), bt.grad.numpy()) <= 1e-5


def test_errors():
    x = torch.zeros((8, 16), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((16, 5), dtype=torch.float32, device="cuda")
    pred = torch.arange(-1, 7, dtype=torch.int32, device="cuda")
    with pytest.raises(T.TreeTrainError) as e:
        T.tree_conv_fwd(x, w, None, pred)
    assert e.value.status == -8
    w = torch.zeros((12, 4), dtype=torch.float32, device="cuda")
    with pytest.raises(T.TreeTrainError) as e:
        T.tree_conv_fwd(x[:, :12], w, None, pred)
    assert e.value.status == -2
