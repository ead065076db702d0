"""GPU parity at the benchmark configurations' full sizes, in the launch configuration bench.py
times.  The per-branch oracle is too slow to run in full there, so it is evaluated (a) for one
complete key/value head group on config 2 and (b) for sampled outputs elsewhere: O / LSE / dQ rows of
sampled query tokens and dK / dV of sampled key tokens (the oracle then evaluates every query that
can see the key).  For the cached-prefix step of config 5 the prefix gradients are additionally
checked through the column-sum identity sum_j dV_j = sum_i dO_i (softmax rows sum to one).
Keys near the root, which tens of thousands of queries see and whose gradients go through the cut
tiles' partial sums, are checked with an upstream gradient that is zero outside a sample of query
rows (test_large_configs_trunk_keys).  Every comparison asserts the whole-sample relative L2 and the
largest per-row error (tt_testutil.ATTN_TOL)."""
import numpy as np
import pytest
import torch

import paper_2511_00413_amd as T
import workloads as W
from oracle import attention as A
from oracle import meta as M
from tt_testutil import assert_attention_close, dq_allowance, rel_l2

pytestmark = pytest.mark.gpu
TOL = dict(o=1e-2, lse=1e-2, dq=2e-2, dk=2e-2, dv=2e-2)


def _run_gpu(meta, q, k, v, do, kp=None, vp=None):
    from gpu_util import dev
    kend, kmin, kmax = dev(meta.kend), dev(meta.ktile_kend_min), dev(meta.ktile_kend_max)
    qd, kd, vd, dod = dev(q), dev(k), dev(v), dev(do)
    kpd = vpd = dkp = dvp = None
    if kp is not None:
        kpd, vpd = dev(kp), dev(vp)
        dkp = torch.zeros(kp.shape, dtype=torch.float32, device="cuda")
        dvp = torch.zeros(kp.shape, dtype=torch.float32, device="cuda")
    o, lse = T.tree_attn_fwd(qd, kd, vd, kend, kmin, kmax, k_prefix=kpd, v_prefix=vpd)
    dq, dk, dv = T.tree_attn_bwd(qd, kd, vd, kend, kmin, kmax, o, dod, lse, k_prefix=kpd, v_prefix=vpd,
                                 dk_prefix_acc=dkp, dv_prefix_acc=dvp)
    torch.cuda.synchronize()
    return dict(o=o, lse=lse, dq=dq, dk=dk, dv=dv, dkp=dkp, dvp=dvp)


def _sample_check(om, got, q, k, v, do, kvh, rows, keys, G, offset=0):
    """rows / keys are oracle token ids; `offset` maps them to the GPU's own-token index."""
    s = A.rows(om, q, k, v, do, kvh, rows, keys)
    hs = slice(kvh * G, kvh * G + G)
    ridx = torch.tensor([r - offset for r in rows], device="cuda")
    mine = dict(o=got["o"][ridx][:, hs].float().cpu().numpy(), lse=got["lse"][hs][:, ridx].T.cpu().numpy(),
                dq=got["dq"][ridx][:, hs].float().cpu().numpy())
    want = dict(o=s["o"], lse=s["lse"], dq=s["dq"])
    if len(keys):
        kidx = torch.tensor([j - offset for j in keys], device="cuda")
        mine["dk"], mine["dv"] = got["dk"][kidx][:, kvh].float().cpu().numpy(), got["dv"][kidx][:, kvh].float().cpu().numpy()
        want["dk"], want["dv"] = s["dk"], s["dv"]
    kmax = float(np.linalg.norm(k[:, kvh].numpy(), axis=-1).max())
    allow = dq_allowance(do[rows][:, hs].numpy(), s["o"], kmax, k.shape[-1] ** -0.5, "bf16")
    assert_attention_close(mine, want, "bf16",
                           f"kvh {kvh}: rows {len(rows)} keys {len(keys)} (oracle evaluated {s['n_rows_evaluated']} rows)",
                           dq_allow=allow)


def test_cfg2_full_group_and_samples():
    tree, dims = W.tree_config(2), W.DIMS[2]
    meta = T.tree_build_meta(tree.parent, tree.seg_len, tree.trained)
    om = M.dfs_meta(tree.parent, tree.seg_len, tree.trained)
    n = meta.n_tokens
    print(f"[case] cfg2 full size N={n}", flush=True)
    q, k, v, do = W.attn_inputs(n, n, dims, 2)
    got = _run_gpu(meta, q, k, v, do)
    qf, kf, vf, dof = q.float(), k.float(), v.float(), do.float()
    G = dims.hq // dims.hkv
    want = A.branches(om, qf, kf, vf, dof, kv_heads=[0])
    mine = dict(o=got["o"][:, :G].float().cpu().numpy(), lse=got["lse"][:G].cpu().numpy(),
                dq=got["dq"][:, :G].float().cpu().numpy(), dk=got["dk"][:, 0].float().cpu().numpy(),
                dv=got["dv"][:, 0].float().cpu().numpy())
    ref = dict(o=want["o"][:, :G], lse=want["lse"][:G], dq=want["dq"][:, :G], dk=want["dk"][:, 0], dv=want["dv"][:, 0])
    kmax = float(np.linalg.norm(kf[:, 0].numpy(), axis=-1).max())
    assert_attention_close(mine, ref, "bf16", "complete kv group 0",
                           dq_allow=dq_allowance(dof[:, :G].numpy(), ref["o"], kmax, dims.d ** -0.5, "bf16"))
    # other groups: sampled rows at tile edges and node boundaries, keys in leaves
    ns, ne = om["node_start"], om["node_end"]
    rows = sorted({0, 63, 64, 127, 128, int(ns[1]), int(ne[1]) - 1, int(ns[-1]), n - 1, n // 2})
    leaf = int(np.argmax(om["node_g"] == 1))
    keys = [int(ns[leaf]), int(ne[leaf]) - 1, int(ns[-1]) + 5]
    _sample_check(om, got, qf, kf, vf, dof, 5, rows, keys, G)


@pytest.mark.parametrize("cfg", [3, 4])
def test_large_configs_sampled(cfg):
    tree, dims = W.tree_config(cfg), W.DIMS[cfg]
    meta = T.tree_build_meta(tree.parent, tree.seg_len, tree.trained)
    om = M.dfs_meta(tree.parent, tree.seg_len, tree.trained)
    n = meta.n_tokens
    print(f"[case] cfg{cfg} full size N={n}", flush=True)
    q, k, v, do = W.attn_inputs(n, n, dims, cfg)
    got = _run_gpu(meta, q, k, v, do)
    qf, kf, vf, dof = q.float(), k.float(), v.float(), do.float()
    G = dims.hq // dims.hkv
    ns, ne = om["node_start"], om["node_end"]
    last = om["n_nodes"] - 1
    rows = sorted({0, 127, 128, int(ne[0]) - 1, int(ns[1]), int(ns[last]), n - 1, int(ns[last // 2]) + 3,
                   int(ne[last // 2]) - 1})
    # keys whose visible queries are few enough for the oracle: inside the last leaf and at its start
    leaf_rk = max(rk for rk in range(om["n_nodes"]) if om["node_g"][rk] == 1 and ne[rk] - ns[rk] > 16)
    keys = [int(ne[leaf_rk]) - 1, int(ne[leaf_rk]) - 200 if ne[leaf_rk] - ns[leaf_rk] > 200 else int(ns[leaf_rk])]
    _sample_check(om, got, qf, kf, vf, dof, dims.hkv - 1, rows, keys, G)
    _sample_check(om, got, qf, kf, vf, dof, 0, rows[:4], [], G)
    # column-sum identity over all keys (every branch, every head of the group)
    dv_sum = got["dv"].float().sum(dim=0).cpu().numpy()                       # [hkv, d]
    do_sum = do.float().view(n, dims.hkv, G, dims.d).sum(dim=(0, 2)).numpy()
    assert rel_l2(dv_sum, do_sum) <= 2e-2


@pytest.mark.parametrize("cfg", [2, 3, 4])
def test_large_configs_trunk_keys(cfg):
    """dK / dV of keys near the root at full size.  Such a key is seen by every query of its subtree, too
    many for the oracle; but every term of its gradient carries a factor dO_i (Eq. 5), so with an
    upstream gradient that is zero outside a sample of query rows the sample's contributions are the
    whole gradient.  The GPU call is the ordinary full-size backward (all tiles, all chunks of the cut
    tiles, the ordered reduce); only d_o differs.  The sampled rows are spread over the whole subtree so
    that every chunk of the trunk's tiles contributes."""
    tree, dims = W.tree_config(cfg), W.DIMS[cfg]
    meta = T.tree_build_meta(tree.parent, tree.seg_len, tree.trained)
    om = M.dfs_meta(tree.parent, tree.seg_len, tree.trained)
    n = meta.n_tokens
    q, k, v, do = W.attn_inputs(n, n, dims, cfg)
    rng = np.random.default_rng(100 + cfg)
    ns, ne = om["node_start"], om["node_end"]
    n_rows = 96 if cfg == 2 else 48
    rows = np.unique(np.concatenate([rng.choice(n, n_rows, replace=False), [0, int(ne[0]) - 1, int(ns[1]), n - 1]]))
    do_masked = torch.zeros_like(do)
    do_masked[torch.from_numpy(rows)] = do[torch.from_numpy(rows)]
    print(f"[case] cfg{cfg} trunk keys, N={n}, d_o non-zero on {len(rows)} rows", flush=True)
    got = _run_gpu(meta, q, k, v, do_masked)
    G = dims.hq // dims.hkv
    # keys of the root node (first, a tile edge, last) and of the first child (seen by its subtree only)
    keys = sorted({0, 63, 64, int(ne[0]) // 2, int(ne[0]) - 1, int(ns[1]), int(ne[1]) - 1})
    for kvh in (0, dims.hkv - 1):
        s = A.rows(om, q.float(), k.float(), v.float(), do_masked.float(), kvh, [int(r) for r in rows], keys,
                   complete_keys=False)
        kidx = torch.tensor(keys, device="cuda")
        mine = dict(dk=got["dk"][kidx][:, kvh].float().cpu().numpy(), dv=got["dv"][kidx][:, kvh].float().cpu().numpy())
        assert_attention_close(mine, dict(dk=s["dk"], dv=s["dv"]), "bf16", f"kvh {kvh}: {len(keys)} trunk keys")
    # rows outside the sample have zero upstream gradient: their dQ is exactly zero
    outside = np.setdiff1d(np.arange(n), rows)[:: max(1, n // 512)]
    assert float(got["dq"][torch.from_numpy(outside).cuda()].float().abs().max()) == 0.0


def test_cfg5_partition_step_sampled():
    step, dims = W.step_cfg5(), W.DIMS[5]
    nvis = int(step.prefix_visible.sum())
    meta = T.tree_build_meta(step.chunk.parent, step.chunk.seg_len, step.chunk.trained, n_prefix=step.n_prefix,
                             prefix_visible=step.prefix_visible, root_pos_offset=[nvis])
    n, P = meta.n_tokens, step.n_prefix
    print(f"[case] cfg5 step N={n} P={P} visible={nvis}", flush=True)
    q, k, v, do = W.attn_inputs(n, n, dims, 5)
    _, kp, vp, _ = W.attn_inputs(1, P, dims, 105)
    got = _run_gpu(meta, q, k, v, do, kp, vp)
    # equivalent whole tree for the oracle: one root node holding the visible prefix tokens
    parent = np.concatenate([[-1], np.where(step.chunk.parent < 0, 0, step.chunk.parent + 1)]).astype(np.int32)
    seg = np.concatenate([[nvis], step.chunk.seg_len]).astype(np.int32)
    om = M.dfs_meta(parent, seg)
    sel = torch.from_numpy(np.nonzero(step.prefix_visible)[0])
    G = dims.hq // dims.hkv
    qw = torch.cat([torch.zeros(nvis, dims.hq, dims.d), q.float()])
    dow = torch.cat([torch.zeros(nvis, dims.hq, dims.d), do.float()])
    kw = torch.cat([kp.float()[sel], k.float()])
    vw = torch.cat([vp.float()[sel], v.float()])
    ns, ne = om["node_start"], om["node_end"]
    rows = sorted({nvis, nvis + 127, nvis + 128, int(ns[2]), int(ne[2]) - 1, nvis + n - 1, nvis + n // 2})
    keys = [nvis + n - 1, int(ns[-1]), int(ne[-2]) - 1]          # keys of the last two (leaf) nodes
    _sample_check(om, got, qw, kw, vw, dow, 3, rows, keys, G, offset=nvis)
    # prefix gradients: hidden keys untouched, and the column-sum identity over prefix + own keys
    hidden = torch.from_numpy(np.nonzero(step.prefix_visible == 0)[0]).cuda()
    assert float(got["dkp"][hidden].abs().max()) == 0.0 and float(got["dvp"][hidden].abs().max()) == 0.0
    dv_sum = (got["dv"].float().sum(dim=0) + got["dvp"].sum(dim=0)).cpu().numpy()
    do_sum = do.float().view(n, dims.hkv, G, dims.d).sum(dim=(0, 2)).numpy()
    assert rel_l2(dv_sum, do_sum) <= 2e-2


def test_more_than_4096_key_tiles():
    """A sequence longer than 4096 key tiles (262144 keys): the forward / dQ kernels classify their
    candidate tiles in several chunks, and the dK/dV planner cuts the long visible ranges."""
    # trunk, two leaves below it, then a second root whose queries skip every earlier tile
    parent = np.array([-1, 0, 0, -1], dtype=np.int32)
    seg = np.array([255000, 6100, 4037, 1500], dtype=np.int32)
    tree = W.Tree(parent=parent, seg_len=seg, trained=np.ones(4, dtype=np.uint8), name="long-trunk")
    dims = W.AttnDims(2, 1, 128, "bf16", 0.5)
    meta = T.tree_build_meta(tree.parent, tree.seg_len, tree.trained)
    om = M.dfs_meta(tree.parent, tree.seg_len, tree.trained)
    n = meta.n_tokens
    assert n > 4096 * 64
    print(f"[case] long trunk N={n}", flush=True)
    q, k, v, do = W.attn_inputs(n, n, dims, 77)
    got = _run_gpu(meta, q, k, v, do)
    qf, kf, vf, dof = q.float(), k.float(), v.float(), do.float()
    ns, ne = om["node_start"], om["node_end"]
    rows = sorted({0, 4096 * 64 - 1, 4096 * 64, int(ne[0]) - 1, int(ns[1]) + 7, int(ne[1]) - 1, int(ns[2]), int(ne[2]) - 1,
                   int(ns[3]), n - 1})
    keys = [int(ne[1]) - 1, int(ne[2]) - 3, int(ns[3]), n - 1]        # few queries see these
    _sample_check(om, got, qf, kf, vf, dof, 0, rows, keys, 2)
    dv_sum = got["dv"].float().sum(dim=0).cpu().numpy()
    do_sum = do.float().view(n, 1, 2, dims.d).sum(dim=(0, 2)).numpy()
    assert rel_l2(dv_sum, do_sum) <= 2e-2


# ---- the later entry points at config 2's full size, in the launch configurations bench.py times ----

def test_cfg2_partitioned_quarter_capacity():
    """bench.py's partitioned leg: config 2 cut at 5120 tokens; against the whole-tree call on the same
    tensors and against the oracle on sampled rows / keys."""
    t = W.tree_config(2)
    d = W.DIMS[2]
    meta = T.tree_build_meta(t.parent, t.seg_len, t.trained)
    om = M.dfs_meta(t.parent, t.seg_len, t.trained)
    n = meta.n_tokens
    q, k, v, do = W.attn_inputs(n, n, d, 2)
    plan = T.tree_partition_plan(t.parent, t.seg_len, 5120).to_device()
    print(f"[case] cfg2 partitioned, capacity 5120: {plan.n_parts} partitions", flush=True)
    qd, kd, vd, dod = (x.cuda() for x in (q, k, v, do))
    o, lse = T.tree_attn_partitioned_fwd(qd, kd, vd, plan)
    dq, dk, dv = T.tree_attn_partitioned_bwd(qd, kd, vd, plan, o, dod, lse)
    torch.cuda.synchronize()
    got = dict(o=o, lse=lse, dq=dq, dk=dk, dv=dv)
    whole = _run_gpu(meta, q, k, v, do)
    # the partitioned run against the whole-tree call of the same library: both carry bf16 rounding, so
    # the whole-tensor bound applies (the per-row comparison is against the oracle, below)
    for key in TOL:
        e = rel_l2(got[key].float().cpu().numpy(), whole[key].float().cpu().numpy())
        assert e <= TOL[key], (key, e)
    rng = np.random.default_rng(12)
    rows = sorted(rng.choice(n, 24, replace=False).tolist())
    keys = sorted(rng.choice(n, 6, replace=False).tolist())
    _sample_check(om, got, q.float(), k.float(), v.float(), do.float(), 3, rows, keys, d.hq // d.hkv)


def test_cfg2_tree_conv_sampled_channels():
    """bench.py's tree_conv leg: N = 16406, C = 8192, K = 4, bf16.  The convolution is depthwise, so the
    oracle is run on 48 sampled channels (all tokens); dweight / dbias of those channels as well."""
    from oracle import ssm as S
    t = W.tree_config(2)
    meta = T.tree_build_meta(t.parent, t.seg_len, t.trained)
    n, C, K = meta.n_tokens, 8192, 4
    g = torch.Generator().manual_seed(21)
    x = torch.randn((n, C), generator=g).to(torch.bfloat16)
    dy = torch.randn((n, C), generator=g).to(torch.bfloat16)
    w = torch.randn((C, K), generator=g) * 0.5
    b = torch.randn(C, generator=g) * 0.1
    pred = torch.from_numpy(meta.tok_pred).cuda()
    plan = T.tree_conv_plan(meta.tok_pred, K)
    print(f"[case] cfg2 tree conv full size: {len(plan.fix_tok)} fix-up tokens", flush=True)
    y = T.tree_conv_fwd(x.cuda(), w.cuda(), b.cuda(), pred)
    dx, dw, db = T.tree_conv_bwd(x.cuda(), w.cuda(), b.cuda(), pred, dy.cuda(), plan)
    torch.cuda.synchronize()
    ch = np.sort(np.random.default_rng(4).choice(C, 48, replace=False))
    cht = torch.from_numpy(ch)
    want_y, _ = S.tree_conv(x[:, cht], w[cht], b[cht], meta.tok_pred)
    want_dx, want_dw, want_db = S.tree_conv_bwd(x[:, cht], w[cht], b[cht], meta.tok_pred, dy[:, cht])
    assert rel_l2(y[:, cht.cuda()].float().cpu().numpy(), want_y) <= 4e-3
    assert rel_l2(dx[:, cht.cuda()].float().cpu().numpy(), want_dx) <= 4e-3
    assert rel_l2(dw[cht.cuda()].cpu().numpy(), want_dw) <= 1e-4          # fp32 sums over 16 406 tokens
    assert rel_l2(db[cht.cuda()].cpu().numpy(), want_db) <= 1e-4
    rows = np.unique(np.concatenate([plan.fix_tok, plan.fix_t]))
    a, bq = dx[:, cht.cuda()].float().cpu().numpy()[rows], want_dx[rows]
    assert np.abs(a - bq).max() <= 3e-2 * max(1.0, np.abs(bq).max())


def test_cfg2_gdn_sampled_heads():
    """bench.py's tree_gdn leg: N = 16406, 16 key / 32 value heads; the token recurrence is run for two
    sampled value heads."""
    from oracle import ssm as S
    t = W.tree_config(2)
    meta = T.tree_build_meta(t.parent, t.seg_len, t.trained)
    n, hk, hv = meta.n_tokens, 16, 32
    g_ = torch.Generator().manual_seed(22)
    q = torch.randn((n, hk, 128), generator=g_); k = torch.randn((n, hk, 128), generator=g_)
    q = (q / q.norm(dim=-1, keepdim=True)).to(torch.bfloat16)
    k = (k / k.norm(dim=-1, keepdim=True)).to(torch.bfloat16)
    v = torch.randn((n, hv, 128), generator=g_).to(torch.bfloat16)
    gl = -(torch.rand((n, hv), generator=g_) * 0.2 + 0.005)
    beta = torch.rand((n, hv), generator=g_) * 0.8 + 0.1
    plan = T.tree_gdn_plan(t.parent, t.seg_len)
    print(f"[case] cfg2 gdn full size: {plan.n_chunks} chunks, {plan.n_slots} saved states", flush=True)
    o = T.tree_gdn_fwd(q.cuda(), k.cuda(), v.cuda(), gl.cuda(), beta.cuda(), plan)
    torch.cuda.synchronize()
    o = o.float().cpu().numpy()
    for h in (7, 30):
        want = S.gdn_tree(q[:, h // 2:h // 2 + 1], k[:, h // 2:h // 2 + 1], v[:, h:h + 1], gl[:, h:h + 1], beta[:, h:h + 1],
                          meta.tok_pred)
        e = rel_l2(o[:, h], want[:, 0])
        print(f"   head {h}: rel-L2 {e:.2e}", flush=True)
        assert e <= 2e-2, (h, e)


def test_cfg2_gdn_backward_one_key_head():
    """bench.py's tree_gdn leg, backward: N = 16406, 16 key / 32 value heads; the reverse recurrence is run for
    the two value heads of one key head (dq and dk are sums over them)."""
    from oracle import ssm as S
    t = W.tree_config(2)
    meta = T.tree_build_meta(t.parent, t.seg_len, t.trained)
    n, hk, hv = meta.n_tokens, 16, 32
    g_ = torch.Generator().manual_seed(23)
    q = torch.randn((n, hk, 128), generator=g_); k = torch.randn((n, hk, 128), generator=g_)
    q = (q / q.norm(dim=-1, keepdim=True)).to(torch.bfloat16)
    k = (k / k.norm(dim=-1, keepdim=True)).to(torch.bfloat16)
    v = torch.randn((n, hv, 128), generator=g_).to(torch.bfloat16)
    gl = -(torch.rand((n, hv), generator=g_) * 0.2 + 0.005)
    beta = torch.rand((n, hv), generator=g_) * 0.8 + 0.1
    d_o = torch.randn((n, hv, 128), generator=g_).to(torch.bfloat16)
    plan = T.tree_gdn_plan(t.parent, t.seg_len)
    print(f"[case] cfg2 gdn backward full size: {plan.n_chunks} chunks, {plan.n_slots} saved states", flush=True)
    got = T.tree_gdn_bwd(q.cuda(), k.cuda(), v.cuda(), gl.cuda(), beta.cuda(), d_o.cuda(), plan)
    torch.cuda.synchronize()
    kh = 5
    hs = slice(2 * kh, 2 * kh + 2)
    want = S.gdn_tree_bwd(q[:, kh:kh + 1].float().numpy(), k[:, kh:kh + 1].float().numpy(), v[:, hs].float().numpy(),
                          gl[:, hs].numpy(), beta[:, hs].numpy(), meta.tok_pred, d_o[:, hs].float().numpy())
    sel = (got[0][:, kh:kh + 1], got[1][:, kh:kh + 1], got[2][:, hs], got[3][:, hs], got[4][:, hs])
    for name, a, b, tol in zip(("dq", "dk", "dv", "dg", "dbeta"), sel, want, (8e-3, 8e-3, 8e-3, 8e-3, 8e-3)):
        e = rel_l2(a.float().cpu().numpy(), b)
        print(f"   {name}: rel-L2 {e:.2e}", flush=True)
        assert e <= tol, (name, e)
