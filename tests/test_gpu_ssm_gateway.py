"""GPU: the SSM side of the partition gateway (Appendix "SSM State Gateway").  A tree is cut into
partitions by the library's planner; every partition runs the gated delta rule starting from the end
state captured at its cut node in the parent partition, and the tree convolution with the parent's
last K-1 effective tokens handed over as a context node.  Stitched results must equal the oracle on
the whole tree, which knows nothing about partitions."""
import numpy as np
import pytest
import torch

import paper_2511_00413_amd as T
import workloads as W
from oracle import meta as M
from oracle import ssm as S
from tt_testutil import rel_l2

pytestmark = pytest.mark.gpu


def _partitions(tree, cap):
    plan = T.tree_partition_plan(tree.parent, tree.seg_len, cap)
    parts = [plan.part_nodes[plan.part_node_off[p]:plan.part_node_off[p + 1]].tolist() for p in range(plan.n_parts)]
    return plan, parts


@pytest.mark.parametrize("seed,cap", [(0, 400), (1, 250), (2, 600)])
def test_gdn_state_gateway(seed, cap):
    tree = W.random_tree(990 + seed, n_nodes=14, lo=10, hi=180)
    whole = M.dfs_meta(tree.parent, tree.seg_len)
    n, hk, hv = whole["n_tokens"], 1, 2
    g_ = torch.Generator().manual_seed(seed)
    q = torch.randn((n, hk, 128), generator=g_); k = torch.randn((n, hk, 128), generator=g_)
    q = (q / q.norm(dim=-1, keepdim=True)).to(torch.bfloat16)
    k = (k / k.norm(dim=-1, keepdim=True)).to(torch.bfloat16)
    v = torch.randn((n, hv, 128), generator=g_).to(torch.bfloat16)
    g = -(torch.rand((n, hv), generator=g_) * 0.2 + 0.005)
    beta = torch.rand((n, hv), generator=g_) * 0.8 + 0.1
    want = S.gdn_tree(q, k, v, g, beta, whole["tok_pred"])
    plan, parts = _partitions(tree, cap)
    assert plan.n_parts >= 3
    print(f"[case] gdn state gateway seed={seed} cap={cap}: {plan.n_parts} partitions, N={n}", flush=True)
    got = np.zeros((n, hv, 128))
    cut_state = {}                                   # cut node -> its end state [hv, 128, 128] on the device
    for p, part in enumerate(parts):
        local = {nid: i for i, nid in enumerate(part)}
        lparent = [-1 if nid == part[0] else local[int(tree.parent[nid])] for nid in part]
        lseg = [int(tree.seg_len[nid]) for nid in part]
        own = torch.from_numpy(plan.own_tok[plan.part_tok_off[p]:plan.part_tok_off[p + 1]].astype(np.int64))
        # this partition's cut nodes: nodes with a child in another partition
        cuts = sorted({int(tree.parent[c]) for c in range(len(tree.parent))
                       if int(tree.parent[c]) in local and plan.part_of_node[c] != p})
        cn = int(plan.part_cut_node[p])
        init = cut_state[cn] if cn >= 0 else None
        gplan = T.tree_gdn_plan(lparent, lseg, capture_nodes=[local[c] for c in cuts])
        o, states = T.tree_gdn_fwd(q[own].cuda(), k[own].cuda(), v[own].cuda(), g[own].cuda(), beta[own].cuda(), gplan,
                                   initial_state=init, return_states=True)
        torch.cuda.synchronize()
        got[own.numpy()] = o.float().cpu().numpy()
        for i, c in enumerate(cuts):
            cut_state[c] = states[i].contiguous()
    e = rel_l2(got, want)
    print(f"   rel-L2 {e:.2e}", flush=True)
    assert e <= 2e-2, e


@pytest.mark.parametrize("seed,cap", [(0, 400), (1, 250)])
def test_gdn_state_gateway_backward(seed, cap):
    """Backward through the gateway: partitions run in reverse, a child partition returns the gradient of the
    state it started from, and the parent partition takes the sum over the children at each cut node as the
    upstream gradient of that captured state.  Stitched gradients must equal the whole-tree oracle."""
    tree = W.random_tree(990 + seed, n_nodes=14, lo=10, hi=180)
    whole = M.dfs_meta(tree.parent, tree.seg_len)
    n, hk, hv = whole["n_tokens"], 1, 2
    g_ = torch.Generator().manual_seed(seed)
    q = torch.randn((n, hk, 128), generator=g_); k = torch.randn((n, hk, 128), generator=g_)
    q = (q / q.norm(dim=-1, keepdim=True)).to(torch.bfloat16)
    k = (k / k.norm(dim=-1, keepdim=True)).to(torch.bfloat16)
    v = torch.randn((n, hv, 128), generator=g_).to(torch.bfloat16)
    g = -(torch.rand((n, hv), generator=g_) * 0.2 + 0.005)
    beta = torch.rand((n, hv), generator=g_) * 0.8 + 0.1
    d_o = torch.randn((n, hv, 128), generator=g_).to(torch.bfloat16)
    want = S.gdn_tree_bwd(q.float().numpy(), k.float().numpy(), v.float().numpy(), g.numpy(), beta.numpy(), whole["tok_pred"],
                          d_o.float().numpy())
    plan, parts = _partitions(tree, cap)
    assert plan.n_parts >= 3
    print(f"[case] gdn state gateway backward seed={seed} cap={cap}: {plan.n_parts} partitions, N={n}", flush=True)
    cut_state, runs = {}, []
    for p, part in enumerate(parts):                 # forward: capture the cut nodes' end states
        local = {nid: i for i, nid in enumerate(part)}
        lparent = [-1 if nid == part[0] else local[int(tree.parent[nid])] for nid in part]
        lseg = [int(tree.seg_len[nid]) for nid in part]
        own = torch.from_numpy(plan.own_tok[plan.part_tok_off[p]:plan.part_tok_off[p + 1]].astype(np.int64))
        cuts = sorted({int(tree.parent[c]) for c in range(len(tree.parent))
                       if int(tree.parent[c]) in local and plan.part_of_node[c] != p})
        cn = int(plan.part_cut_node[p])
        gplan = T.tree_gdn_plan(lparent, lseg, capture_nodes=[local[c] for c in cuts])
        dev = [t[own].cuda() for t in (q, k, v, g, beta)]
        _, states = T.tree_gdn_fwd(*dev, gplan, initial_state=cut_state[cn] if cn >= 0 else None, return_states=True)
        for i, c in enumerate(cuts):
            cut_state[c] = states[i].contiguous()
        runs.append((own, cuts, cn, gplan, dev))
    got = [np.zeros((n, hk, 128)), np.zeros((n, hk, 128)), np.zeros((n, hv, 128)), np.zeros((n, hv)), np.zeros((n, hv))]
    d_cut = {}                                       # cut node -> summed gradient of its end state
    for own, cuts, cn, gplan, dev in reversed(runs):  # children before parents
        up = torch.stack([d_cut[c] for c in cuts]) if cuts else None
        out = T.tree_gdn_bwd(*dev, d_o[own].cuda(), gplan, initial_state=cut_state[cn] if cn >= 0 else None, d_state_out=up,
                             want_d_initial_state=cn >= 0)
        torch.cuda.synchronize()
        for dstt, t in zip(got, out[:5]):
            dstt[own.numpy()] = t.float().cpu().numpy()
        if cn >= 0:
            d_cut[cn] = d_cut[cn] + out[5] if cn in d_cut else out[5]
    for name, a, b, tol in zip(("dq", "dk", "dv", "dg", "dbeta"), got, want, (8e-3, 8e-3, 8e-3, 8e-3, 8e-3)):
        e = rel_l2(a, b)
        print(f"   {name}: rel-L2 {e:.2e}", flush=True)
        assert e <= tol, (name, e)


@pytest.mark.parametrize("seed,cap,K", [(0, 120, 4), (1, 60, 3)])
def test_conv_context_gateway(seed, cap, K):
    """The convolution needs no extra entry point: the parent's last K-1 effective tokens become a context
    node in front of the partition's root; its output rows are dropped and its dx rows are the gradient that
    flows back into the parent partition."""
    tree = W.random_tree(995 + seed, n_nodes=16, lo=1, hi=50, p_zero=0.1)
    whole = M.dfs_meta(tree.parent, tree.seg_len)
    n, C = whole["n_tokens"], 32
    g_ = torch.Generator().manual_seed(seed)
    x = torch.randn((n, C), generator=g_)
    dy = torch.randn((n, C), generator=g_)
    w = torch.randn((C, K), generator=g_) * 0.5
    b = torch.randn(C, generator=g_) * 0.1
    want_y, _ = S.tree_conv(x, w, b, whole["tok_pred"])
    want_dx, want_dw, want_db = S.tree_conv_bwd(x, w, b, whole["tok_pred"], dy)
    plan, parts = _partitions(tree, cap)
    assert plan.n_parts >= 3
    print(f"[case] conv context gateway seed={seed} cap={cap} K={K}: {plan.n_parts} partitions, N={n}", flush=True)
    P = S.pred_chain(whole["tok_pred"], K)
    y = np.zeros((n, C)); dx = np.zeros((n, C)); dw = np.zeros((C, K)); db = np.zeros(C)
    for p, part in enumerate(parts):
        own = plan.own_tok[plan.part_tok_off[p]:plan.part_tok_off[p + 1]].astype(np.int64)
        if len(own) == 0:
            continue
        # context = the K-1 predecessors of the partition's first token on its own sequence, oldest first
        first = int(own[0])
        ctx = [int(P[m][first]) for m in range(K - 1, 0, -1) if P[m][first] >= 0]
        local = {nid: i + 1 for i, nid in enumerate(part)}
        lparent = [-1] + [0 if nid == part[0] else local[int(tree.parent[nid])] for nid in part]
        lseg = [len(ctx)] + [int(tree.seg_len[nid]) for nid in part]
        lmeta = T.tree_build_meta(lparent, lseg)
        rows = torch.from_numpy(np.concatenate([np.asarray(ctx, dtype=np.int64), own]))
        dy_loc = dy[rows].clone()
        dy_loc[:len(ctx)] = 0                        # the context rows' outputs belong to the parent partition
        pred = torch.from_numpy(lmeta.tok_pred).cuda()
        cplan = T.tree_conv_plan(lmeta.tok_pred, K)
        yl = T.tree_conv_fwd(x[rows].cuda(), w.cuda(), b.cuda(), pred)
        dxl, dwl, dbl = T.tree_conv_bwd(x[rows].cuda(), w.cuda(), b.cuda(), pred, dy_loc.cuda(), cplan)
        torch.cuda.synchronize()
        y[own] = yl.cpu().numpy()[len(ctx):]
        np.add.at(dx, rows.numpy(), dxl.cpu().numpy().astype(np.float64))      # context rows: gradient into the parent
        dw += dwl.cpu().numpy()
        db += dbl.cpu().numpy()
    for name, a, bq, tol in (("y", y, want_y, 2e-6), ("dx", dx, want_dx, 2e-6), ("dw", dw, want_dw, 1e-5), ("db", db, want_db, 1e-5)):
        e = rel_l2(a, bq)
        print(f"   {name}: rel-L2 {e:.2e}", flush=True)
        assert e <= tol, (name, e)


def test_gdn_initial_state_zero_equals_none():
    """No initial state and an explicit all-zero initial state are the same computation: every output of the
    backward, the gradient of the initial state included, must agree bit for bit."""
    tree = W.random_tree(1234, n_nodes=9, lo=5, hi=120, n_roots=2)
    whole = M.dfs_meta(tree.parent, tree.seg_len)
    n, hk, hv = whole["n_tokens"], 1, 2
    g_ = torch.Generator().manual_seed(5)
    q = torch.randn((n, hk, 128), generator=g_); k = torch.randn((n, hk, 128), generator=g_)
    q = (q / q.norm(dim=-1, keepdim=True)).to(torch.bfloat16).cuda()
    k = (k / k.norm(dim=-1, keepdim=True)).to(torch.bfloat16).cuda()
    v = torch.randn((n, hv, 128), generator=g_).to(torch.bfloat16).cuda()
    g = (-(torch.rand((n, hv), generator=g_) * 0.2 + 0.005)).cuda()
    beta = (torch.rand((n, hv), generator=g_) * 0.8 + 0.1).cuda()
    d_o = torch.randn((n, hv, 128), generator=g_).to(torch.bfloat16).cuda()
    plan = T.tree_gdn_plan(tree.parent, tree.seg_len)
    print(f"[case] gdn zero initial state: N={n}, {plan.n_chunks} chunks", flush=True)
    a = T.tree_gdn_bwd(q, k, v, g, beta, d_o, plan, want_d_initial_state=True)
    zero = torch.zeros((hv, 128, 128), dtype=torch.float32, device="cuda")
    b = T.tree_gdn_bwd(q, k, v, g, beta, d_o, plan, initial_state=zero, want_d_initial_state=True)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    assert torch.isfinite(a[5]).all() and float(a[5].abs().max()) > 0      # two roots send gradient into it
