"""Redundancy-free tree partitioning, end to end through the C ABI: a tree is cut into connected
subtrees at node boundaries; every partition attends to the cached K/V of its ancestors' partition
(with the non-ancestor part of the cached slice masked), gradients for the cached keys come back
through the fp32 accumulators, and the stitched result must equal the oracle run on the whole tree
(which knows nothing about partitions).  The first group of tests stitches the partitions by hand on the
host (its own small packer and gateway bookkeeping); the second group runs the library's planner and
its one-call driver."""
import numpy as np
import pytest
import torch

import paper_2511_00413_amd as T
import workloads as W
from oracle import attention as A
from oracle import meta as M
from tt_testutil import rel_l2

pytestmark = pytest.mark.gpu


def greedy_partitions(parent, seg_len, cap):
    n = len(parent)
    kids = [[] for _ in range(n)]
    roots = []
    for i, p in enumerate(parent):
        (roots if p < 0 else kids[p]).append(i)
    parts = []          # each: list of node ids in DFS order, first is the partition root

    def grow(part, size, node):
        part.append(node)
        size += int(seg_len[node])
        for c in kids[node]:
            if size + int(seg_len[c]) <= cap:
                size = grow(part, size, c)
            else:
                pending.append(c)
        return size

    pending = list(roots)
    while pending:
        r = pending.pop(0)
        part = []
        grow(part, 0, r)
        parts.append(part)
    return parts


@pytest.mark.parametrize("seed,cap,dtype", [(3, 700, "bf16"), (5, 300, "bf16"), (7, 500, "fp32")])
def test_stitched_partitions_equal_whole_tree(seed, cap, dtype):
    tree = W.random_tree(200 + seed, n_nodes=14, lo=20, hi=260, shuffle=False)
    d = 128 if dtype == "bf16" else 64
    dims = W.AttnDims(4, 2, d, dtype, 0.5 if dtype == "bf16" else 1.0)
    whole = M.dfs_meta(tree.parent, tree.seg_len, tree.trained)
    n = whole["n_tokens"]
    q, k, v, do = W.attn_inputs(n, n, dims, seed)           # whole-tree DFS order
    want = A.branches(whole, q.float(), k.float(), v.float(), do.float())

    rank = {int(nid): rk for rk, nid in enumerate(whole["dfs_order"])}
    node_tokens = lambda nid: np.arange(whole["node_start"][rank[nid]], whole["node_end"][rank[nid]])
    parts = greedy_partitions(list(tree.parent), list(tree.seg_len), cap)
    assert len(parts) >= 3
    print(f"[case] partitions seed={seed} cap={cap} {dtype}: {len(parts)} partitions, N={n}", flush=True)

    got = dict(o=np.zeros((n, dims.hq, d)), lse=np.zeros((dims.hq, n)), dq=np.zeros((n, dims.hq, d)),
               dk=np.zeros((n, dims.hkv, d)), dv=np.zeros((n, dims.hkv, d)))
    ctx = {}            # partition root node -> (cached token ids, visible flags) it sees as prefix
    part_of = {}
    for pi, part in enumerate(parts):
        for nid in part:
            part_of[nid] = pi
    for part in parts:
        root = part[0]
        ctx_tok, ctx_vis = ctx.get(root, (np.zeros(0, dtype=np.int64), np.zeros(0, dtype=np.uint8)))
        # partition-local tree
        local = {nid: i for i, nid in enumerate(part)}
        lparent = [-1 if nid == root else local[int(tree.parent[nid])] for nid in part]
        lseg = [int(tree.seg_len[nid]) for nid in part]
        pos_off = int(whole["node_pos0"][rank[root]])
        g_glob = [int(whole["node_g"][rank[nid]]) for nid in part]
        ltrained = [int(tree.trained[nid]) for nid in part]
        meta = T.tree_build_meta(lparent, lseg, ltrained, root_pos_offset=[pos_off], g_override=g_glob,
                                 K_override=int(whole["K"]), n_prefix=len(ctx_tok), prefix_visible=ctx_vis)
        own = np.concatenate([node_tokens(part[i]) for i in meta.dfs_order])   # global ids, local DFS order
        assert bool(np.array_equal(meta.tok_pos, whole["tok_pos"][own])), "depth-based positions"
        assert bool(np.array_equal(meta.tok_weight, whole["tok_weight"][own])), "global g / K weights"
        sel = torch.from_numpy(own)
        dev = lambda x: x.cuda()
        kend, kmin, kmax = (torch.from_numpy(x).cuda() for x in (meta.kend, meta.ktile_kend_min, meta.ktile_kend_max))
        kp = vp = dkp = dvp = None
        if len(ctx_tok):
            csel = torch.from_numpy(ctx_tok)
            kp, vp = dev(k[csel].contiguous()), dev(v[csel].contiguous())
            dkp = torch.zeros(kp.shape, dtype=torch.float32, device="cuda")
            dvp = torch.zeros(kp.shape, dtype=torch.float32, device="cuda")
        qd, kd, vd, dod = dev(q[sel].contiguous()), dev(k[sel].contiguous()), dev(v[sel].contiguous()), dev(do[sel].contiguous())
        o, lse = T.tree_attn_fwd(qd, kd, vd, kend, kmin, kmax, k_prefix=kp, v_prefix=vp)
        dq, dk, dv = T.tree_attn_bwd(qd, kd, vd, kend, kmin, kmax, o, dod, lse, k_prefix=kp, v_prefix=vp,
                                     dk_prefix_acc=dkp, dv_prefix_acc=dvp)
        torch.cuda.synchronize()
        got["o"][own] = o.float().cpu().numpy()
        got["lse"][:, own] = lse.cpu().numpy()
        got["dq"][own] = dq.float().cpu().numpy()
        got["dk"][own] += dk.float().cpu().numpy()
        got["dv"][own] += dv.float().cpu().numpy()
        if len(ctx_tok):
            vis = ctx_vis.astype(bool)
            dkc, dvc = dkp.cpu().numpy(), dvp.cpu().numpy()
            assert np.all(dkc[~vis] == 0) and np.all(dvc[~vis] == 0)
            np.add.at(got["dk"], ctx_tok[vis], dkc[vis])
            np.add.at(got["dv"], ctx_tok[vis], dvc[vis])
        # gateways for the child partitions cut below this one: cached slice = this partition's own
        # cache + its own tokens up to the end of the cut node; visible = ancestors of the child
        for nid in part:
            for c in [x for x in range(len(tree.parent)) if int(tree.parent[x]) == nid and part_of[x] != part_of[nid]]:
                anc = set()
                a = nid
                while a in local:
                    anc.add(a)
                    a = int(tree.parent[a]) if a != root else -2
                upto = int(np.nonzero(meta.dfs_order == local[nid])[0][0])       # local DFS rank of the cut node
                toks, flags = [ctx_tok], [ctx_vis]
                for rk in range(upto + 1):
                    lid = part[int(meta.dfs_order[rk])]
                    t = node_tokens(lid)
                    toks.append(t)
                    flags.append(np.full(len(t), 1 if lid in anc else 0, dtype=np.uint8))
                ctx[c] = (np.concatenate(toks).astype(np.int64), np.concatenate(flags))
    tol = dict(o=1e-2, lse=1e-2, dq=2e-2, dk=2e-2, dv=2e-2) if dtype == "bf16" else dict.fromkeys(("o", "lse", "dq", "dk", "dv"), 1e-5)
    errs = {key: rel_l2(got[key], want[key]) for key in tol}
    print("   rel-L2:", {k_: f"{e:.2e}" for k_, e in errs.items()}, flush=True)
    for key, e in errs.items():
        assert e <= tol[key], (key, e)


# ---- the partition driver inside the library: planner + one call for the whole tree ----

def _whole_tree_case(seed, n_nodes, lo, hi, dtype, p_zero=0.0, n_roots=1, shuffle=False):
    tree = W.random_tree(seed, n_nodes=n_nodes, lo=lo, hi=hi, shuffle=shuffle, p_zero=p_zero, n_roots=n_roots)
    d = 128 if dtype == "bf16" else 64
    dims = W.AttnDims(4, 2, d, dtype, 0.5 if dtype == "bf16" else 1.0)
    whole = M.dfs_meta(tree.parent, tree.seg_len, tree.trained)
    n = whole["n_tokens"]
    q, k, v, do = W.attn_inputs(n, n, dims, seed)
    return tree, dims, whole, n, q, k, v, do


def _tol(dtype):
    if dtype == "bf16":
        return dict(o=1e-2, lse=1e-2, dq=2e-2, dk=2e-2, dv=2e-2)
    return dict.fromkeys(("o", "lse", "dq", "dk", "dv"), 1e-5)


@pytest.mark.parametrize("seed,cap,dtype,kw", [
    (11, 700, "bf16", {}),
    (12, 300, "bf16", dict(shuffle=True)),
    (13, 450, "bf16", dict(p_zero=0.2, n_roots=2)),
    (14, 500, "fp32", {}),
])
def test_library_driver_equals_whole_tree_oracle(seed, cap, dtype, kw):
    tree, dims, whole, n, q, k, v, do = _whole_tree_case(400 + seed, 16, 20, 260, dtype, **kw)
    want = A.branches(whole, q.float(), k.float(), v.float(), do.float())
    plan = T.tree_partition_plan(tree.parent, tree.seg_len, cap).to_device()
    assert plan.n_parts >= 3 and plan.max_prefix > 0
    print(f"[case] library driver seed={seed} cap={cap} {dtype}: {plan.n_parts} partitions, N={n}, "
          f"longest slice {plan.max_prefix}", flush=True)
    qd, kd, vd, dod = (x.cuda() for x in (q, k, v, do))
    o, lse = T.tree_attn_partitioned_fwd(qd, kd, vd, plan)
    dq, dk, dv = T.tree_attn_partitioned_bwd(qd, kd, vd, plan, o, dod, lse)
    torch.cuda.synchronize()
    got = dict(o=o, lse=lse, dq=dq, dk=dk, dv=dv)
    errs = {key: rel_l2(got[key].float().cpu().numpy(), want[key]) for key in got}
    print("   rel-L2:", {k_: f"{e:.2e}" for k_, e in errs.items()}, flush=True)
    for key, e in errs.items():
        assert e <= _tol(dtype)[key], (key, e)
    # a second call with the same workspace contents left behind gives the same bits
    o2, lse2 = T.tree_attn_partitioned_fwd(qd, kd, vd, plan)
    dq2, dk2, dv2 = T.tree_attn_partitioned_bwd(qd, kd, vd, plan, o2, dod, lse2)
    torch.cuda.synchronize()
    for a, b in ((o, o2), (lse, lse2), (dq, dq2), (dk, dk2), (dv, dv2)):
        assert torch.equal(a, b)
    # partitions whose rows are one contiguous run are processed in place; gathering them instead
    # runs the same kernels on the same values
    n_ip = int((plan.part_own_start >= 0).sum()), int((plan.part_prefix_start >= 0).sum())
    print(f"   in place: own rows of {n_ip[0]}, cached slices of {n_ip[1]} of {plan.n_parts} partitions", flush=True)
    plan.in_place = False
    o3, lse3 = T.tree_attn_partitioned_fwd(qd, kd, vd, plan)
    dq3, dk3, dv3 = T.tree_attn_partitioned_bwd(qd, kd, vd, plan, o3, dod, lse3)
    torch.cuda.synchronize()
    for a, b in ((o, o3), (lse, lse3), (dq, dq3)):
        assert torch.equal(a, b)
    # cached-key gradients reach the fp32 accumulators in another order (added in place by the kernels
    # vs. summed per partition first), so dk / dv agree to fp32 rounding before the final rounding
    for a, b in ((dk, dk3), (dv, dv3)):
        assert rel_l2(a.float().cpu().numpy(), b.float().cpu().numpy()) <= (2e-3 if dtype == "bf16" else 1e-6)


def test_library_driver_single_partition_is_the_plain_call():
    """Capacity >= N: one partition, identity gather; bit-identical to tt_tree_attn_fwd / bwd."""
    tree, dims, whole, n, q, k, v, do = _whole_tree_case(431, 12, 30, 200, "bf16")
    plan = T.tree_partition_plan(tree.parent, tree.seg_len, n).to_device()
    assert plan.n_parts == 1 and plan.max_prefix == 0
    meta = T.tree_build_meta(tree.parent, tree.seg_len, tree.trained)
    kend, kmin, kmax = (torch.from_numpy(x).cuda() for x in (meta.kend, meta.ktile_kend_min, meta.ktile_kend_max))
    qd, kd, vd, dod = (x.cuda() for x in (q, k, v, do))
    print(f"[case] library driver single partition N={n}", flush=True)
    o, lse = T.tree_attn_partitioned_fwd(qd, kd, vd, plan)
    dq, dk, dv = T.tree_attn_partitioned_bwd(qd, kd, vd, plan, o, dod, lse)
    o1, lse1 = T.tree_attn_fwd(qd, kd, vd, kend, kmin, kmax)
    dq1, dk1, dv1 = T.tree_attn_bwd(qd, kd, vd, kend, kmin, kmax, o1, dod, lse1)
    torch.cuda.synchronize()
    for a, b in ((o, o1), (lse, lse1), (dq, dq1), (dk, dk1), (dv, dv1)):
        assert torch.equal(a, b)


def test_library_driver_strided_qkv_and_sampled_rows():
    """q, k, v as slices of one fused [N, (hq+2hkv)*d] buffer; a mid-size tree (several key tiles per
    partition), checked on sampled query rows / key rows against the oracle's row-wise functions."""
    tree = W.random_tree(777, n_nodes=40, lo=100, hi=900, shuffle=False)
    dims = W.AttnDims(8, 2, 128, "bf16", 0.5)
    whole = M.dfs_meta(tree.parent, tree.seg_len, tree.trained)
    n = whole["n_tokens"]
    q, k, v, do = W.attn_inputs(n, n, dims, 777)
    fused = torch.cat([q.reshape(n, -1), k.reshape(n, -1), v.reshape(n, -1)], dim=1).cuda()
    hq, hkv, d = dims.hq, dims.hkv, dims.d
    qd = fused[:, :hq * d].view(n, hq, d)
    kd = fused[:, hq * d:(hq + hkv) * d].view(n, hkv, d)
    vd = fused[:, (hq + hkv) * d:].view(n, hkv, d)
    assert not qd.is_contiguous()
    plan = T.tree_partition_plan(tree.parent, tree.seg_len, 4096).to_device()
    print(f"[case] library driver fused qkv N={n}: {plan.n_parts} partitions, longest slice {plan.max_prefix}", flush=True)
    assert plan.n_parts >= 4
    dod = do.cuda()
    o, lse = T.tree_attn_partitioned_fwd(qd, kd, vd, plan)
    dq, dk, dv = T.tree_attn_partitioned_bwd(qd, kd, vd, plan, o, dod, lse)
    # the plain whole-tree call on the same tensors: same kernels, other tiling / summation order
    meta = T.tree_build_meta(tree.parent, tree.seg_len, tree.trained)
    kend, kmin, kmax = (torch.from_numpy(x).cuda() for x in (meta.kend, meta.ktile_kend_min, meta.ktile_kend_max))
    o1, lse1 = T.tree_attn_fwd(qd, kd, vd, kend, kmin, kmax)
    dq1, dk1, dv1 = T.tree_attn_bwd(qd, kd, vd, kend, kmin, kmax, o1, dod, lse1)
    torch.cuda.synchronize()
    for name, a, b in (("o", o, o1), ("lse", lse, lse1), ("dq", dq, dq1), ("dk", dk, dk1), ("dv", dv, dv1)):
        e = rel_l2(a.float().cpu().numpy(), b.float().cpu().numpy())
        print(f"   partitioned vs whole-tree call {name}: {e:.2e}", flush=True)
        assert e <= 1e-2, (name, e)
    rng = np.random.default_rng(5)
    rows = np.sort(rng.choice(n, 48, replace=False))
    keys = np.sort(rng.choice(n, 48, replace=False))
    for kvh in range(hkv):
        r = A.rows(whole, q.float(), k.float(), v.float(), do.float(), kvh, rows, keys)
        G = hq // hkv
        hs = slice(kvh * G, (kvh + 1) * G)
        assert rel_l2(o[rows][:, hs].float().cpu().numpy(), r["o"]) <= 1e-2
        assert rel_l2(lse[hs][:, rows].T.cpu().numpy(), r["lse"]) <= 1e-2
        assert rel_l2(dq[rows][:, hs].float().cpu().numpy(), r["dq"]) <= 2e-2
        assert rel_l2(dk[keys][:, kvh].float().cpu().numpy(), r["dk"]) <= 2e-2
        assert rel_l2(dv[keys][:, kvh].float().cpu().numpy(), r["dv"]) <= 2e-2


def test_library_driver_errors():
    tree, dims, whole, n, q, k, v, do = _whole_tree_case(440, 8, 20, 100, "bf16")
    plan = T.tree_partition_plan(tree.parent, tree.seg_len, 150).to_device()
    qd, kd, vd = (x.cuda() for x in (q, k, v))
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(T.TreeTrainError) as e:
        T.tree_attn_partitioned_fwd(qd, kd, vd, plan, workspace=small)
    assert e.value.status == -6
    with pytest.raises(T.TreeTrainError) as e:                  # plan of another tree size
        T.tree_attn_partitioned_fwd(qd[:-1], kd[:-1], vd[:-1], plan)
    assert e.value.status == -2
