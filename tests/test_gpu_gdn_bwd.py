"""GPU parity: backward of the gated delta rule with tree state routing against the fp64 reverse recurrence.
Like the forward, the kernels round the operands of their matrix products to bf16 once each (per-chunk
operands, entering state, Vn, gradient of the leaving state, dVn, the solved right-hand sides) and accumulate in
fp32; solves and element-wise work are fp32; dq, dk, dv are rounded to bf16 at the end (dq, dk after the fp32 sum
over the value heads of a key head).  Tolerance: rel-L2 <= 8e-3 on every output (a product of two or three
operands rounded to bf16, fp32 sums; measured 2.3e-3 .. 3.4e-3)."""
import numpy as np
import pytest
import torch

import paper_2511_00413_amd as T
import workloads as W
from oracle import meta as M
from oracle import ssm as S
from tt_testutil import rel_l2

pytestmark = pytest.mark.gpu


def _inputs(n, hk, hv, seed):
    g_ = torch.Generator().manual_seed(seed)
    q = torch.randn((n, hk, 128), generator=g_)
    k = torch.randn((n, hk, 128), generator=g_)
    q = (q / q.norm(dim=-1, keepdim=True)).to(torch.bfloat16)
    k = (k / k.norm(dim=-1, keepdim=True)).to(torch.bfloat16)
    v = torch.randn((n, hv, 128), generator=g_).to(torch.bfloat16)
    g = -(torch.rand((n, hv), generator=g_) * 0.2 + 0.005)
    beta = torch.rand((n, hv), generator=g_) * 0.8 + 0.1
    d_o = torch.randn((n, hv, 128), generator=g_).to(torch.bfloat16)
    return q, k, v, g, beta, d_o


def _check(tree, hk, hv, seed):
    m = M.dfs_meta(tree.parent, tree.seg_len)
    n = m["n_tokens"]
    q, k, v, g, beta, d_o = _inputs(n, hk, hv, seed)
    plan = T.tree_gdn_plan(tree.parent, tree.seg_len)
    print(f"[case] gdn bwd n={n} hk={hk} hv={hv}: {plan.n_chunks} chunks, {plan.n_slots} saved states", flush=True)
    got = T.tree_gdn_bwd(q.cuda(), k.cuda(), v.cuda(), g.cuda(), beta.cuda(), d_o.cuda(), plan)
    torch.cuda.synchronize()
    got = [t.float().cpu().numpy() for t in got]
    want = S.gdn_tree_bwd(q.float().numpy(), k.float().numpy(), v.float().numpy(), g.numpy(), beta.numpy(), m["tok_pred"],
                          d_o.float().numpy())
    for name, a, b, tol in zip(("dq", "dk", "dv", "dg", "dbeta"), got, want, (8e-3, 8e-3, 8e-3, 8e-3, 8e-3)):
        e = rel_l2(a, b)
        print(f"   {name}: rel-L2 {e:.2e}", flush=True)
        assert np.isfinite(a).all(), name
        assert e <= tol, (name, e)


@pytest.mark.parametrize("seed", range(3))
def test_level_schedule_against_sequence_order(seed):
    """The backward with the level schedule (forward walk and reverse walk one launch per dependency level, sibling
    subtrees side by side; state gradients of a slot's readers stored per segment and added in list order) against
    the walk over all chunks in sequence order.  dv and the per-chunk work are identical; where several readers'
    gradients meet, the two walks add them in a different association, so the comparison is to fp32 rounding of the
    sums (1e-5 relative on fp32 outputs, equal up to one bf16 ulp on a few bf16 elements), not bit for bit.  Also
    checks run-to-run reproducibility of the scheduled walk and the gradient of the initial state."""
    t = W.random_tree(940 + seed, n_nodes=9 + 7 * seed, lo=1, hi=150, n_roots=1 + seed % 2, p_zero=0.15)
    m = M.dfs_meta(t.parent, t.seg_len)
    n = m["n_tokens"]
    q, k, v, g, beta, d_o = (x.cuda() for x in _inputs(n, 2, 4, 30 + seed))
    plan = T.tree_gdn_plan(t.parent, t.seg_len).to_device()
    init = torch.randn((4, 128, 128), generator=torch.Generator().manual_seed(seed)).cuda() * 0.1
    print(f"[case] gdn bwd schedule n={n}: {plan.n_chunks} chunks in {plan.n_segments} segments, {plan.n_levels} levels", flush=True)
    plan.parallel = True
    par = T.tree_gdn_bwd(q, k, v, g, beta, d_o, plan, initial_state=init, want_d_initial_state=True)
    par2 = T.tree_gdn_bwd(q, k, v, g, beta, d_o, plan, initial_state=init, want_d_initial_state=True)
    plan.parallel = False
    seq = T.tree_gdn_bwd(q, k, v, g, beta, d_o, plan, initial_state=init, want_d_initial_state=True)
    torch.cuda.synchronize()
    for name, a, b, c in zip(("dq", "dk", "dv", "dg", "dbeta", "d_initial_state"), par, par2, seq):
        assert torch.equal(a, b), f"{name}: the scheduled walk is not reproducible"
        e = rel_l2(a.float().cpu().numpy(), c.float().cpu().numpy())
        print(f"   {name}: scheduled vs sequence order rel-L2 {e:.2e}", flush=True)
        assert e <= (2e-3 if a.dtype == torch.bfloat16 else 1e-4), (name, e)


@pytest.mark.parametrize("parallel", [True, False])
def test_passes_of_key_head_groups(parallel):
    """A workspace too small for all heads makes the call run in passes of whole key-head groups (here 3 key heads x 2
    value heads: one, two or all three key heads per pass).  The heads are independent, so every output must be
    bit-identical whatever the pass size -- with the state gateway in both directions, with and without the level
    schedule; below the smallest size the call is refused."""
    t = W.random_tree(977, n_nodes=12, lo=1, hi=140, n_roots=2, p_zero=0.1)
    m = M.dfs_meta(t.parent, t.seg_len)
    n, hk, hv = m["n_tokens"], 3, 6
    q, k, v, g, beta, d_o = (x.cuda() for x in _inputs(n, hk, hv, 41))
    cap = [i for i in range(len(t.seg_len)) if t.seg_len[i] > 0][:2]
    plan = T.tree_gdn_plan(t.parent, t.seg_len, capture_nodes=cap).to_device()
    plan.parallel = parallel
    gen = torch.Generator().manual_seed(5)
    init = (torch.randn((hv, 128, 128), generator=gen) * 0.1).cuda()
    d_state = (torch.randn((plan.n_capture, hv, 128, 128), generator=gen) * 0.1).cuda()
    full = T.tree_gdn_bwd_workspace(n, hk, hv, plan)
    least = T.tree_gdn_bwd_workspace(n, hk, hv, plan, smallest=True)
    assert least < full
    print(f"[case] gdn bwd passes n={n} hk={hk} hv={hv} schedule={parallel}: workspace {least} .. {full} bytes", flush=True)

    def run(nbytes):
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        out = T.tree_gdn_bwd(q, k, v, g, beta, d_o, plan, initial_state=init, d_state_out=d_state, want_d_initial_state=True,
                             workspace=ws)
        torch.cuda.synchronize()
        return out

    ref = run(full)
    for nbytes in (least, (least + full) // 2 + 4096, full - 16):
        got = run(nbytes)
        for name, a, b in zip(("dq", "dk", "dv", "dg", "dbeta", "d_initial_state"), got, ref):
            assert torch.equal(a, b), (name, nbytes)
    with pytest.raises(T.TreeTrainError) as e:
        run(least - 256)
    assert e.value.status == -6


def test_chain_partial_chunks():
    """One sequence of 150 tokens: chunks of 64, 64, 22; then a 1-token sequence."""
    _check(W._mk([-1], [150], [1], "chain"), 1, 2, 0)
    _check(W._mk([-1], [1], [1], "one"), 1, 1, 1)


@pytest.mark.parametrize("seed", range(4))
def test_random_trees(seed):
    t = W.random_tree(880 + seed, n_nodes=6 + 4 * seed, lo=1, hi=150, n_roots=1 + seed % 2, p_zero=0.15)
    _check(t, 2, 4, seed)


def test_branch_point_inside_deep_tree():
    """Several children per node and zero-length nodes: slots are reused, gradients meet at branch points."""
    t = W.random_tree(991, n_nodes=24, lo=0, hi=90, n_roots=2, p_zero=0.2)
    _check(t, 1, 2, 7)


@pytest.mark.parametrize("hk,hv", [(3, 3), (2, 8), (8, 8)])
def test_head_layouts(hk, hv):
    """One value head per key head (no group sum), four per key head, and a head count that is a multiple of
    eight (the workgroup-to-head mapping differs there)."""
    t = W.random_tree(870 + hv, n_nodes=7, lo=1, hi=100, p_zero=0.1)
    _check(t, hk, hv, 40 + hk)


def test_chunk_boundary_lengths():
    """Node lengths at and around the chunk size (63, 64, 65, 128, 129), a zero-length node between two others,
    two roots: chunks of full and of one-token length, branch points at chunk ends."""
    parent = [-1, 0, 0, 1, 1, 2, -1, 6, 7]
    seg = [64, 63, 65, 128, 1, 0, 129, 0, 2]
    _check(W._mk(parent, seg, [1] * len(seg), "boundaries"), 1, 2, 77)
