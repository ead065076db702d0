"""GPU parity: gated delta rule with tree state routing (forward) against the fp64 token recurrence.
Tolerance: the chunked kernel rounds its per-chunk operands (U, W, decayed Q / K, the entering
state) to bf16 once each (2^-9 relative) and accumulates in fp32; rel-L2 <= 2e-2 on o, measured a
few 1e-3."""
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
    return q, k, v, g, beta


def _check(tree, hk, hv, seed, heads_checked=None):
    m = M.dfs_meta(tree.parent, tree.seg_len)
    n = m["n_tokens"]
    q, k, v, g, beta = _inputs(n, hk, hv, seed)
    plan = T.tree_gdn_plan(tree.parent, tree.seg_len)
    print(f"[case] gdn n={n} hk={hk} hv={hv}: {plan.n_chunks} chunks, {plan.n_slots} saved states", flush=True)
    o = T.tree_gdn_fwd(q.cuda(), k.cuda(), v.cuda(), g.cuda(), beta.cuda(), plan)
    torch.cuda.synchronize()
    o = o.float().cpu().numpy()
    hs = list(range(hv)) if heads_checked is None else heads_checked
    rep = hv // hk
    for h in hs:                                  # the oracle runs one value head at a time
        want = S.gdn_tree(q[:, h // rep:h // rep + 1], k[:, h // rep:h // rep + 1], v[:, h:h + 1], g[:, h:h + 1],
                          beta[:, h:h + 1], m["tok_pred"])
        e = rel_l2(o[:, h], want[:, 0])
        print(f"   head {h}: rel-L2 {e:.2e}", flush=True)
        assert e <= 2e-2, (h, e)
    return o


def test_chain_partial_chunks():
    """One sequence of 150 tokens: chunks of 64, 64, 22; then a 1-token sequence."""
    _check(W._mk([-1], [150], [1], "chain"), 1, 2, 0)
    _check(W._mk([-1], [1], [1], "one"), 1, 1, 1)


@pytest.mark.parametrize("seed", range(4))
def test_random_trees(seed):
    t = W.random_tree(880 + seed, n_nodes=6 + 4 * seed, lo=1, hi=150, n_roots=1 + seed % 2, p_zero=0.15)
    _check(t, 2, 4, seed)


def test_short_nodes_many_saved_states():
    t = W.random_tree(891, n_nodes=60, lo=1, hi=5, p_zero=0.2)
    _check(t, 1, 2, 5)


def test_routing_figure_and_reproducible():
    """n0 -> {n1 -> {n3, n4}, n2}: n2 continues from n0's end state."""
    t = W._mk([-1, 0, 0, 1, 1], [70, 30, 40, 20, 64], [1] * 5, "routing")
    o1 = _check(t, 2, 4, 9)
    o2 = _check(t, 2, 4, 9)
    assert np.array_equal(o1, o2)


@pytest.mark.parametrize("seed", range(3))
def test_level_schedule_equals_sequence_order(seed):
    """Sibling subtrees walked side by side (one launch per dependency level of the chunk program) give bit-identical
    outputs and captured states to one walk over all chunks in sequence order: every chunk does the same arithmetic
    on the same entering state, only when and where it runs differs."""
    t = W.random_tree(930 + seed, n_nodes=10 + 8 * seed, lo=1, hi=160, n_roots=1 + seed % 2, p_zero=0.15)
    m = M.dfs_meta(t.parent, t.seg_len)
    n = m["n_tokens"]
    q, k, v, g, beta = (x.cuda() for x in _inputs(n, 2, 4, 20 + seed))
    cap = [i for i in range(len(t.parent)) if t.seg_len[i] > 0][:: max(1, len(t.parent) // 3)][:3]
    plan = T.tree_gdn_plan(t.parent, t.seg_len, capture_nodes=cap)
    print(f"[case] gdn schedule n={n}: {plan.n_chunks} chunks in {plan.n_segments} segments, {plan.n_levels} levels", flush=True)
    init = torch.randn((4, 128, 128), generator=torch.Generator().manual_seed(seed)).cuda() * 0.1
    plan.to_device()
    plan.parallel = True
    o_par, st_par = T.tree_gdn_fwd(q, k, v, g, beta, plan, initial_state=init, return_states=True)
    plan.parallel = False
    o_seq, st_seq = T.tree_gdn_fwd(q, k, v, g, beta, plan, initial_state=init, return_states=True)
    torch.cuda.synchronize()
    assert torch.equal(o_par, o_seq) and torch.equal(st_par, st_seq)


def test_larger_tree_sampled_heads():
    t = W.random_tree(895, n_nodes=24, lo=50, hi=400)
    _check(t, 4, 8, 11, heads_checked=[0, 5])


def test_errors():
    q = torch.zeros((4, 1, 64), dtype=torch.bfloat16, device="cuda")
    v = torch.zeros((4, 1, 64), dtype=torch.bfloat16, device="cuda")
    gb = torch.zeros((4, 1), dtype=torch.float32, device="cuda")
    plan = T.tree_gdn_plan([-1], [4])
    with pytest.raises(T.TreeTrainError) as e:
        T.tree_gdn_fwd(q, q, v, gb, gb, plan)
    assert e.value.status == -8
