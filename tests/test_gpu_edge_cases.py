"""GPU: empty and degenerate inputs of the later entry points (nothing may be launched with a zero grid,
nothing may be written out of bounds)."""
import numpy as np
import pytest
import torch

import paper_2511_00413_amd as T

pytestmark = pytest.mark.gpu


def test_empty_tree_everywhere():
    print("[case] empty inputs", flush=True)
    z_i32 = torch.zeros(0, dtype=torch.int32, device="cuda")
    # convolution: no tokens
    x = torch.zeros((0, 16), dtype=torch.bfloat16, device="cuda")
    w = torch.ones((16, 4), dtype=torch.float32, device="cuda")
    y = T.tree_conv_fwd(x, w, None, z_i32)
    assert y.shape == (0, 16)
    dx, dw, db = T.tree_conv_bwd(x, w, None, z_i32, x, T.tree_conv_plan([], 4))
    torch.cuda.synchronize()
    assert dx.shape == (0, 16) and torch.all(dw == 0) and torch.all(db == 0)
    # gated delta rule: no tokens
    q = torch.zeros((0, 1, 128), dtype=torch.bfloat16, device="cuda")
    gb = torch.zeros((0, 1), dtype=torch.float32, device="cuda")
    o = T.tree_gdn_fwd(q, q, q, gb, gb, T.tree_gdn_plan([], []))
    assert o.shape == (0, 1, 128)
    grads = T.tree_gdn_bwd(q, q, q, gb, gb, q, T.tree_gdn_plan([], []))
    assert grads[0].shape == (0, 1, 128) and grads[3].shape == (0, 1)
    # partition driver: no tokens
    plan = T.tree_partition_plan([], [], 8).to_device()
    qa = torch.zeros((0, 2, 128), dtype=torch.bfloat16, device="cuda")
    ka = torch.zeros((0, 1, 128), dtype=torch.bfloat16, device="cuda")
    o, lse = T.tree_attn_partitioned_fwd(qa, ka, ka, plan)
    dq, dk, dv = T.tree_attn_partitioned_bwd(qa, ka, ka, plan, o, qa, lse)
    torch.cuda.synchronize()
    assert o.shape == (0, 2, 128) and dk.shape == (0, 1, 128)


def test_zero_length_nodes_only_and_single_token():
    print("[case] degenerate trees", flush=True)
    # a tree of empty nodes and one token at a leaf
    parent, seg = [-1, 0, 1, 1], [0, 0, 1, 0]
    meta = T.tree_build_meta(parent, seg)
    pred = torch.from_numpy(meta.tok_pred).cuda()
    x = torch.full((1, 8), 2.0, dtype=torch.bfloat16, device="cuda")
    w = torch.ones((8, 3), dtype=torch.float32, device="cuda")
    y = T.tree_conv_fwd(x, w, None, pred, silu=False)
    dx, dw, db = T.tree_conv_bwd(x, w, None, pred, x, T.tree_conv_plan(meta.tok_pred, 3), silu=False)
    torch.cuda.synchronize()
    assert torch.all(y == 2.0) and torch.all(dx == 2.0) and torch.all(db == 2.0)
    assert torch.equal(dw.cpu(), torch.tensor([[0.0, 0.0, 4.0]] * 8))
    k = torch.zeros((1, 1, 128), dtype=torch.bfloat16, device="cuda"); k[0, 0, 3] = 1.0
    v = torch.randn((1, 1, 128), device="cuda").bfloat16()
    one = torch.ones((1, 1), dtype=torch.float32, device="cuda")
    o = T.tree_gdn_fwd(k, k, v, 0 * one, one, T.tree_gdn_plan(parent, seg), scale=1.0)
    torch.cuda.synchronize()
    assert torch.allclose(o.float(), v.float(), rtol=1e-2, atol=1e-3)      # S = k v^T, o = (q.k) v
    d_o = torch.randn((1, 1, 128), device="cuda").bfloat16()
    dq, dk, dv, dg, dbeta = T.tree_gdn_bwd(k, k, v, 0 * one, one, d_o, T.tree_gdn_plan(parent, seg), scale=1.0)
    torch.cuda.synchronize()
    assert torch.allclose(dv.float(), d_o.float(), rtol=1e-2, atol=1e-3)   # o = beta (q.k) v  ->  dv = d_o
    assert torch.allclose(dbeta, (d_o.float() * v.float()).sum().reshape(1, 1), rtol=1e-3, atol=1e-3)
    assert torch.all(dg == 0)                                              # no earlier state to decay
    plan = T.tree_partition_plan(parent, seg, 1).to_device()
    qa = torch.randn((1, 2, 128), device="cuda").bfloat16()
    ka = torch.randn((1, 1, 128), device="cuda").bfloat16()
    oa, lse = T.tree_attn_partitioned_fwd(qa, ka, ka, plan)
    torch.cuda.synchronize()
    assert torch.allclose(oa.float(), ka.float().expand(1, 2, 128), rtol=1e-2, atol=1e-3)   # one key: softmax = 1
