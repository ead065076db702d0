"""The hot path recorded into a HIP graph and replayed: rotary embedding, attention forward and backward, inverse
rotation, the one-pass loss, and the SSM-layer calls, all with caller-provided outputs and workspaces (the
library allocates nothing and never synchronises, so its calls can be captured).  Every kernel is deterministic, so
each replay must reproduce the eager results bit for bit -- also after the inputs have changed and other work has run
between the replays (the dK/dV planner's counters and work queues are rebuilt inside every replay)."""
import numpy as np
import pytest
import torch

import paper_2511_00413_amd as T
import workloads as W

pytestmark = pytest.mark.gpu


def test_attention_path_in_a_graph():
    dev = torch.device("cuda")
    tree = W.random_tree(88, n_nodes=9, lo=40, hi=260, n_roots=2)
    meta = T.tree_build_meta(tree.parent, tree.seg_len, tree.trained)
    n = meta.n_tokens
    dims = W.AttnDims(8, 2, 128, "bf16", 0.5)
    q0, k0, v, do = (x.to(dev) for x in W.attn_inputs(n, n, dims, 9))
    V = 4096
    logits, target = (x.to(dev) for x in W.loss_inputs(n, V, 17, 2.0, "bf16"))
    kend, kmin, kmax = (torch.from_numpy(x).to(dev) for x in (meta.kend, meta.ktile_kend_min, meta.ktile_kend_max))
    pos = torch.from_numpy(meta.tok_pos).to(dev)
    w = torch.from_numpy(meta.tok_weight).to(dev)
    print(f"[case] graph replay N={n} hq={dims.hq} hkv={dims.hkv}", flush=True)

    q, k = torch.empty_like(q0), torch.empty_like(k0)
    o = torch.empty_like(q0)
    lse = torch.empty((dims.hq, n), dtype=torch.float32, device=dev)
    dq, dk, dv = torch.empty_like(q0), torch.empty_like(k0), torch.empty_like(v)
    ws_f = torch.empty(max(T.tree_attn_workspace(q, k, v, 0, False), 256), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(T.tree_attn_workspace(q, k, v, 0, True), dtype=torch.uint8, device=dev)
    logp = torch.empty(n, dtype=torch.float32, device=dev)
    lse_l = torch.empty(n, dtype=torch.float32, device=dev)
    loss = torch.zeros(1, dtype=torch.float32, device=dev)
    dlogits = torch.empty_like(logits)

    def step():
        T.tree_rope(q0, pos, out=q)
        T.tree_rope(k0, pos, out=k)
        T.tree_attn_fwd(q, k, v, kend, kmin, kmax, o=o, lse=lse, workspace=ws_f)
        T.tree_attn_bwd(q, k, v, kend, kmin, kmax, o, do, lse, dq=dq, dk=dk, dv=dv, workspace=ws_b)
        T.tree_rope(dq, pos, inverse=True, out=dq)
        T.tree_rope(dk, pos, inverse=True, out=dk)
        loss.zero_()                                   # a fill kernel, not a memset node
        T.tree_weighted_logprob_fwd_bwd(logits, target, w, loss_acc=loss, logp=logp, lse=lse_l, out=dlogits)

    outs = (o, lse, dq, dk, dv, logp, lse_l, loss, dlogits)
    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in outs]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                          # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        step()
    for replay in range(3):
        for t in outs:
            t.fill_(7 if t.dtype != torch.float32 else float("nan"))      # stale results must not survive
        (q0 * 2).sum().item()                            # unrelated eager work and a synchronisation in between
        g.replay()
        torch.cuda.synchronize()
        for name, a, b in zip("o lse dq dk dv logp lse_l loss dlogits".split(), outs, want):
            assert torch.equal(a, b), (replay, name)
    # new inputs, same graph: the replay must follow them
    q0.mul_(0.5)
    logits.add_(0.25)
    step()
    torch.cuda.synchronize()
    want2 = [t.clone() for t in outs]
    assert not torch.equal(want2[0], want[0])
    g.replay()
    torch.cuda.synchronize()
    for name, a, b in zip("o lse dq dk dv logp lse_l loss dlogits".split(), outs, want2):
        assert torch.equal(a, b), name


def test_ssm_layer_calls_in_a_graph():
    dev = torch.device("cuda")
    tree = W.random_tree(91, n_nodes=8, lo=10, hi=150)
    meta = T.tree_build_meta(tree.parent, tree.seg_len, tree.trained)
    n, hk, hv, C, K = meta.n_tokens, 2, 4, 256, 4
    gen = torch.Generator().manual_seed(4)
    qg = torch.nn.functional.normalize(torch.randn((n, hk, 128), generator=gen), dim=-1).to(torch.bfloat16).to(dev)
    kg = torch.nn.functional.normalize(torch.randn((n, hk, 128), generator=gen), dim=-1).to(torch.bfloat16).to(dev)
    vg = torch.randn((n, hv, 128), generator=gen).to(torch.bfloat16).to(dev)
    g_ = (-(torch.rand((n, hv), generator=gen) * 0.2 + 0.005)).to(dev)
    beta = (torch.rand((n, hv), generator=gen) * 0.8 + 0.1).to(dev)
    d_o = torch.randn((n, hv, 128), generator=gen).to(torch.bfloat16).to(dev)
    x = torch.randn((n, C), generator=gen).to(torch.bfloat16).to(dev)
    dy = torch.randn((n, C), generator=gen).to(torch.bfloat16).to(dev)
    cw = (torch.randn((C, K), generator=gen) * 0.5).to(dev)
    cb = torch.randn((C,), generator=gen).to(dev)
    pred = torch.from_numpy(meta.tok_pred).to(dev)
    plan = T.tree_gdn_plan(tree.parent, tree.seg_len).to_device(dev)
    cplan = T.tree_conv_plan(meta.tok_pred, K).to_device(dev)
    print(f"[case] graph replay of the SSM-layer calls N={n}: {plan.n_chunks} chunks, {plan.n_levels} levels", flush=True)

    def step():
        y = T.tree_conv_fwd(x, cw, cb, pred)
        dx, dw, db = torch.empty_like(x), torch.empty_like(cw), torch.empty_like(cb)
        T.tree_conv_bwd_static(x, cw, cb, pred, dy, cplan, dx, dw, db)        # scratch: the library's static array
        og = T.tree_gdn_fwd(qg, kg, vg, g_, beta, plan)
        gg = T.tree_gdn_bwd(qg, kg, vg, g_, beta, d_o, plan)
        return (y, dx, dw, db, og) + tuple(gg)

    want = [t.clone() for t in step()]
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        outs = step()                                   # outputs and workspaces come from the graph's private pool
    for replay in range(3):
        for t in outs:
            t.zero_()
        (x.float() * 2).sum().item()
        g.replay()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(outs, want)):
            assert torch.equal(a, b), (replay, i)
