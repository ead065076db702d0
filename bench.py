#!/usr/bin/env python3
"""Benchmark of the tree-attention hot path on one MI355X.

One "step" = one pass of the whole path over one synthetic tree: host metadata build
(tree_build_meta) + upload of the mask bounds, tree attention forward, backward, and the weighted
log-prob loss.  The headline value is the attention forward+backward rate in *useful* TFLOP/s:
14 * Hq * D * visible_pairs flops (4 D per pair forward, 10 D backward) divided by the forward +
backward time measured with events on the launch stream.  Inputs are resident in HBM before the
timed region starts.

Prints one JSON line (see README for the fields).
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0

# HBM bytes per launch (read + write) of the attention kernels, from the rocprofv3 FETCH_SIZE /
# WRITE_SIZE runs summarised under profiles/ (FETCH_SIZE scaled x2.0, WRITE_SIZE x1.0 by the plain
# 1 GiB copy of the same run).  Offline measurements: reported only for the workload they cover.
MEASURED_TRAFFIC_BYTES = {
    (2, "attn_fwd"): 230.3e6 + 149.2e6,
    (2, "attn_dkdv"): 2394.4e6 + 271.8e6,
    (2, "attn_dq"): 372.4e6 + 142.8e6,
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 3, 4, 5],
                    help="benchmark configuration (5 = one partition step: 32K chunk x 64K prefix)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-linearized", action="store_true")
    ap.add_argument("--no-loss", action="store_true")
    ap.add_argument("--no-rope", action="store_true")
    ap.add_argument("--no-partitioned", action="store_true")
    ap.add_argument("--no-conv", action="store_true")
    ap.add_argument("--no-gdn", action="store_true")
    ap.add_argument("--no-gdn-bwd", action="store_true")
    ap.add_argument("--gdn-heads", type=int, default=32, help="value heads of the gated-delta-rule leg (key heads = half)")
    ap.add_argument("--conv-channels", type=int, default=8192,
                    help="channels of the tree-convolution leg (2*16*128 + 32*128 for a GDN layer with 16 key / 32 value heads)")
    ap.add_argument("--partition-gather-all", action="store_true",
                    help="partitioned leg: gather / scatter every partition, also those that could be used in place")
    ap.add_argument("--partition-capacity", type=int, default=0,
                    help="token capacity for the partitioned leg (0 = about a quarter of the tree)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="after the timed region, run one plain 1 GiB device copy (a known-size kernel "
                         "for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2511_00413_amd as T
    import linearize
    import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = args.config
    dims = W.DIMS[cfg]
    tdt = torch.bfloat16 if dims.dtype == "bf16" else torch.float32

    # ---------------- workload ----------------
    if cfg == 5:
        step_w = W.step_cfg5()
        tree, n_prefix, prefix_visible = step_w.chunk, step_w.n_prefix, step_w.prefix_visible
        root_off = [int(prefix_visible.sum())]
        workload = "cfg5-step: 32768-token chunk (8 nodes) x 65536 cached prefix keys (variant b), GQA 64/8, d=128, bf16"
    else:
        tree, n_prefix, prefix_visible, root_off = W.tree_config(cfg), 0, None, None
        workload = {
            1: "cfg1: worked 3-leaf tree, N=240, MHA 4x64, fp32",
            2: "cfg2: random depth-4 tree seed 117, N=16406, GQA 32/8, d=128, bf16, vocab 32768",
            3: "cfg3: agentic fan-out 8K->16x(2K->2x1K), N=73728, GQA 64/8, d=128, bf16, vocab 151936 in 4K-row chunks",
            4: "cfg4: deep chain seed 195, N=131091, GQA 32/8, d=128, bf16",
        }[cfg]

    def build_meta():
        return T.tree_build_meta(tree.parent, tree.seg_len, tree.trained, root_pos_offset=root_off,
                                 n_prefix=n_prefix, prefix_visible=prefix_visible)

    meta = build_meta()
    N = meta.n_tokens
    pairs = linearize.visible_pairs(meta)
    q, k, v, do = (x.to(dev) for x in W.attn_inputs(N, N, dims, cfg))
    kp = vp = dkp = dvp = None
    if n_prefix:
        _, kp, vp, _ = (x.to(dev) for x in W.attn_inputs(1, n_prefix, dims, cfg + 100))
        dkp = torch.zeros(kp.shape, dtype=torch.float32, device=dev)
        dvp = torch.zeros(kp.shape, dtype=torch.float32, device=dev)
    kend_d = torch.empty(n_prefix + N, dtype=torch.int32, device=dev)
    kmin_d = torch.empty(meta.n_ktiles, dtype=torch.int32, device=dev)
    kmax_d = torch.empty(meta.n_ktiles, dtype=torch.int32, device=dev)
    kend_h = torch.empty(n_prefix + N, dtype=torch.int32).pin_memory()
    kmin_h = torch.empty(meta.n_ktiles, dtype=torch.int32).pin_memory()
    kmax_h = torch.empty(meta.n_ktiles, dtype=torch.int32).pin_memory()
    w_h = torch.empty(N, dtype=torch.float32).pin_memory()
    w_d = torch.empty(N, dtype=torch.float32, device=dev)

    # loss inputs (value distribution of the config; drawn on the device to keep start-up short)
    do_loss = dims.vocab > 0 and not args.no_loss
    loss_rows = 0
    if do_loss:
        gen = torch.Generator(device=dev)
        gen.manual_seed(cfg * 1000 + 5)
        chunk_rows = N if cfg != 3 else 4096
        logits = (torch.randn((chunk_rows, dims.vocab), generator=gen, device=dev, dtype=torch.float32)
                  * dims.logit_std).to(torch.bfloat16 if dims.logit_dtype == "bf16" else torch.float32)
        target = torch.randint(0, dims.vocab, (N,), generator=gen, device=dev, dtype=torch.int32)
        logp = torch.empty(N, dtype=torch.float32, device=dev)
        lse_l = torch.empty(N, dtype=torch.float32, device=dev)
        loss_acc = torch.zeros(1, dtype=torch.float32, device=dev)
        dlogits = torch.empty_like(logits)          # gradient of the loss w.r.t. the logits (same chunking)
        loss_rows = N

    ws_f = torch.empty(T.tree_attn_workspace(q, k, v, n_prefix, False), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(T.tree_attn_workspace(q, k, v, n_prefix, True), dtype=torch.uint8, device=dev)
    o = torch.empty_like(q)
    lse = torch.empty((dims.hq, N), dtype=torch.float32, device=dev)
    dq = torch.empty_like(q)
    dk = torch.empty_like(k)
    dv = torch.empty_like(v)

    # rotary embedding with the tree position ids: q_raw / k_raw -> q / k before the attention, and the
    # inverse rotation of dq / dk after it (the steps either side of the attention path)
    q_raw, k_raw = q.clone(), k.clone()
    pos_h = torch.empty(N, dtype=torch.int32).pin_memory()
    pos_d = torch.empty(N, dtype=torch.int32, device=dev)
    do_rope = dims.dtype == "bf16" and not args.no_rope

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    host_ms = []

    def step(events=None):
        t0 = time.perf_counter()
        m = build_meta()                                   # a1-a4 on the host
        kend_h.numpy()[:] = m.kend
        kmin_h.numpy()[:] = m.ktile_kend_min
        kmax_h.numpy()[:] = m.ktile_kend_max
        w_h.numpy()[:] = m.tok_weight
        kend_d.copy_(kend_h, non_blocking=True)
        kmin_d.copy_(kmin_h, non_blocking=True)
        kmax_d.copy_(kmax_h, non_blocking=True)
        w_d.copy_(w_h, non_blocking=True)
        if do_rope:
            pos_h.numpy()[:] = m.tok_pos
            pos_d.copy_(pos_h, non_blocking=True)
        host_ms.append((time.perf_counter() - t0) * 1e3)
        if do_rope:
            T.tree_rope(q_raw, pos_d, out=q)
            T.tree_rope(k_raw, pos_d, out=k)
        if events:
            events[0].record()
        T.tree_attn_fwd(q, k, v, kend_d, kmin_d, kmax_d, k_prefix=kp, v_prefix=vp, o=o, lse=lse, workspace=ws_f)
        if events:
            events[1].record()
        T.tree_attn_bwd(q, k, v, kend_d, kmin_d, kmax_d, o, do, lse, k_prefix=kp, v_prefix=vp,
                        dk_prefix_acc=dkp, dv_prefix_acc=dvp, dq=dq, dk=dk, dv=dv, workspace=ws_b)
        if events:
            events[2].record()
        if do_rope:
            T.tree_rope(dq, pos_d, inverse=True, out=dq)
            T.tree_rope(dk, pos_d, inverse=True, out=dk)
        if do_loss:
            loss_acc.zero_()
            rows = logits.shape[0]
            for lo in range(0, N, rows):
                n = min(rows, N - lo)
                T.tree_weighted_logprob(logits[:n], target[lo:lo + n], w_d[lo:lo + n], loss_acc=loss_acc,
                                        logp=logp[lo:lo + n], lse=lse_l[lo:lo + n])
                T.tree_weighted_logprob_bwd(logits[:n], target[lo:lo + n], w_d[lo:lo + n], lse_l[lo:lo + n],
                                            out=dlogits[:n])
        if events:
            events[3].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    host_ms.clear()
    T.kernel_timing_enable(True)
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(ev[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ktimes = T.kernel_timing_read()
    T.kernel_timing_enable(False)

    ms_fwd = sum(e[0].elapsed_time(e[1]) for e in ev) / args.steps
    ms_bwd = sum(e[1].elapsed_time(e[2]) for e in ev) / args.steps
    ms_loss = sum(e[2].elapsed_time(e[3]) for e in ev) / args.steps
    useful_flop = 14.0 * dims.hq * dims.d * pairs
    value = useful_flop / ((ms_fwd + ms_bwd) * 1e-3) / 1e12

    # ---------------- roofline of the dominant kernel ----------------
    alg_flop = {"attn_fwd": 4.0, "attn_dkdv": 8.0, "attn_dq": 2.0, "ref_fwd": 4.0, "ref_bwd": 10.0}
    attn_k = {n: t for n, t in ktimes.items() if n in alg_flop and t[1] > 0}
    roofline = None
    kernel_ms = {n: (t[0] / t[1]) for n, t in ktimes.items() if t[1] > 0}
    if attn_k:
        dom = max(attn_k, key=lambda n: attn_k[n][0])
        avg_ms = attn_k[dom][0] / attn_k[dom][1]
        achieved = alg_flop[dom] * dims.hq * dims.d * pairs / (avg_ms * 1e-3) / 1e12
        peak = PEAK_BF16_TFLOPS if dims.dtype == "bf16" else 157.3
        roofline = {"kernel": dom, "bound": "mfma" if dims.dtype == "bf16" else "alu", "achieved": round(achieved, 2),
                    "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4), "traffic": MEASURED_TRAFFIC_BYTES.get((cfg, dom)),
                    "avg_ms": round(avg_ms, 4),
                    "algorithmic_flop_per_launch": alg_flop[dom] * dims.hq * dims.d * pairs}
    loss_gbps = loss_bwd_gbps = None
    if do_loss and "loss_rows" in kernel_ms:
        esz = 2 if dims.logit_dtype == "bf16" else 4
        bytes_total = loss_rows * (dims.vocab * esz + 12)
        loss_ms_total = ktimes["loss_rows"][0] / args.steps
        loss_gbps = bytes_total / (loss_ms_total * 1e-3) / 1e9
        # backward: one read of the logits + one write of the gradient + target, weight, lse per row
        loss_bwd_gbps = loss_rows * (2 * dims.vocab * esz + 12) / (ktimes["loss_bwd"][0] / args.steps * 1e-3) / 1e9

    rope_gbps = None
    if do_rope and "rope" in kernel_ms:
        esz_a = 2
        rope_bytes = 2 * (dims.hq + dims.hkv) * N * dims.d * esz_a * 2 + 4 * N * 4      # q, k, dq, dk: read + write; positions
        rope_gbps = rope_bytes / (ktimes["rope"][0] / args.steps * 1e-3) / 1e9

    # ---------------- linearised per-branch baseline on the same GPU ----------------
    lin = None
    if not args.no_linearized and n_prefix == 0:
        idx, lparent, lseg = linearize.linearized_forest(meta)
        lmeta = T.tree_build_meta(lparent, lseg)
        idx_d = torch.from_numpy(idx).to(dev)
        ql, kl, vl, dol = (x.index_select(0, idx_d) for x in (q, k, v, do))
        lk = [torch.from_numpy(x).to(dev) for x in (lmeta.kend, lmeta.ktile_kend_min, lmeta.ktile_kend_max)]
        ol = torch.empty_like(ql); lsel = torch.empty((dims.hq, len(idx)), dtype=torch.float32, device=dev)
        dql = torch.empty_like(ql); dkl = torch.empty_like(kl); dvl = torch.empty_like(vl)
        wsl = torch.empty(T.tree_attn_workspace(ql, kl, vl, 0, True), dtype=torch.uint8, device=dev)
        n_it = max(3, min(args.steps, 10))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for it in range(2 + n_it):
            if it == 2:
                e0.record()
            T.tree_attn_fwd(ql, kl, vl, *lk, o=ol, lse=lsel, workspace=wsl)
            T.tree_attn_bwd(ql, kl, vl, *lk, ol, dol, lsel, dq=dql, dk=dkl, dv=dvl, workspace=wsl)
        e1.record()
        torch.cuda.synchronize()
        ms_lin = e0.elapsed_time(e1) / n_it
        pairs_lin = linearize.visible_pairs(lmeta)
        lin = {"ms_fwd_bwd": round(ms_lin, 4), "n_lin": int(len(idx)), "pairs_lin": pairs_lin,
               "speedup": round(ms_lin / (ms_fwd + ms_bwd), 3),
               "r_tok": round(len(idx) / N, 3), "r_pair": round(pairs_lin / pairs, 3)}
        lin["speedup_over_r_tok"] = round(lin["speedup"] / lin["r_tok"], 3)
        lin["speedup_over_r_pair"] = round(lin["speedup"] / lin["r_pair"], 3)
        del ql, kl, vl, dol, ol, dql, dkl, dvl

    # ---------------- the same tree cut into partitions (boundary overhead) ----------------
    part = None
    if not args.no_partitioned and n_prefix == 0 and dims.dtype == "bf16":
        cap = args.partition_capacity or max(1024, (N // 4 + 1023) // 1024 * 1024)
        t0p = time.perf_counter()
        plan = T.tree_partition_plan(tree.parent, tree.seg_len, cap)
        plan_ms = (time.perf_counter() - t0p) * 1e3
        plan.to_device(dev)
        if args.partition_gather_all:
            plan.in_place = False
            plan.part_own_start[:] = -1
            plan.part_prefix_start[:] = -1
        wsp = torch.empty(T.tree_attn_partitioned_workspace(q, k, v, plan, True), dtype=torch.uint8, device=dev)
        op = torch.empty_like(q); lsep = torch.empty_like(lse)
        dqp = torch.empty_like(q); dkp_ = torch.empty_like(k); dvp_ = torch.empty_like(v)
        n_it = max(3, min(args.steps, 10))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        def part_step():
            T.tree_attn_partitioned_fwd(q, k, v, plan, o=op, lse=lsep, workspace=wsp)
            T.tree_attn_partitioned_bwd(q, k, v, plan, op, do, lsep, dq=dqp, dk=dkp_, dv=dvp_, workspace=wsp)
        for it in range(2 + n_it):
            if it == 2:
                e0.record()
            part_step()
        e1.record()
        torch.cuda.synchronize()
        ms_part = e0.elapsed_time(e1) / n_it
        T.kernel_timing_enable(True)               # a second pass for the per-kernel split
        for it in range(n_it):
            part_step()
        pt = T.kernel_timing_read()
        T.kernel_timing_enable(False)
        # bytes the copy kernels move per fwd+bwd (each row read once and written once)
        esz_a = 2
        q_row, kv_row, kvf = dims.hq * dims.d * esz_a, dims.hkv * dims.d * esz_a, dims.hkv * dims.d * 4
        own = np.diff(plan.part_tok_off).astype(np.int64)
        pre = np.diff(plan.part_prefix_off).astype(np.int64)
        own_g = own * (plan.part_own_start < 0)          # rows that are gathered / scattered (not used in place)
        pre_g = pre * (plan.part_prefix_start < 0)
        gather_b = int((2 * (own_g * (q_row + 2 * kv_row) + pre_g * 2 * kv_row)).sum()                # forward
                       + (2 * (own_g * (3 * q_row + 2 * kv_row) + pre_g * 2 * kv_row)).sum() + 2 * dims.hq * N * 4)
        scatter_b = int((2 * own_g * q_row).sum() + 2 * dims.hq * N * 4                                  # forward
                        + (2 * own_g * (q_row + 2 * kv_row)).sum() + (pre_g * 2 * kvf).sum()             # results, zeroing
                        + (pre_g * 2 * 3 * kvf).sum()                                                    # accumulate
                        + 2 * N * kvf + 2 * N * (kvf + 2 * kv_row))                                      # clear, finalise
        move_ms = (pt["part_gather"][0] + pt["part_scatter"][0]) / n_it
        part = {"capacity": cap, "n_parts": plan.n_parts, "max_prefix": plan.max_prefix,
                "in_place_own": int((plan.part_own_start >= 0).sum()), "in_place_prefix": int((plan.part_prefix_start >= 0).sum()),
                "sum_prefix": int(plan.part_prefix_off[-1]), "ms_fwd_bwd": round(ms_part, 4),
                "ms_whole_fwd_bwd": round(ms_fwd + ms_bwd, 4),
                "ratio_to_whole": round(ms_part / (ms_fwd + ms_bwd), 3),
                "ms_attn_kernels": round(sum(pt[n][0] for n in ("attn_fwd", "attn_delta", "attn_dkdv", "attn_dq", "attn_plan", "attn_reduce")) / n_it, 4),
                "ms_gather": round(pt["part_gather"][0] / n_it, 4), "ms_scatter": round(pt["part_scatter"][0] / n_it, 4),
                "movement_gb": round((gather_b + scatter_b) / 1e9, 4),
                "movement_hbm_gbps": round((gather_b + scatter_b) / (move_ms * 1e-3) / 1e9, 1) if move_ms > 0 else None,
                "ms_host_plan": round(plan_ms, 3)}
        del op, lsep, dqp, dkp_, dvp_, wsp

    # ---------------- tree-correct causal convolution on the same tree (SSM-layer adaptation) ----------------
    conv = None
    if not args.no_conv and n_prefix == 0 and dims.dtype == "bf16":
        C, Kc = args.conv_channels, 4
        gen = torch.Generator(device=dev)
        gen.manual_seed(cfg * 1000 + 9)
        xc = torch.randn((N, C), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        dyc = torch.randn((N, C), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        wc = torch.randn((C, Kc), generator=gen, device=dev, dtype=torch.float32) * 0.5
        bc = torch.randn(C, generator=gen, device=dev, dtype=torch.float32) * 0.1
        pred_d = torch.from_numpy(meta.tok_pred).to(dev)
        cplan = T.tree_conv_plan(meta.tok_pred, Kc).to_device(dev)
        yc = torch.empty_like(xc)
        n_it = max(3, min(args.steps, 10))
        for it in range(2 + n_it):
            if it == 2:
                torch.cuda.synchronize()
                T.kernel_timing_enable(True)
            T.tree_conv_fwd(xc, wc, bc, pred_d, out=yc)
            T.tree_conv_bwd(xc, wc, bc, pred_d, dyc, cplan)
        ct = T.kernel_timing_read()
        T.kernel_timing_enable(False)
        f_ms, b_ms, x_ms = (ct[n][0] / n_it for n in ("conv_fwd", "conv_bwd", "conv_fix"))
        f_bytes = 2 * N * C * 2 + 4 * N                      # read x, write y, tok_pred
        b_bytes = 3 * N * C * 2 + 4 * N                      # read x and dy, write dx
        conv = {"channels": C, "kernel_size": Kc, "fix_tokens": int(len(cplan.fix_tok)),
                "ms_fwd": round(f_ms, 4), "ms_bwd": round(b_ms, 4), "ms_bwd_fix_and_reduce": round(x_ms, 4),
                "fwd_hbm_gbps": round(f_bytes / (f_ms * 1e-3) / 1e9, 1), "bwd_hbm_gbps": round(b_bytes / (b_ms * 1e-3) / 1e9, 1),
                "fwd_frac_of_hbm_peak": round(f_bytes / (f_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4),
                "bwd_frac_of_hbm_peak": round(b_bytes / (b_ms * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4)}
        del xc, dyc, yc

    # ---------------- gated delta rule with tree state routing on the same tree (SSM-layer adaptation) ----------------
    gdn = None
    if not args.no_gdn and n_prefix == 0 and dims.dtype == "bf16":
        ghk, ghv = max(args.gdn_heads // 2, 1), args.gdn_heads   # key / value heads of the GDN layer, 128 x 128 states
        gen = torch.Generator(device=dev)
        gen.manual_seed(cfg * 1000 + 11)
        gq = torch.randn((N, ghk, 128), generator=gen, device=dev, dtype=torch.float32)
        gk = torch.randn((N, ghk, 128), generator=gen, device=dev, dtype=torch.float32)
        gq = (gq / gq.norm(dim=-1, keepdim=True)).to(torch.bfloat16)
        gk = (gk / gk.norm(dim=-1, keepdim=True)).to(torch.bfloat16)
        gv = torch.randn((N, ghv, 128), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        gg = -(torch.rand((N, ghv), generator=gen, device=dev) * 0.2 + 0.005)
        gb = torch.rand((N, ghv), generator=gen, device=dev) * 0.8 + 0.1
        gplan = T.tree_gdn_plan(tree.parent, tree.seg_len).to_device(dev)
        go = torch.empty_like(gv)
        gws = torch.empty(T.binding._lib().tt_tree_gdn_workspace(gplan.n_chunks, gplan.n_slots, ghv), dtype=torch.uint8, device=dev)
        n_it = max(3, min(args.steps, 10))
        for it in range(2 + n_it):
            if it == 2:
                torch.cuda.synchronize()
                T.kernel_timing_enable(True)
            T.tree_gdn_fwd(gq, gk, gv, gg, gb, gplan, out=go, workspace=gws)
        gt = T.kernel_timing_read()
        T.kernel_timing_enable(False)
        p_ms, s_ms = gt["gdn_prepare"][0] / n_it, gt["gdn_scan"][0] / n_it
        # MFMA flop actually needed per 64-token chunk and head: K K^T, Q K^T (lower halves count in full here),
        # W S0, Q S0, P Vn, K^T Vn
        chunk_flop = 2.0 * (2 * 64 * 64 * 128 + 2 * 64 * 128 * 128 + 64 * 64 * 128 + 128 * 64 * 128)
        gdn = {"hk": ghk, "hv": ghv, "dk": 128, "dv": 128, "n_chunks": gplan.n_chunks, "saved_states": gplan.n_slots,
               "ms_prepare": round(p_ms, 4), "ms_scan": round(s_ms, 4), "ms_fwd": round(p_ms + s_ms, 4),
               "tokens_per_s": round(N / ((p_ms + s_ms) * 1e-3), 1),
               "chunk_tflops": round(chunk_flop * gplan.n_chunks * ghv / ((p_ms + s_ms) * 1e-3) / 1e12, 2),
               "us_per_chunk_step": round(s_ms * 1e3 / max(gplan.n_chunks, 1), 3),
               "workspace_mb": round(gws.numel() / 1e6, 1)}
        del gws
        if not args.no_gdn_bwd:
            gdo = torch.randn((N, ghv, 128), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
            bws = torch.empty(T.binding._lib().tt_tree_gdn_bwd_workspace(N, gplan.n_chunks, gplan.n_slots, ghk, ghv), dtype=torch.uint8,
                              device=dev)
            n_it = 3
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            for it in range(1 + n_it):
                if it == 1:
                    torch.cuda.synchronize()
                    T.kernel_timing_enable(True)
                    ev[0].record()
                T.tree_gdn_bwd(gq, gk, gv, gg, gb, gdo, gplan, workspace=bws)
            ev[1].record()
            ev[1].synchronize()
            bt = T.kernel_timing_read()
            T.kernel_timing_enable(False)
            # multiply-adds per chunk and head of the backward as written (the forward walk it recomputes included)
            bwd_flop = 2.0 * (2 * 64 * 64 * 128                       # prepare: K K^T, Q K^T
                              + 64 * 128 * 128 * 2                    # forward walk: W S0, Kd^T Vn
                              + 64 * 64 * 128 + 64 * 128 * 128 * 3    # reverse walk: P^T dO, Kd dS1, Qg^T dO, W^T dVn
                              + 64 * 128 * 128 * 3 + 64 * 64 * 256 + 64 * 64 * 128   # finish: dW, dQg, dKd, dA, dP
                              + 64 * 64 * 128 * 3 + 64 * 64 * 128)    # products with dP and dA, the two triangular solves
            b_ms = ev[0].elapsed_time(ev[1]) / n_it
            gdn.update({"ms_bwd": round(b_ms, 4),
                        "ms_bwd_kernels": {"prepare": round(bt["gdn_prepare"][0] / n_it, 4), "forward_walk": round(bt["gdn_bwd_fscan"][0] / n_it, 4),
                                           "reverse_walk": round(bt["gdn_bwd_rscan"][0] / n_it, 4), "finish": round(bt["gdn_bwd_finish"][0] / n_it, 4)},
                        "bwd_tflops": round(bwd_flop * gplan.n_chunks * ghv / (b_ms * 1e-3) / 1e12, 2),
                        "bwd_workspace_mb": round(bws.numel() / 1e6, 1)})
            del gdo, bws
        del gq, gk, gv, go

    # ---------------- CPU oracle on a bounded sample (context only) ----------------
    cpu = None
    if not args.no_cpu_baseline and n_prefix == 0:
        from oracle import attention as OA, meta as OM
        om = OM.dfs_meta(tree.parent, tree.seg_len, tree.trained)
        G = dims.hq // dims.hkv
        if cfg in (1, 2):
            t0c = time.perf_counter()
            n_groups = min(dims.hkv, 4)          # about 10 s of host time at config 2
            OA.branches(om, q.float().cpu(), k.float().cpu(), v.float().cpu(), do.float().cpu(), kv_heads=list(range(n_groups)))
            dtc = time.perf_counter() - t0c
            cpu_flop = 14.0 * G * n_groups * dims.d * pairs
            sample = "per-branch oracle, fwd+bwd, all branches, kv head groups 0..%d of %d (%d query heads)" % (n_groups - 1, dims.hkv, G * n_groups)
        else:
            # a slice of rows of the deepest leaf: same arithmetic, bounded time
            rows = list(range(N - 96, N))
            t0c = time.perf_counter()
            OA.rows(om, q.float().cpu(), k.float().cpu(), v.float().cpu(), do.float().cpu(), 0, rows)
            dtc = time.perf_counter() - t0c
            depth = om["tok_pos"][rows].astype(np.int64) + 1
            cpu_flop = 14.0 * G * dims.d * float(depth.sum())
            sample = "per-row oracle, fwd+bwd, last 96 tokens, kv head group 0 (%d query heads)" % G
        cpu = {"value": round(cpu_flop / dtc / 1e12, 6), "unit": "useful TFLOP/s", "cores": OA.n_threads(),
               "kind": "oracle", "sample": sample, "seconds": round(dtc, 2)}

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    out = {
        "metric": "tree-attn fwd+bwd useful TFLOP/s",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dims.dtype, "data": "synthetic",
        "config": {"workload": workload, "n_tokens": N, "n_prefix": n_prefix, "hq": dims.hq, "hkv": dims.hkv,
                   "d": dims.d, "visible_pairs": pairs, "useful_tflop_per_step": round(useful_flop / 1e12, 4)},
        "pct_of_bf16_mfma_peak": round(100.0 * value / PEAK_BF16_TFLOPS, 2),
        "ms_attn_fwd": round(ms_fwd, 4), "ms_attn_bwd": round(ms_bwd, 4), "ms_loss": round(ms_loss, 4),
        "ms_host_meta": round(float(np.mean(host_ms)), 4),
        "kernel_avg_ms": {n: round(t, 4) for n, t in kernel_ms.items()},
        "loss_hbm_gbps": None if loss_gbps is None else round(loss_gbps, 1),
        "loss_frac_of_hbm_peak": None if loss_gbps is None else round(loss_gbps / PEAK_HBM_GBPS, 4),
        "rope_hbm_gbps": None if rope_gbps is None else round(rope_gbps, 1),
        "loss_bwd_hbm_gbps": None if loss_bwd_gbps is None else round(loss_bwd_gbps, 1),
        "loss_bwd_frac_of_hbm_peak": None if loss_bwd_gbps is None else round(loss_bwd_gbps / PEAK_HBM_GBPS, 4),
        "linearized": lin,
        "partitioned": part,
        "tree_conv": conv,
        "tree_gdn": gdn,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
