#!/usr/bin/env python3
"""Benchmark of the tree-attention hot path on one MI355X.

One "step" = one pass of the whole path over one synthetic tree: host metadata build
(tree_build_meta) + upload of the mask bounds and position ids, rotary embedding of Q and K with the tree
position ids, tree attention forward, backward, inverse rotation of dQ and dK, and the weighted log-prob
loss forward and backward.  The headline value is the attention forward+backward rate in *useful* TFLOP/s:
14 * Hq * D * visible_pairs flops (4 D per pair forward, 10 D backward) divided by the forward + backward
time measured with events on the launch stream, with no other instrumentation switched on.  Inputs are
resident in HBM before the timed region starts.  Per-kernel durations (kernel_avg_ms, roofline) come from
a second pass over the same steps with the library's per-kernel event bracketing on.

Prints one JSON line: metric / value / unit and the timing fields of the step, `roofline` (dominant kernel),
`linearized` (the per-branch forest through the same library: attention-only and whole-path speedup),
`other_configs` (configs 1, 3, 4 and the config-5 step, each with its own linearized run and CPU sample), `partitioned`, `tree_conv`, `tree_gdn`, `cpu_baseline`.
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
# WRITE_SIZE runs summarised in the named profile (FETCH_SIZE scaled x2.0, WRITE_SIZE x1.0 by the plain
# 1 GiB copy of the same run).  Offline measurements: reported only for the workload they cover, and
# refreshed whenever an attention kernel changes.
TRAFFIC_SOURCE = "profiles/attention_and_loss_kernels_cfg2.md"
MEASURED_TRAFFIC_BYTES = {
    (2, "attn_fwd"): 226.6e6 + 149.2e6,
    (2, "attn_dkdv"): 2377.8e6 + 206.3e6,
    (2, "attn_dq"): 513.2e6 + 151.4e6,
}

WORKLOADS = {
    1: "cfg1: worked 3-leaf tree, N=240, MHA 4x64, fp32",
    2: "cfg2: random depth-4 tree seed 117, N=16406, GQA 32/8, d=128, bf16, vocab 32768",
    3: "cfg3: agentic fan-out 8K->16x(2K->2x1K), N=73728, GQA 64/8, d=128, bf16, vocab 151936 in 4K-row chunks",
    4: "cfg4: deep chain seed 195, N=131091, GQA 32/8, d=128, bf16",
    5: "cfg5-step: 32768-token chunk (8 nodes) x 65536 cached prefix keys (variant b), GQA 64/8, d=128, bf16",
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
    ap.add_argument("--loss-two-pass", action="store_true",
                    help="loss forward and backward as two calls (two reads of the logits) instead of the one-pass call")
    ap.add_argument("--no-rope", action="store_true")
    ap.add_argument("--no-partitioned", action="store_true")
    ap.add_argument("--no-conv", action="store_true")
    ap.add_argument("--no-gdn", action="store_true")
    ap.add_argument("--no-gdn-bwd", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the step's device part")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short runs of the other full-size configurations (3, 4 and the config-5 step)")
    ap.add_argument("--other-configs-budget-s", type=float, default=150.0,
                    help="wall-clock budget for the other configurations; one that would start after it is skipped")
    ap.add_argument("--gdn-heads", type=int, default=32, help="value heads of the gated-delta-rule leg (key heads = half)")
    ap.add_argument("--gdn-capped-workspace-mb", type=int, default=1000,
                    help="also time the gated-delta-rule backward with its workspace capped at this size (0: skip)")
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


def make_workload(cfg):
    """(tree, n_prefix, prefix_visible, root_pos_offset) of a benchmark configuration."""
    import workloads as W
    if cfg == 5:
        s = W.step_cfg5()
        return s.chunk, s.n_prefix, s.prefix_visible, [int(s.prefix_visible.sum())]
    return W.tree_config(cfg), 0, None, None


def device_randn(torch, shape, std, dtype, seed, dev):
    """std * N(0,1) drawn on the device (timing-only inputs: same distribution as workloads.randn, drawn
    where they are used because the large configurations would spend minutes in the host generator)."""
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    return (torch.randn(shape, generator=gen, device=dev, dtype=torch.float32) * std).to(dtype)


class PathRun:
    """Device buffers and the step of one pass of the hot path over one tree or forest.

    step(events): host metadata + uploads, RoPE(Q, K), attention forward, backward, inverse RoPE(dQ, dK),
    loss forward + backward; events (6 of them) are recorded before the rotary embedding, before and after
    the forward, after the backward, after the inverse rotation and after the loss."""

    def __init__(self, T, torch, dev, dims, tree, n_prefix, prefix_visible, root_off, q_raw, k_raw, v, do, kp=None, vp=None,
                 logits=None, target=None, weight=None, do_rope=True, loss_one_pass=True):
        self.T, self.torch, self.dims, self.tree = T, torch, dims, tree
        self.n_prefix, self.prefix_visible, self.root_off = n_prefix, prefix_visible, root_off
        self.meta = self.build_meta()
        N = self.N = self.meta.n_tokens
        self.q_raw, self.k_raw, self.v, self.do, self.kp, self.vp = q_raw, k_raw, v, do, kp, vp
        self.do_rope = do_rope and dims.dtype == "bf16"
        self.q = torch.empty_like(q_raw) if self.do_rope else q_raw
        self.k = torch.empty_like(k_raw) if self.do_rope else k_raw
        self.dkp = self.dvp = None
        if n_prefix:
            self.dkp = torch.zeros(kp.shape, dtype=torch.float32, device=dev)
            self.dvp = torch.zeros(kp.shape, dtype=torch.float32, device=dev)
        nk = self.meta.n_ktiles
        self.kend_d = torch.empty(n_prefix + N, dtype=torch.int32, device=dev)
        self.kmin_d = torch.empty(nk, dtype=torch.int32, device=dev)
        self.kmax_d = torch.empty(nk, dtype=torch.int32, device=dev)
        self.pos_d = torch.empty(N, dtype=torch.int32, device=dev)
        self.w_d = torch.empty(N, dtype=torch.float32, device=dev)
        self.kend_h = torch.empty(n_prefix + N, dtype=torch.int32).pin_memory()
        self.kmin_h = torch.empty(nk, dtype=torch.int32).pin_memory()
        self.kmax_h = torch.empty(nk, dtype=torch.int32).pin_memory()
        self.pos_h = torch.empty(N, dtype=torch.int32).pin_memory()
        self.w_h = torch.empty(N, dtype=torch.float32).pin_memory()
        self.weight_override = weight
        self.ws_f = torch.empty(T.tree_attn_workspace(self.q, self.k, v, n_prefix, False), dtype=torch.uint8, device=dev)
        self.ws_b = torch.empty(T.tree_attn_workspace(self.q, self.k, v, n_prefix, True), dtype=torch.uint8, device=dev)
        self.o = torch.empty_like(q_raw)
        self.lse = torch.empty((dims.hq, N), dtype=torch.float32, device=dev)
        self.dq, self.dk, self.dv = torch.empty_like(q_raw), torch.empty_like(k_raw), torch.empty_like(v)
        self.logits, self.target = logits, target
        self.do_loss = logits is not None
        self.loss_one_pass = loss_one_pass
        if self.do_loss:
            self.logp = torch.empty(N, dtype=torch.float32, device=dev)
            self.lse_l = torch.empty(N, dtype=torch.float32, device=dev)
            self.loss_acc = torch.zeros(1, dtype=torch.float32, device=dev)
            self.dlogits = torch.empty_like(logits)        # gradient w.r.t. the logits (same row chunking)
        self.host_ms = []

    def build_meta(self):
        t = self.tree
        return self.T.tree_build_meta(t.parent, t.seg_len, t.trained, root_pos_offset=self.root_off, n_prefix=self.n_prefix,
                                      prefix_visible=self.prefix_visible)

    def step(self, events=None):
        T, N = self.T, self.N
        t0 = time.perf_counter()
        m = self.build_meta()                                   # a1-a4 on the host
        self.kend_h.numpy()[:] = m.kend
        self.kmin_h.numpy()[:] = m.ktile_kend_min
        self.kmax_h.numpy()[:] = m.ktile_kend_max
        self.kend_d.copy_(self.kend_h, non_blocking=True)
        self.kmin_d.copy_(self.kmin_h, non_blocking=True)
        self.kmax_d.copy_(self.kmax_h, non_blocking=True)
        if self.weight_override is None:
            self.w_h.numpy()[:] = m.tok_weight
            self.w_d.copy_(self.w_h, non_blocking=True)
        if self.do_rope:
            self.pos_h.numpy()[:] = m.tok_pos
            self.pos_d.copy_(self.pos_h, non_blocking=True)
        self.host_ms.append((time.perf_counter() - t0) * 1e3)
        self.device_part(events)

    def device_part(self, events=None):
        """The library calls of one step (what a HIP graph of the step holds)."""
        T, N = self.T, self.N
        w_d = self.w_d if self.weight_override is None else self.weight_override
        kb = (self.kend_d, self.kmin_d, self.kmax_d)
        if events:
            events[0].record()
        if self.do_rope:
            T.tree_rope(self.q_raw, self.pos_d, out=self.q)
            T.tree_rope(self.k_raw, self.pos_d, out=self.k)
        if events:
            events[1].record()
        T.tree_attn_fwd(self.q, self.k, self.v, *kb, k_prefix=self.kp, v_prefix=self.vp, o=self.o, lse=self.lse, workspace=self.ws_f)
        if events:
            events[2].record()
        T.tree_attn_bwd(self.q, self.k, self.v, *kb, self.o, self.do, self.lse, k_prefix=self.kp, v_prefix=self.vp,
                        dk_prefix_acc=self.dkp, dv_prefix_acc=self.dvp, dq=self.dq, dk=self.dk, dv=self.dv, workspace=self.ws_b)
        if events:
            events[3].record()
        if self.do_rope:
            T.tree_rope(self.dq, self.pos_d, inverse=True, out=self.dq)
            T.tree_rope(self.dk, self.pos_d, inverse=True, out=self.dk)
        if events:
            events[4].record()
        if self.do_loss:
            self.loss_acc.zero_()
            rows = self.logits.shape[0]
            for lo in range(0, N, rows):
                n = min(rows, N - lo)
                if self.loss_one_pass:
                    T.tree_weighted_logprob_fwd_bwd(self.logits[:n], self.target[lo:lo + n], w_d[lo:lo + n], loss_acc=self.loss_acc,
                                                    logp=self.logp[lo:lo + n], lse=self.lse_l[lo:lo + n], out=self.dlogits[:n])
                else:
                    T.tree_weighted_logprob(self.logits[:n], self.target[lo:lo + n], w_d[lo:lo + n], loss_acc=self.loss_acc,
                                            logp=self.logp[lo:lo + n], lse=self.lse_l[lo:lo + n])
                    T.tree_weighted_logprob_bwd(self.logits[:n], self.target[lo:lo + n], w_d[lo:lo + n], self.lse_l[lo:lo + n],
                                                out=self.dlogits[:n])
        if events:
            events[5].record()

    def timed(self, warmup, steps):
        """Runs warmup + steps; returns (wall seconds of the timed steps, per-phase mean ms)."""
        torch = self.torch
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(steps)]
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        self.host_ms.clear()
        t0 = time.perf_counter()
        for s in range(steps):
            self.step(ev[s])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        names = ("rope", "attn_fwd", "attn_bwd", "rope_inverse", "loss")
        ms = {n: sum(e[i].elapsed_time(e[i + 1]) for e in ev) / steps for i, n in enumerate(names)}
        ms["path"] = sum(e[0].elapsed_time(e[5]) for e in ev) / steps
        return wall, ms


def linearized_run(T, torch, dev, dims, run: PathRun, linearize):
    """The same path on the K-chain forest (every root-to-leaf branch written out in full, packed): the
    paper's baseline layout, run through the same library so that only the redundancy differs."""
    import workloads as W
    idx, lparent, lseg = linearize.linearized_forest(run.meta)
    idx_d = torch.from_numpy(idx).to(dev)
    forest = W.Tree(parent=lparent, seg_len=lseg, trained=np.ones(len(lparent), dtype=np.uint8), name="linearized")
    ql, kl, vl, dol = (x.index_select(0, idx_d) for x in (run.q_raw, run.k_raw, run.v, run.do))
    tl = wl = None
    if run.do_loss:
        tl = run.target.index_select(0, idx_d)
        # per-branch weights (1/K on trained tokens): the tree weight g/K split over the g branches of a token
        g_tok = torch.from_numpy(run.meta.node_g[run.meta.tok_node].astype(np.float32)).to(dev)
        wl = (run.w_d / g_tok).index_select(0, idx_d)
    lin = PathRun(T, torch, dev, dims, forest, 0, None, None, ql, kl, vl, dol, logits=run.logits, target=tl, weight=wl,
                  do_rope=run.do_rope, loss_one_pass=run.loss_one_pass)
    return lin, idx


def speedup_record(ms_tree, ms_lin, run: PathRun, lin: PathRun, pairs, pairs_lin):
    attn_t, attn_l = ms_tree["attn_fwd"] + ms_tree["attn_bwd"], ms_lin["attn_fwd"] + ms_lin["attn_bwd"]
    r_tok, r_pair = lin.N / run.N, pairs_lin / pairs
    rec = {"ms_fwd_bwd": round(attn_l, 4), "n_lin": lin.N, "pairs_lin": pairs_lin, "speedup": round(attn_l / attn_t, 3),
           "r_tok": round(r_tok, 3), "r_pair": round(r_pair, 3),
           "speedup_over_r_tok": round(attn_l / attn_t / r_tok, 3), "speedup_over_r_pair": round(attn_l / attn_t / r_pair, 3),
           # the whole device path (rotary embedding, attention, inverse rotation, loss forward + backward): the
           # token-linear steps speed up by r_tok, the attention by at most r_pair
           "path": {"steps": "rope + attn fwd + attn bwd + inverse rope" + ((" + loss fwd and bwd in one pass" if run.loss_one_pass else " + loss fwd + loss bwd") if run.do_loss else ""),
                    "ms_tree": round(ms_tree["path"], 4), "ms_linearized": round(ms_lin["path"], 4),
                    "speedup": round(ms_lin["path"] / ms_tree["path"], 3),
                    "speedup_over_r_tok": round(ms_lin["path"] / ms_tree["path"] / r_tok, 3),
                    "ms_tree_by_step": {k_: round(v_, 4) for k_, v_ in ms_tree.items() if k_ != "path"},
                    "ms_linearized_by_step": {k_: round(v_, 4) for k_, v_ in ms_lin.items() if k_ != "path"}}}
    return rec


def other_config(T, torch, dev, linearize, cfg, with_linearized, with_cpu):
    """Short run (2 warm-up + 3 timed steps) of another configuration: attention rates, the linearized forest
    beside it, the path-level times and a bounded sample of the CPU oracle; inputs drawn on the device."""
    import workloads as W
    dims = W.DIMS[cfg]
    tree, n_prefix, vis, root_off = make_workload(cfg)
    N = int(tree.seg_len.sum())
    tdt = torch.bfloat16 if dims.dtype == "bf16" else torch.float32
    q = device_randn(torch, (N, dims.hq, dims.d), dims.std, tdt, cfg * 1000 + 1, dev)
    k = device_randn(torch, (N, dims.hkv, dims.d), dims.std, tdt, cfg * 1000 + 2, dev)
    v = device_randn(torch, (N, dims.hkv, dims.d), dims.std, tdt, cfg * 1000 + 3, dev)
    do = device_randn(torch, (N, dims.hq, dims.d), dims.std, tdt, cfg * 1000 + 4, dev)
    kp = vp = None
    if n_prefix:
        kp = device_randn(torch, (n_prefix, dims.hkv, dims.d), dims.std, tdt, cfg * 1000 + 102, dev)
        vp = device_randn(torch, (n_prefix, dims.hkv, dims.d), dims.std, tdt, cfg * 1000 + 103, dev)
    logits = target = None
    if dims.vocab > 0:
        rows = min(N, 4096)
        logits = device_randn(torch, (rows, dims.vocab), dims.logit_std,
                              torch.bfloat16 if dims.logit_dtype == "bf16" else torch.float32, cfg * 1000 + 5, dev)
        gen = torch.Generator(device=dev)
        gen.manual_seed(cfg * 1000 + 6)
        target = torch.randint(0, dims.vocab, (N,), generator=gen, device=dev, dtype=torch.int32)
    run = PathRun(T, torch, dev, dims, tree, n_prefix, vis, root_off, q, k, v, do, kp, vp, logits, target)
    pairs = linearize.visible_pairs(run.meta)
    _, ms = run.timed(2, 3)
    attn = ms["attn_fwd"] + ms["attn_bwd"]
    useful = 14.0 * dims.hq * dims.d * pairs
    rec = {"workload": WORKLOADS[cfg], "n_tokens": N, "n_prefix": n_prefix, "visible_pairs": pairs,
           "dtype": dims.dtype, "useful_tflops": round(useful / (attn * 1e-3) / 1e12, 2 if dims.dtype == "bf16" else 4),
           ("pct_of_bf16_mfma_peak" if dims.dtype == "bf16" else "pct_of_fp32_alu_peak"):
               round(100.0 * useful / (attn * 1e-3) / 1e12 / (PEAK_BF16_TFLOPS if dims.dtype == "bf16" else 157.3), 2),
           "ms_attn_fwd": round(ms["attn_fwd"], 4), "ms_attn_bwd": round(ms["attn_bwd"], 4), "ms_path": round(ms["path"], 4),
           "ms_host_meta": round(float(np.mean(run.host_ms)), 4), "steps": 3, "warmup": 2}
    if n_prefix:
        rec["prefix_grad_accumulate_bytes"] = 2 * n_prefix * dims.hkv * dims.d * 4
    if with_linearized and n_prefix == 0:
        lin, _ = linearized_run(T, torch, dev, dims, run, linearize)
        _, ms_l = lin.timed(1, 3)
        rec["linearized"] = speedup_record(ms, ms_l, run, lin, pairs, linearize.visible_pairs(lin.meta))
        del lin
    if with_cpu and n_prefix == 0:
        rec["cpu_baseline"] = cpu_rows_sample(tree, dims, q, k, v, do, n_rows=512)
    del run, q, k, v, do, kp, vp, logits, target
    torch.cuda.empty_cache()
    return rec


def leg_partitioned(c):
    args, T, torch, dev, cfg, dims, tree, meta, N, n_prefix = c.args, c.T, c.torch, c.dev, c.cfg, c.dims, c.tree, c.meta, c.N, c.n_prefix
    q, k, v, do, lse, ms_fwd, ms_bwd, pairs = c.q, c.k, c.v, c.do, c.lse, c.ms_fwd, c.ms_bwd, c.pairs
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
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_it + 1)]
        def part_step():
            T.tree_attn_partitioned_fwd(q, k, v, plan, o=op, lse=lsep, workspace=wsp)
            T.tree_attn_partitioned_bwd(q, k, v, plan, op, do, lsep, dq=dqp, dk=dkp_, dv=dvp_, workspace=wsp)
        for it in range(2):
            part_step()
        evs[0].record()
        for it in range(n_it):
            part_step()
            evs[it + 1].record()
        torch.cuda.synchronize()
        per_step = [evs[i].elapsed_time(evs[i + 1]) for i in range(n_it)]
        ms_part = evs[0].elapsed_time(evs[n_it]) / n_it
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
                "ms_fwd_bwd_per_step": [round(x, 3) for x in per_step],
                "ms_whole_fwd_bwd": round(ms_fwd + ms_bwd, 4),
                "ratio_to_whole": round(ms_part / (ms_fwd + ms_bwd), 3),
                "ms_attn_kernels": round(sum(pt[n][0] for n in ("attn_fwd", "attn_dkdv", "attn_dq", "attn_plan", "attn_reduce")) / n_it, 4),
                "ms_gather": round(pt["part_gather"][0] / n_it, 4), "ms_scatter": round(pt["part_scatter"][0] / n_it, 4),
                "movement_gb": round((gather_b + scatter_b) / 1e9, 4),
                "movement_hbm_gbps": round((gather_b + scatter_b) / (move_ms * 1e-3) / 1e9, 1) if move_ms > 0 else None,
                "ms_host_plan": round(plan_ms, 3)}
        del op, lsep, dqp, dkp_, dvp_, wsp

    return part


def leg_conv(c):
    args, T, torch, dev, cfg, dims, tree, meta, N, n_prefix = c.args, c.T, c.torch, c.dev, c.cfg, c.dims, c.tree, c.meta, c.N, c.n_prefix
    q, k, v, do, lse, ms_fwd, ms_bwd, pairs = c.q, c.k, c.v, c.do, c.lse, c.ms_fwd, c.ms_bwd, c.pairs
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

    return conv


def leg_gdn(c):
    args, T, torch, dev, cfg, dims, tree, meta, N, n_prefix = c.args, c.T, c.torch, c.dev, c.cfg, c.dims, c.tree, c.meta, c.N, c.n_prefix
    q, k, v, do, lse, ms_fwd, ms_bwd, pairs = c.q, c.k, c.v, c.do, c.lse, c.ms_fwd, c.ms_bwd, c.pairs
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
            bws = torch.empty(T.tree_gdn_bwd_workspace(N, ghk, ghv, gplan), dtype=torch.uint8, device=dev)
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
            # the same with the workspace capped at 1 GB: the call then takes the heads in passes of whole key-head groups
            cap = args.gdn_capped_workspace_mb * 1_000_000
            if cap > 0 and T.tree_gdn_bwd_workspace(N, ghk, ghv, gplan, smallest=True) <= cap < bws.numel():
                small = bws[:cap]
                for it in range(1 + n_it):
                    if it == 1:
                        ev[0].record()
                    T.tree_gdn_bwd(gq, gk, gv, gg, gb, gdo, gplan, workspace=small)
                ev[1].record()
                ev[1].synchronize()
                gdn.update({"ms_bwd_capped_workspace": round(ev[0].elapsed_time(ev[1]) / n_it, 4), "capped_workspace_mb": cap / 1e6})
            del gdo, bws
        del gq, gk, gv, go

    return gdn


def leg_cpu(c):
    args, T, torch, dev, cfg, dims, tree, meta, N, n_prefix = c.args, c.T, c.torch, c.dev, c.cfg, c.dims, c.tree, c.meta, c.N, c.n_prefix
    q, k, v, do, lse, ms_fwd, ms_bwd, pairs = c.q, c.k, c.v, c.do, c.lse, c.ms_fwd, c.ms_bwd, c.pairs
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
            cpu = {"value": round(cpu_flop / dtc / 1e12, 6), "unit": "useful TFLOP/s", "cores": OA.n_threads(),
                   "kind": "oracle", "sample": sample, "seconds": round(dtc, 2)}
        else:
            cpu = cpu_rows_sample(tree, dims, q, k, v, do)
    return cpu


def cpu_rows_sample(tree, dims, q, k, v, do, n_rows=96):
    """The oracle on a slice of rows of the deepest leaf (the last tokens in DFS order), kv head group 0: the same
    arithmetic as a full run, bounded time."""
    from oracle import attention as OA, meta as OM
    om = OM.dfs_meta(tree.parent, tree.seg_len, tree.trained)
    N = om["n_tokens"]
    G = dims.hq // dims.hkv
    rows = list(range(max(0, N - n_rows), N))
    # only kv head 0 and its query heads travel to the host
    qc, kc, vc, dc = (x[:, :h].float().cpu() for x, h in ((q, G), (k, 1), (v, 1), (do, G)))
    t0c = time.perf_counter()
    OA.rows(om, qc, kc, vc, dc, 0, rows)
    dtc = time.perf_counter() - t0c
    depth = om["tok_pos"][rows].astype(np.int64) + 1
    cpu_flop = 14.0 * G * dims.d * float(depth.sum())
    return {"value": round(cpu_flop / dtc / 1e12, 6), "unit": "useful TFLOP/s", "cores": OA.n_threads(), "kind": "oracle",
            "sample": "per-row oracle, fwd+bwd, last %d tokens, kv head group 0 (%d query heads)" % (len(rows), G),
            "seconds": round(dtc, 2)}


class Ctx:
    pass


def guarded(fn, *a):
    """The side legs report a failure in their own field; the headline has been measured by then and must get out."""
    try:
        return fn(*a)
    except Exception as e:      # noqa: BLE001
        return {"error": f"{fn.__name__}: {type(e).__name__}: {e}"[:300]}


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

    # ---------------- workload (headline configuration: inputs from the seeded host generator) ----------------
    tree, n_prefix, prefix_visible, root_off = make_workload(cfg)
    N = int(tree.seg_len.sum())
    q, k, v, do = (x.to(dev) for x in W.attn_inputs(N, N, dims, cfg))
    kp = vp = None
    if n_prefix:
        _, kp, vp, _ = (x.to(dev) for x in W.attn_inputs(1, n_prefix, dims, cfg + 100))
    do_loss = dims.vocab > 0 and not args.no_loss
    logits = target = None
    if do_loss:
        # value distribution of the config; drawn on the device to keep start-up short
        chunk_rows = N if cfg != 3 else 4096
        logits = device_randn(torch, (chunk_rows, dims.vocab), dims.logit_std,
                              torch.bfloat16 if dims.logit_dtype == "bf16" else torch.float32, cfg * 1000 + 5, dev)
        gen = torch.Generator(device=dev)
        gen.manual_seed(cfg * 1000 + 6)
        target = torch.randint(0, dims.vocab, (N,), generator=gen, device=dev, dtype=torch.int32)
    run = PathRun(T, torch, dev, dims, tree, n_prefix, prefix_visible, root_off, q, k, v, do, kp, vp, logits, target,
                  do_rope=not args.no_rope, loss_one_pass=not args.loss_two_pass)
    meta = run.meta
    pairs = linearize.visible_pairs(meta)

    # ---------------- the timed region: W warm-up steps, K timed steps, nothing else switched on ----------------
    wall, ms = run.timed(args.warmup, args.steps)
    ms_fwd, ms_bwd, ms_loss = ms["attn_fwd"], ms["attn_bwd"], ms["loss"]
    host_ms = float(np.mean(run.host_ms))
    useful_flop = 14.0 * dims.hq * dims.d * pairs
    value = useful_flop / ((ms_fwd + ms_bwd) * 1e-3) / 1e12

    # ---------------- second pass over the same steps with per-kernel event bracketing ----------------
    k_steps = args.steps
    T.kernel_timing_enable(True)
    for _ in range(k_steps):
        run.step()
    torch.cuda.synchronize()
    ktimes = T.kernel_timing_read()
    T.kernel_timing_enable(False)

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
        traffic = MEASURED_TRAFFIC_BYTES.get((cfg, dom))
        roofline = {"kernel": dom, "bound": "mfma" if dims.dtype == "bf16" else "alu", "achieved": round(achieved, 2),
                    "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4), "traffic": traffic,
                    "traffic_source": TRAFFIC_SOURCE if traffic is not None else None,
                    "avg_ms": round(avg_ms, 4), "launches_timed": attn_k[dom][1],
                    "algorithmic_flop_per_launch": alg_flop[dom] * dims.hq * dims.d * pairs}
    loss_gbps = loss_bwd_gbps = loss_fused_gbps = None
    if do_loss:
        esz = 2 if dims.logit_dtype == "bf16" else 4
        if "loss_fused" in kernel_ms:
            # one read of the logits + one write of the gradient + target, weight in, logp, lse out per row
            loss_fused_gbps = N * (2 * dims.vocab * esz + 16) / (ktimes["loss_fused"][0] / k_steps * 1e-3) / 1e9
            # the two separate kernels on the same rows, outside the step, for their own figures
            T.kernel_timing_enable(True)
            rows = run.logits.shape[0]
            for _ in range(3):
                for lo in range(0, N, rows):
                    n = min(rows, N - lo)
                    T.tree_weighted_logprob(run.logits[:n], run.target[lo:lo + n], run.w_d[lo:lo + n], loss_acc=run.loss_acc,
                                            logp=run.logp[lo:lo + n], lse=run.lse_l[lo:lo + n])
                    T.tree_weighted_logprob_bwd(run.logits[:n], run.target[lo:lo + n], run.w_d[lo:lo + n], run.lse_l[lo:lo + n],
                                                out=run.dlogits[:n])
            torch.cuda.synchronize()
            lt = T.kernel_timing_read()
            T.kernel_timing_enable(False)
            t_rows, t_bwd = lt["loss_rows"][0] / 3, lt["loss_bwd"][0] / 3
        else:
            t_rows, t_bwd = ktimes["loss_rows"][0] / k_steps, ktimes["loss_bwd"][0] / k_steps
        loss_gbps = N * (dims.vocab * esz + 12) / (t_rows * 1e-3) / 1e9
        # backward: one read of the logits + one write of the gradient + target, weight, lse per row
        loss_bwd_gbps = N * (2 * dims.vocab * esz + 12) / (t_bwd * 1e-3) / 1e9
    rope_gbps = None
    if run.do_rope and "rope" in kernel_ms:
        rope_bytes = 2 * (dims.hq + dims.hkv) * N * dims.d * 2 * 2 + 4 * N * 4      # q, k, dq, dk: read + write; positions
        rope_gbps = rope_bytes / (ktimes["rope"][0] / k_steps * 1e-3) / 1e9

    # ---------------- linearised per-branch baseline on the same GPU ----------------
    lin = None
    if not args.no_linearized and n_prefix == 0:
        lrun, _ = linearized_run(T, torch, dev, dims, run, linearize)
        _, ms_l = lrun.timed(2, max(3, min(args.steps, 10)))
        lin = speedup_record(ms, ms_l, run, lrun, pairs, linearize.visible_pairs(lrun.meta))
        del lrun
        torch.cuda.empty_cache()

    c = Ctx()
    c.args, c.T, c.torch, c.dev, c.cfg, c.dims, c.tree, c.meta, c.N, c.n_prefix = args, T, torch, dev, cfg, dims, tree, meta, N, n_prefix
    c.q, c.k, c.v, c.do, c.lse, c.ms_fwd, c.ms_bwd, c.pairs = run.q, run.k, run.v, run.do, run.lse, ms_fwd, ms_bwd, pairs
    part = guarded(leg_partitioned, c)
    conv = guarded(leg_conv, c)
    gdn = guarded(leg_gdn, c)
    cpu = guarded(leg_cpu, c)

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---------------- the other full-size configurations, briefly ----------------
    others = None
    if not args.no_other_configs and cfg == 2:
        del c
        torch.cuda.empty_cache()
        others = {}
        t_start = time.perf_counter()
        for oc in (1, 3, 4, 5):
            if time.perf_counter() - t_start > args.other_configs_budget_s:
                others[f"cfg{oc}"] = {"skipped": "time budget"}
                continue
            others[f"cfg{oc}" if oc != 5 else "cfg5_step"] = guarded(other_config, T, torch, dev, linearize, oc,
                                                                         not args.no_linearized, not args.no_cpu_baseline)

    out = {
        "metric": "tree-attn fwd+bwd useful TFLOP/s",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dims.dtype, "data": "synthetic",
        "config": {"workload": WORKLOADS[cfg], "n_tokens": N, "n_prefix": n_prefix, "hq": dims.hq, "hkv": dims.hkv,
                   "d": dims.d, "visible_pairs": pairs, "useful_tflop_per_step": round(useful_flop / 1e12, 4)},
        "pct_of_bf16_mfma_peak": round(100.0 * value / PEAK_BF16_TFLOPS, 2),
        "ms_attn_fwd": round(ms_fwd, 4), "ms_attn_bwd": round(ms_bwd, 4), "ms_loss": round(ms_loss, 4),
        "ms_rope": round(ms["rope"] + ms["rope_inverse"], 4), "ms_device_path": round(ms["path"], 4),
        "ms_host_meta": round(host_ms, 4),
        "kernel_avg_ms": {n: round(t, 4) for n, t in kernel_ms.items()},
        "kernel_avg_ms_source": "second pass over the same steps with per-kernel event bracketing (the headline is timed without it)",
        "loss_hbm_gbps": None if loss_gbps is None else round(loss_gbps, 1),
        "loss_frac_of_hbm_peak": None if loss_gbps is None else round(loss_gbps / PEAK_HBM_GBPS, 4),
        "rope_hbm_gbps": None if rope_gbps is None else round(rope_gbps, 1),
        "rope_frac_of_hbm_peak": None if rope_gbps is None else round(rope_gbps / PEAK_HBM_GBPS, 4),
        "loss_bwd_hbm_gbps": None if loss_bwd_gbps is None else round(loss_bwd_gbps, 1),
        "loss_bwd_frac_of_hbm_peak": None if loss_bwd_gbps is None else round(loss_bwd_gbps / PEAK_HBM_GBPS, 4),
        "loss_one_pass_hbm_gbps": None if loss_fused_gbps is None else round(loss_fused_gbps, 1),
        "loss_one_pass_frac_of_hbm_peak": None if loss_fused_gbps is None else round(loss_fused_gbps / PEAK_HBM_GBPS, 4),
        "hip_graph": None,
        "linearized": lin,
        "partitioned": part,
        "tree_conv": conv,
        "tree_gdn": gdn,
        "other_configs": others,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    # ---------------- last: the device part of the step as one HIP graph ----------------
    # (after everything else has been measured, and guarded: a capture that fails must not cost the line)
    if not args.no_graph:
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                run.device_part()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                run.device_part()
            n_rep = max(3, min(args.steps, 10))
            gev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            g.replay()
            gev[0].record()
            for i in range(n_rep):
                g.replay()
            gev[1].record()
            torch.cuda.synchronize()
            out["hip_graph"] = {"ms_device_path_replayed": round(gev[0].elapsed_time(gev[1]) / n_rep, 4),
                                "ms_device_path_eager": round(ms["path"], 4), "replays": n_rep}
        except Exception as e:      # noqa: BLE001 -- reported in the line instead of losing it
            out["hip_graph"] = {"error": f"{type(e).__name__}: {e}"[:300]}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
