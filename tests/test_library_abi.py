"""The C-ABI library loads on a CPU-only box, exports every symbol the header declares, and
reports invalid arguments by status code before launching anything (no GPU needed)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2511_00413_amd as T
from paper_2511_00413_amd import binding as B
from tt_testutil import ROOT


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "treetrain.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tt_[a-z_0-9]+)\s*\(", text)))


def test_exports_every_declared_symbol():
    lib = ctypes.CDLL(T.lib_path())
    names = _declared_symbols()
    assert {"tt_tree_build_meta", "tt_tree_attn_fwd", "tt_tree_attn_bwd", "tt_tree_weighted_logprob",
            "tt_tree_weighted_logprob_bwd", "tt_tree_weighted_logprob_fwd_bwd", "tt_tree_rope", "tt_tree_partition_sizes", "tt_tree_partition_plan", "tt_tree_path_weights", "tt_tree_conv_fwd", "tt_tree_conv_bwd", "tt_tree_conv_plan", "tt_tree_conv_plan_sizes",
            "tt_tree_conv_bwd_workspace", "tt_tree_gdn_plan_sizes", "tt_tree_gdn_plan", "tt_tree_gdn_workspace", "tt_tree_gdn_fwd",
            "tt_tree_gdn_bwd_workspace", "tt_tree_gdn_bwd_workspace_min", "tt_tree_gdn_bwd",
            "tt_tree_attn_partitioned_workspace", "tt_tree_attn_partitioned_fwd", "tt_tree_attn_partitioned_bwd",
            "tt_tree_attn_workspace", "tt_tree_meta_sizes", "tt_last_error", "tt_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert T.version() >= 100


def test_header_constants_match_binding():
    text = open(os.path.join(ROOT, "include", "treetrain.h")).read()
    assert int(re.search(r"#define TT_KTILE (\d+)", text).group(1)) == T.KTILE
    assert int(re.search(r"#define TT_DTYPE_BF16 (\d+)", text).group(1)) == B.DTYPE_BF16
    assert int(re.search(r"#define TT_DTYPE_FP32 (\d+)", text).group(1)) == B.DTYPE_FP32


@pytest.mark.parametrize("parent,seg,code", [
    ([1, 0], [1, 1], -3),          # cycle
    ([0], [1], -3),                # self loop
    ([-1, 5], [1, 1], -3),         # out of range
    ([-1, -2], [1, 1], -3),
    ([-1, 0], [1, -1], -2),        # negative length
    ([-1, 0], [2**30, 2**30], -2), # token count overflows int32
])
def test_meta_rejects_bad_trees(parent, seg, code):
    with pytest.raises(T.TreeTrainError) as e:
        T.tree_build_meta(parent, seg)
    assert e.value.status == code and T.last_error()


def test_meta_empty_inputs():
    m = T.tree_build_meta([], [])
    assert m.n_tokens == 0 and m.n_leaves == 0 and m.n_ktiles == 0
    m = T.tree_build_meta([-1, 0], [0, 0])
    assert m.n_tokens == 0 and m.n_leaves == 1


def test_device_calls_validate_before_launch():
    lib = B._lib()
    d = B._AttnDesc(16, 0, 4, 2, 128, 0, 0.1, 0, 0, 0, 0)
    assert lib.tt_tree_attn_workspace(ctypes.byref(d), 0) > 0
    null = ctypes.c_void_p(0)
    fake = ctypes.c_void_p(4096)         # never dereferenced: the call must fail before any launch
    rc = lib.tt_tree_attn_fwd(ctypes.byref(d), null, null, null, null, null, null, null, null, null, null, null, 0, null)
    assert rc == -1
    rc = lib.tt_tree_attn_fwd(ctypes.byref(d), fake, fake, fake, null, null, fake, fake, fake, fake, fake, null, 0, null)
    assert rc == -6                      # workspace missing
    rc = lib.tt_tree_attn_fwd(ctypes.byref(d), ctypes.c_void_p(4100), fake, fake, null, null, fake, fake, fake, fake, fake, fake, 1 << 20, null)
    assert rc == -5                      # misaligned q
    rc = lib.tt_tree_attn_fwd(ctypes.byref(d), fake, fake, fake, fake, null, fake, fake, fake, fake, fake, fake, 1 << 20, null)
    assert rc == -1                      # prefix pointers without n_prefix
    for bad in (dict(hq=3), dict(d=100), dict(dtype=7), dict(scale=0.0), dict(flags=64), dict(n_q=-1)):
        vals = dict(n_q=16, n_prefix=0, hq=4, hkv=2, d=128, dtype=0, scale=0.1, flags=0)
        vals.update(bad)
        dd = B._AttnDesc(vals["n_q"], vals["n_prefix"], vals["hq"], vals["hkv"], vals["d"], vals["dtype"],
                         vals["scale"], vals["flags"], 0, 0, 0)
        assert lib.tt_tree_attn_workspace(ctypes.byref(dd), 0) == 0, bad
        rc = lib.tt_tree_attn_fwd(ctypes.byref(dd), fake, fake, fake, null, null, fake, fake, fake, fake, fake, fake, 1 << 20, null)
        assert rc < 0 and T.last_error(), bad
    rc = lib.tt_tree_attn_bwd(ctypes.byref(d), *([fake] * 3), null, null, *([fake] * 3), *([fake] * 3), fake, fake, null, null, null, fake, 1 << 30, null)
    assert rc == -1                      # dv_own NULL
    rc = lib.tt_tree_weighted_logprob(4, 0, 0, fake, 0, fake, null, fake, null, null, null)
    assert rc == -2
    rc = lib.tt_tree_weighted_logprob(4, 128, 3, fake, 0, fake, null, fake, null, null, null)
    assert rc == -4
    rc = lib.tt_tree_weighted_logprob(4, 128, 0, fake, 64, fake, null, fake, null, null, null)
    assert rc == -2                      # row stride smaller than vocab
    rc = lib.tt_tree_weighted_logprob(4, 128, 0, null, 0, fake, null, fake, null, null, null)
    assert rc == -1
    fb = lib.tt_tree_weighted_logprob_fwd_bwd
    assert fb(4, 128, 0, fake, 0, fake, null, 1.0, fake, null, null, fake, 0, null) == -1         # lse is required
    assert fb(4, 128, 0, fake, 64, fake, null, 1.0, fake, fake, null, fake, 0, null) == -2        # stride < vocab
    assert fb(4, 128, 0, fake, 0, fake, null, float("inf"), fake, fake, null, fake, 0, null) == -2
    assert fb(4, 128, 0, fake, 256, fake, null, 1.0, fake, fake, null, fake, 128, null) == -2     # in place, unequal strides
    assert fb(4, 128, 9, fake, 0, fake, null, 1.0, fake, fake, null, fake, 0, null) == -4
    assert fb(0, 128, 0, null, 0, null, null, 1.0, null, null, null, null, 0, null) == 0          # nothing to do


def test_gdn_calls_validate_before_launch():
    """Shape, pointer, alignment and workspace errors of the gated-delta-rule entry points are reported before
    anything is launched (the pointers below are never dereferenced)."""
    lib = B._lib()
    null, fake = ctypes.c_void_p(0), ctypes.c_void_p(4096)
    n, hk, hv, nc, ns = 128, 2, 4, 2, 1
    plan = [fake] * 4                                        # chunk_tok0, chunk_len, chunk_src, chunk_dst

    def fwd(*, dk=128, dv=128, hv_=hv, scale=0.1, q=fake, o=fake, cap=null, state_out=null, ws=fake, ws_bytes=1 << 40, sched=null):
        return lib.tt_tree_gdn_fwd(n, hk, hv_, dk, dv, scale, q, fake, fake, fake, fake, nc, *plan, ns, cap, sched, null, state_out, o,
                                   ws, ws_bytes, null)

    def bwd(*, dk=128, hv_=hv, scale=0.1, q=fake, d_o=fake, dq=ctypes.c_void_p(24576), cap=null, d_state_out=null, ws=fake,
            ws_bytes=1 << 40, sched=null):
        return lib.tt_tree_gdn_bwd(n, hk, hv_, dk, 128, scale, q, fake, fake, fake, fake, d_o, nc, *plan, ns, cap, sched, null,
                                   d_state_out, dq, ctypes.c_void_p(8192), ctypes.c_void_p(12288), ctypes.c_void_p(16384),
                                   ctypes.c_void_p(20480), null, ws, ws_bytes, null)

    assert lib.tt_tree_gdn_workspace(nc, ns, hv) > 0
    assert lib.tt_tree_gdn_bwd_workspace(n, nc, ns, 0, hk, hv) > lib.tt_tree_gdn_workspace(nc, ns, hv)
    assert lib.tt_tree_gdn_bwd_workspace(n, nc, ns, 3, hk, hv) == lib.tt_tree_gdn_bwd_workspace(n, nc, ns, 0, hk, hv) + 3 * hv * 128 * 128 * 4
    least = lib.tt_tree_gdn_bwd_workspace_min(n, nc, ns, 0, hk, hv)
    assert 0 < least < lib.tt_tree_gdn_bwd_workspace(n, nc, ns, 0, hk, hv)       # one of the two key heads per pass
    assert lib.tt_tree_gdn_bwd_workspace_min(n, nc, ns, 0, 1, hv) == lib.tt_tree_gdn_bwd_workspace(n, nc, ns, 0, 1, hv)
    assert lib.tt_tree_gdn_bwd_workspace_min(n, nc, ns, 0, 3, hv) == 0           # hv not a multiple of hk
    assert bwd(ws_bytes=least - 256) == -6
    assert fwd(dk=64) == -8 and bwd(dk=64) == -8             # only 128 x 128 states (TT_ERR_UNSUPPORTED)
    assert fwd(hv_=3) == -2 and bwd(hv_=3) == -2             # hv not a multiple of hk
    assert fwd(scale=0.0) == -2 and bwd(scale=float("nan")) == -2
    assert fwd(q=null) == -1 and bwd(d_o=null) == -1 and bwd(dq=null) == -1
    assert fwd(cap=fake) == -1                               # chunk_cap without state_out
    assert bwd(d_state_out=fake) == -1                       # d_state_out without chunk_cap
    assert fwd(q=ctypes.c_void_p(4100)) == -5 and bwd(q=ctypes.c_void_p(4100)) == -5
    assert fwd(ws=null) == -6 and fwd(ws_bytes=16) == -6 and bwd(ws=null) == -6 and bwd(ws_bytes=16) == -6
    assert bwd(dq=fake, q=fake) == -2                        # an output aliases an input
    # a schedule whose host-side level table does not cover its segments, or with a missing device array
    lo = (ctypes.c_int32 * 2)(0, 1)
    bad = B._GdnSchedule(2, 1, ctypes.cast(lo, ctypes.c_void_p), fake, fake, fake, fake)
    assert fwd(sched=ctypes.byref(bad)) == -2 and bwd(sched=ctypes.byref(bad)) == -2
    missing = B._GdnSchedule(1, 1, ctypes.cast(lo, ctypes.c_void_p), null, fake, fake, fake)
    assert fwd(sched=ctypes.byref(missing)) == -1
    assert T.last_error()
