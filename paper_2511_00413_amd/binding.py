"""ctypes binding of libtreetrain.so.  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
KTILE = 64
DTYPE_BF16, DTYPE_FP32 = 0, 1
FLAG_REFERENCE_KERNELS = 1

_c_i32p = ctypes.POINTER(ctypes.c_int32)
_c_u8p = ctypes.POINTER(ctypes.c_uint8)
_c_f32p = ctypes.POINTER(ctypes.c_float)
_vp = ctypes.c_void_p


class TreeTrainError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libtreetrain status {status}: {message}")
        self.status = status


class _MetaSizes(ctypes.Structure):
    _fields_ = [("n_nodes", ctypes.c_int32), ("n_tokens", ctypes.c_int32), ("n_leaves", ctypes.c_int32),
                ("n_roots", ctypes.c_int32), ("n_ktiles", ctypes.c_int32)]


class _PartitionSizes(ctypes.Structure):
    _fields_ = [("n_parts", ctypes.c_int32), ("n_tokens", ctypes.c_int32), ("max_part_tokens", ctypes.c_int32),
                ("max_prefix", ctypes.c_int32), ("sum_prefix", ctypes.c_int64), ("sum_ktiles", ctypes.c_int64)]


class _PartitionPlan(ctypes.Structure):
    _fields_ = [("n_parts", ctypes.c_int32), ("n_tokens", ctypes.c_int32),
                ("part_tok_off", _vp), ("part_prefix_off", _vp), ("part_ktile_off", _vp),
                ("part_own_start", _vp), ("part_prefix_start", _vp),
                ("own_tok", _vp), ("prefix_tok", _vp), ("kend", _vp), ("kt_min", _vp), ("kt_max", _vp)]


class _AttnDesc(ctypes.Structure):
    _fields_ = [("n_q", ctypes.c_int32), ("n_prefix", ctypes.c_int32), ("hq", ctypes.c_int32),
                ("hkv", ctypes.c_int32), ("d", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("scale", ctypes.c_float), ("flags", ctypes.c_int32),
                ("q_stride_tok", ctypes.c_int64), ("k_stride_tok", ctypes.c_int64),
                ("v_stride_tok", ctypes.c_int64)]


def lib_path() -> str:
    return os.path.join(HERE, "libtreetrain.so")


_LIB = None


def _lib() -> ctypes.CDLL:
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError(
                f"{path} is missing: build it with `python -m paper_2511_00413_amd.build` "
                "(there is no fallback implementation)")
        # The library and PyTorch must share one HIP runtime.  PyTorch ships its own copy under the same soname, so
        # whichever is loaded first serves both; with the system's copy loaded first, device calls made after
        # `import torch` have failed with "no ROCm-capable device".  Load PyTorch's first when it is there.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        lib = ctypes.CDLL(path)
        lib.tt_last_error.restype = ctypes.c_char_p
        lib.tt_version.restype = ctypes.c_int32
        lib.tt_tree_attn_workspace.restype = ctypes.c_size_t
        lib.tt_tree_attn_workspace.argtypes = [ctypes.POINTER(_AttnDesc), ctypes.c_int32]
        lib.tt_tree_meta_sizes.restype = ctypes.c_int32
        lib.tt_tree_meta_sizes.argtypes = [ctypes.c_int32, _vp, _vp, ctypes.c_int32, ctypes.POINTER(_MetaSizes)]
        lib.tt_tree_build_meta.restype = ctypes.c_int32
        lib.tt_tree_build_meta.argtypes = [ctypes.c_int32, _vp, _vp, _vp, _vp, _vp, ctypes.c_int32,
                                           ctypes.c_int32, _vp] + [_vp] * 13
        lib.tt_tree_attn_fwd.restype = ctypes.c_int32
        lib.tt_tree_attn_fwd.argtypes = [ctypes.POINTER(_AttnDesc)] + [_vp] * 10 + [_vp, ctypes.c_size_t, _vp]
        lib.tt_tree_attn_bwd.restype = ctypes.c_int32
        lib.tt_tree_attn_bwd.argtypes = [ctypes.POINTER(_AttnDesc)] + [_vp] * 16 + [_vp, ctypes.c_size_t, _vp]
        lib.tt_tree_weighted_logprob.restype = ctypes.c_int32
        lib.tt_tree_weighted_logprob.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, _vp,
                                                 ctypes.c_int64, _vp, _vp, _vp, _vp, _vp, _vp]
        lib.tt_tree_weighted_logprob_bwd.restype = ctypes.c_int32
        lib.tt_tree_weighted_logprob_bwd.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, _vp, ctypes.c_int64,
                                                     _vp, _vp, _vp, ctypes.c_float, _vp, ctypes.c_int64, _vp]
        lib.tt_tree_weighted_logprob_fwd_bwd.restype = ctypes.c_int32
        lib.tt_tree_weighted_logprob_fwd_bwd.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, _vp, ctypes.c_int64,
                                                         _vp, _vp, ctypes.c_float, _vp, _vp, _vp, _vp, ctypes.c_int64, _vp]
        lib.tt_tree_rope.restype = ctypes.c_int32
        lib.tt_tree_rope.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _vp, ctypes.c_int64,
                                     _vp, ctypes.c_float, ctypes.c_int32, _vp, ctypes.c_int64, _vp]
        lib.tt_tree_conv_fwd.restype = ctypes.c_int32
        lib.tt_tree_conv_fwd.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _vp,
                                         ctypes.c_int64, _vp, _vp, _vp, _vp, ctypes.c_int64, _vp]
        lib.tt_tree_conv_plan_sizes.restype = ctypes.c_int32
        lib.tt_tree_conv_plan_sizes.argtypes = [ctypes.c_int64, _vp, ctypes.c_int32, _c_i32p, _c_i32p]
        lib.tt_tree_conv_plan.restype = ctypes.c_int32
        lib.tt_tree_conv_plan.argtypes = [ctypes.c_int64, _vp, ctypes.c_int32, _vp, _vp, _vp, _vp]
        lib.tt_tree_conv_bwd_workspace.restype = ctypes.c_size_t
        lib.tt_tree_conv_bwd_workspace.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
        lib.tt_tree_conv_bwd.restype = ctypes.c_int32
        lib.tt_tree_conv_bwd.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _vp,
                                         ctypes.c_int64, _vp, _vp, _vp, _vp, ctypes.c_int64, ctypes.c_int32, _vp, _vp, _vp, _vp,
                                         _vp, ctypes.c_int64, _vp, _vp, _vp, ctypes.c_size_t, _vp]
        lib.tt_tree_conv_bwd_static.restype = ctypes.c_int32
        lib.tt_tree_conv_bwd_static.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, _vp,
                                                ctypes.c_int64, _vp, _vp, _vp, _vp, ctypes.c_int64, ctypes.c_int32, _vp, _vp, _vp,
                                                _vp, _vp, ctypes.c_int64, _vp, _vp, _vp]
        lib.tt_tree_gdn_plan_sizes.restype = ctypes.c_int32
        lib.tt_tree_gdn_plan_sizes.argtypes = [ctypes.c_int32, _vp, _vp, _c_i32p, _c_i32p]
        lib.tt_tree_gdn_plan.restype = ctypes.c_int32
        lib.tt_tree_gdn_plan.argtypes = [ctypes.c_int32, _vp, _vp, ctypes.c_int32, _vp, _vp, _vp, _vp, _vp, _vp]
        lib.tt_tree_gdn_workspace.restype = ctypes.c_size_t
        lib.tt_tree_gdn_workspace.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
        lib.tt_tree_gdn_fwd.restype = ctypes.c_int32
        lib.tt_tree_gdn_fwd.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_float,
                                        _vp, _vp, _vp, _vp, _vp, ctypes.c_int32, _vp, _vp, _vp, _vp, ctypes.c_int32, _vp, _vp, _vp, _vp,
                                        _vp, _vp, ctypes.c_size_t, _vp]
        lib.tt_tree_gdn_schedule_sizes.restype = ctypes.c_int32
        lib.tt_tree_gdn_schedule_sizes.argtypes = [ctypes.c_int32, _vp, _vp, ctypes.c_int32, _c_i32p, _c_i32p, _c_i32p]
        lib.tt_tree_gdn_schedule.restype = ctypes.c_int32
        lib.tt_tree_gdn_schedule.argtypes = [ctypes.c_int32, _vp, _vp, ctypes.c_int32, _vp, _vp, _vp, _vp, _vp]
        lib.tt_tree_gdn_bwd_workspace.restype = ctypes.c_size_t
        lib.tt_tree_gdn_bwd_workspace.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
        lib.tt_tree_gdn_bwd_workspace_min.restype = ctypes.c_size_t
        lib.tt_tree_gdn_bwd_workspace_min.argtypes = lib.tt_tree_gdn_bwd_workspace.argtypes
        lib.tt_tree_gdn_bwd.restype = ctypes.c_int32
        lib.tt_tree_gdn_bwd.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_float,
                                        _vp, _vp, _vp, _vp, _vp, _vp, ctypes.c_int32, _vp, _vp, _vp, _vp, ctypes.c_int32, _vp, _vp, _vp, _vp,
                                        _vp, _vp, _vp, _vp, _vp, _vp, _vp, ctypes.c_size_t, _vp]
        lib.tt_tree_path_weights.restype = ctypes.c_int32
        lib.tt_tree_path_weights.argtypes = [ctypes.c_int32, _vp, _vp, _vp, ctypes.c_int32, _vp, _vp, _vp, _vp]
        lib.tt_tree_partition_sizes.restype = ctypes.c_int32
        lib.tt_tree_partition_sizes.argtypes = [ctypes.c_int32, _vp, _vp, ctypes.c_int32, ctypes.POINTER(_PartitionSizes)]
        lib.tt_tree_partition_plan.restype = ctypes.c_int32
        lib.tt_tree_partition_plan.argtypes = [ctypes.c_int32, _vp, _vp, ctypes.c_int32] + [_vp] * 17
        lib.tt_tree_attn_partitioned_workspace.restype = ctypes.c_size_t
        lib.tt_tree_attn_partitioned_workspace.argtypes = [ctypes.POINTER(_AttnDesc), ctypes.POINTER(_PartitionPlan), ctypes.c_int32]
        lib.tt_tree_attn_partitioned_fwd.restype = ctypes.c_int32
        lib.tt_tree_attn_partitioned_fwd.argtypes = [ctypes.POINTER(_AttnDesc), ctypes.POINTER(_PartitionPlan)] + [_vp] * 5 + [_vp, ctypes.c_size_t, _vp]
        lib.tt_tree_attn_partitioned_bwd.restype = ctypes.c_int32
        lib.tt_tree_attn_partitioned_bwd.argtypes = [ctypes.POINTER(_AttnDesc), ctypes.POINTER(_PartitionPlan)] + [_vp] * 9 + [_vp, ctypes.c_size_t, _vp]
        lib.tt_kernel_timing_enable.restype = ctypes.c_int32
        lib.tt_kernel_timing_enable.argtypes = [ctypes.c_int32]
        lib.tt_kernel_timing_read.restype = ctypes.c_int32
        lib.tt_kernel_timing_read.argtypes = [ctypes.POINTER(_KernelTimes)]
        _LIB = lib
    return _LIB


KERNEL_NAMES = ("attn_fwd", "loss_fused", "attn_dkdv", "attn_dq", "loss_rows", "loss_sum", "ref_fwd", "ref_bwd",
                "attn_plan", "attn_reduce", "loss_bwd", "rope", "part_gather", "part_scatter", "conv_fwd", "conv_bwd", "conv_fix", "gdn_prepare", "gdn_scan",
                "gdn_bwd_fscan", "gdn_bwd_rscan", "gdn_bwd_finish")


class _KernelTimes(ctypes.Structure):
    _fields_ = [("ms", ctypes.c_double * len(KERNEL_NAMES)), ("launches", ctypes.c_int64 * len(KERNEL_NAMES))]


def kernel_timing_enable(on: bool) -> None:
    """Bracket every kernel launch with HIP events on its stream (resets the totals)."""
    _check(_lib().tt_kernel_timing_enable(1 if on else 0))


def kernel_timing_read() -> dict:
    """Blocks until the recorded events completed; {kernel: (total_ms, launches)} since enable."""
    out = _KernelTimes()
    _check(_lib().tt_kernel_timing_read(ctypes.byref(out)))
    return {n: (float(out.ms[i]), int(out.launches[i])) for i, n in enumerate(KERNEL_NAMES)}


def last_error() -> str:
    return _lib().tt_last_error().decode()


def version() -> int:
    return int(_lib().tt_version())


def _check(status: int) -> None:
    if status != 0:
        raise TreeTrainError(status, last_error())


def _np(a, dtype):
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def _hp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_vp)


@dataclass
class TreeMeta:
    n_nodes: int
    n_tokens: int
    n_leaves: int
    n_roots: int
    n_prefix: int
    n_ktiles: int
    dfs_order: np.ndarray
    node_start: np.ndarray
    node_end: np.ndarray
    subtree_end: np.ndarray
    node_parent: np.ndarray
    node_g: np.ndarray
    tok_node: np.ndarray
    tok_pos: np.ndarray
    tok_pred: np.ndarray
    tok_weight: np.ndarray
    kend: np.ndarray
    ktile_kend_min: np.ndarray
    ktile_kend_max: np.ndarray


def tree_meta_sizes(parent, seg_len, n_prefix: int = 0) -> dict:
    parent, seg_len = _np(parent, np.int32), _np(seg_len, np.int32)
    out = _MetaSizes()
    _check(_lib().tt_tree_meta_sizes(len(parent), _hp(parent), _hp(seg_len), n_prefix, ctypes.byref(out)))
    return {k: getattr(out, k) for k, _ in _MetaSizes._fields_}


def tree_build_meta(parent, seg_len, trained=None, root_pos_offset=None, g_override=None,
                    K_override: int = 0, n_prefix: int = 0, prefix_visible=None) -> TreeMeta:
    parent, seg_len = _np(parent, np.int32), _np(seg_len, np.int32)
    if parent.shape != seg_len.shape or parent.ndim != 1:
        raise ValueError("parent and seg_len must be 1-D arrays of equal length")
    trained = _np(trained, np.uint8)
    root_pos_offset = _np(root_pos_offset, np.int32)
    g_override = _np(g_override, np.int32)
    prefix_visible = _np(prefix_visible, np.uint8)
    for name, arr, n in (("trained", trained, len(parent)), ("g_override", g_override, len(parent)),
                         ("prefix_visible", prefix_visible, n_prefix)):
        if arr is not None and arr.shape != (n,):
            raise ValueError(f"{name} must have shape ({n},)")
    sz = tree_meta_sizes(parent, seg_len, n_prefix)
    if root_pos_offset is not None and root_pos_offset.shape != (sz["n_roots"],):
        raise ValueError(f"root_pos_offset must have one entry per root ({sz['n_roots']})")
    nn, nt, nk = sz["n_nodes"], sz["n_tokens"], sz["n_ktiles"]
    i32 = lambda n: np.zeros(n, dtype=np.int32)
    m = TreeMeta(nn, nt, sz["n_leaves"], sz["n_roots"], n_prefix, nk,
                 i32(nn), i32(nn), i32(nn), i32(nn), i32(nn), i32(nn), i32(nt), i32(nt), i32(nt),
                 np.zeros(nt, dtype=np.float32), i32(n_prefix + nt), i32(nk), i32(nk))
    _check(_lib().tt_tree_build_meta(
        nn, _hp(parent), _hp(seg_len), _hp(trained), _hp(root_pos_offset), _hp(g_override), K_override,
        n_prefix, _hp(prefix_visible),
        _hp(m.dfs_order), _hp(m.node_start), _hp(m.node_end), _hp(m.subtree_end), _hp(m.node_parent),
        _hp(m.node_g), _hp(m.tok_node), _hp(m.tok_pos), _hp(m.tok_pred), _hp(m.tok_weight),
        _hp(m.kend), _hp(m.ktile_kend_min), _hp(m.ktile_kend_max)))
    return m


WEIGHT_PATH_SUM, WEIGHT_UNIFORM, WEIGHT_PATH_TOKEN_MEAN = 0, 1, 2


@dataclass
class ConvPlan:
    """Host output of tt_tree_conv_plan: tokens with successors that do not directly follow them."""
    kernel_size: int
    fix_tok: np.ndarray
    fix_off: np.ndarray
    fix_t: np.ndarray
    fix_r: np.ndarray
    device: Optional[dict] = None

    def to_device(self, device="cuda"):
        torch = _torch()
        self.device = {n: torch.from_numpy(getattr(self, n)).to(device) for n in ("fix_tok", "fix_off", "fix_t", "fix_r")}
        return self


GDN_CHUNK = 64


class _GdnSchedule(ctypes.Structure):
    _fields_ = [("n_segments", ctypes.c_int32), ("n_levels", ctypes.c_int32), ("level_off", ctypes.c_void_p),
                ("seg_chunk0", ctypes.c_void_p), ("seg_chunk1", ctypes.c_void_p), ("slot_cons_off", ctypes.c_void_p),
                ("slot_cons", ctypes.c_void_p)]


def _sched_ref(plan):
    sc = plan._schedule()
    return None if sc is None else ctypes.byref(sc)


@dataclass
class GdnPlan:
    """Host output of tt_tree_gdn_plan: the chunk program of the gated-delta-rule scan."""
    n_chunks: int
    n_slots: int
    chunk_tok0: np.ndarray
    chunk_len: np.ndarray
    chunk_src: np.ndarray
    chunk_dst: np.ndarray
    chunk_cap: np.ndarray
    n_capture: int = 0
    device: Optional[dict] = None
    # tt_tree_gdn_schedule: segments of the chunk program by dependency level (sibling subtrees side by side)
    seg_chunk0: Optional[np.ndarray] = None
    seg_chunk1: Optional[np.ndarray] = None
    level_off: Optional[np.ndarray] = None
    slot_cons_off: Optional[np.ndarray] = None
    slot_cons: Optional[np.ndarray] = None
    parallel: bool = True          # False: the device calls walk all chunks in sequence order (for cross-checks)

    @property
    def n_segments(self) -> int:
        return 0 if self.seg_chunk0 is None else len(self.seg_chunk0)

    @property
    def n_levels(self) -> int:
        return 0 if self.level_off is None else len(self.level_off) - 1

    def to_device(self, device="cuda"):
        torch = _torch()
        names = ["chunk_tok0", "chunk_len", "chunk_src", "chunk_dst", "chunk_cap"]
        if self.seg_chunk0 is not None:
            names += ["seg_chunk0", "seg_chunk1", "slot_cons_off", "slot_cons"]
        self.device = {n: torch.from_numpy(getattr(self, n)).to(device) for n in names}
        return self

    def _schedule(self):
        """ctypes tt_gdn_schedule for the device calls, or None (sequential walk)."""
        if not self.parallel or self.seg_chunk0 is None or self.device is None or "seg_chunk0" not in self.device:
            return None
        d = self.device
        return _GdnSchedule(self.n_segments, self.n_levels, _hp(self.level_off), ctypes.c_void_p(d["seg_chunk0"].data_ptr()),
                            ctypes.c_void_p(d["seg_chunk1"].data_ptr()), ctypes.c_void_p(d["slot_cons_off"].data_ptr()),
                            ctypes.c_void_p(d["slot_cons"].data_ptr()) if len(self.slot_cons) else None)


def tree_gdn_plan(parent, seg_len, capture_nodes=()) -> GdnPlan:
    parent, seg_len = _np(parent, np.int32), _np(seg_len, np.int32)
    if len(parent) != len(seg_len):
        raise ValueError("parent and seg_len differ in length")
    nc, ns = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(_lib().tt_tree_gdn_plan_sizes(len(parent), _hp(parent), _hp(seg_len), ctypes.byref(nc), ctypes.byref(ns)))
    arrs = [np.zeros(nc.value, np.int32) for _ in range(5)]
    cap = _np(list(capture_nodes), np.int32)
    _check(_lib().tt_tree_gdn_plan(len(parent), _hp(parent), _hp(seg_len), len(cap), _hp(cap), *(_hp(a) for a in arrs)))
    plan = GdnPlan(nc.value, ns.value, *arrs, n_capture=len(cap))
    nseg, nlev, ncons = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int32(0)
    _check(_lib().tt_tree_gdn_schedule_sizes(plan.n_chunks, _hp(plan.chunk_src), _hp(plan.chunk_dst), plan.n_slots,
                                             ctypes.byref(nseg), ctypes.byref(nlev), ctypes.byref(ncons)))
    plan.seg_chunk0, plan.seg_chunk1 = np.zeros(nseg.value, np.int32), np.zeros(nseg.value, np.int32)
    plan.level_off = np.zeros(nlev.value + 1, np.int32)
    plan.slot_cons_off, plan.slot_cons = np.zeros(plan.n_slots + 1, np.int32), np.zeros(ncons.value, np.int32)
    _check(_lib().tt_tree_gdn_schedule(plan.n_chunks, _hp(plan.chunk_src), _hp(plan.chunk_dst), plan.n_slots, _hp(plan.seg_chunk0),
                                       _hp(plan.seg_chunk1), _hp(plan.level_off), _hp(plan.slot_cons_off), _hp(plan.slot_cons)))
    return plan


def tree_conv_plan(tok_pred, kernel_size: int) -> ConvPlan:
    tok_pred = _np(tok_pred, np.int32)
    nf, npairs = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(_lib().tt_tree_conv_plan_sizes(len(tok_pred), _hp(tok_pred), int(kernel_size), ctypes.byref(nf), ctypes.byref(npairs)))
    fix_tok, fix_off = np.zeros(nf.value, np.int32), np.zeros(nf.value + 1, np.int32)
    fix_t, fix_r = np.zeros(npairs.value, np.int32), np.zeros(npairs.value, np.int32)
    _check(_lib().tt_tree_conv_plan(len(tok_pred), _hp(tok_pred), int(kernel_size), _hp(fix_tok), _hp(fix_off), _hp(fix_t), _hp(fix_r)))
    return ConvPlan(int(kernel_size), fix_tok, fix_off, fix_t, fix_r)


def tree_path_weights(parent, seg_len, trained=None, *, scheme: int = WEIGHT_PATH_SUM, path_weight=None, advantage=None):
    """General loss weights lambda_t = sum of path weights over the paths through t (host).
    Returns (tok_weight [n_tokens] fp32, leaf_node [n_leaves] int32: the leaf of path k)."""
    parent, seg_len = _np(parent, np.int32), _np(seg_len, np.int32)
    if len(parent) != len(seg_len):
        raise ValueError("parent and seg_len differ in length")
    trained = _np(trained, np.uint8)
    sz = tree_meta_sizes(parent, seg_len)
    path_weight, advantage = _np(path_weight, np.float32), _np(advantage, np.float32)
    if path_weight is not None and len(path_weight) != sz["n_leaves"]:
        raise ValueError(f"path_weight has {len(path_weight)} entries for {sz['n_leaves']} paths")
    if advantage is not None and len(advantage) != sz["n_tokens"]:
        raise ValueError("advantage must have one entry per token")
    w = np.zeros(sz["n_tokens"], np.float32)
    leaf = np.zeros(sz["n_leaves"], np.int32)
    _check(_lib().tt_tree_path_weights(len(parent), _hp(parent), _hp(seg_len), _hp(trained), int(scheme), _hp(path_weight),
                                       _hp(advantage), _hp(w), _hp(leaf)))
    return w, leaf


@dataclass
class PartitionPlan:
    """Outputs of tt_tree_partition_plan (numpy, host).  `device` holds torch copies of the five arrays the
    device driver reads, once to_device() was called."""
    n_parts: int
    n_tokens: int
    capacity: int
    max_part_tokens: int
    max_prefix: int
    part_of_node: np.ndarray
    part_node_off: np.ndarray
    part_nodes: np.ndarray
    part_parent: np.ndarray
    part_cut_node: np.ndarray
    part_pos_offset: np.ndarray
    part_tok_off: np.ndarray
    own_tok: np.ndarray
    part_prefix_off: np.ndarray
    prefix_tok: np.ndarray
    prefix_visible: np.ndarray
    kend: np.ndarray
    part_ktile_off: np.ndarray
    kt_min: np.ndarray
    kt_max: np.ndarray
    part_own_start: np.ndarray
    part_prefix_start: np.ndarray
    device: Optional[dict] = None
    in_place: bool = True          # False: the driver gathers every partition (for cross-checks)

    def to_device(self, device="cuda"):
        torch = _torch()
        self.device = {name: torch.from_numpy(getattr(self, name)).to(device)
                       for name in ("own_tok", "prefix_tok", "kend", "kt_min", "kt_max")}
        return self

    def _c(self) -> _PartitionPlan:
        if self.device is None:
            raise ValueError("call to_device() on the plan first")
        d = self.device
        return _PartitionPlan(self.n_parts, self.n_tokens, _hp(self.part_tok_off), _hp(self.part_prefix_off),
                              _hp(self.part_ktile_off), _hp(self.part_own_start) if self.in_place else None,
                              _hp(self.part_prefix_start) if self.in_place else None, *(ctypes.c_void_p(d[n].data_ptr()) for n in
                                                         ("own_tok", "prefix_tok", "kend", "kt_min", "kt_max")))


def tree_partition_sizes(parent, seg_len, capacity: int) -> dict:
    parent, seg_len = _np(parent, np.int32), _np(seg_len, np.int32)
    out = _PartitionSizes()
    _check(_lib().tt_tree_partition_sizes(len(parent), _hp(parent), _hp(seg_len), int(capacity), ctypes.byref(out)))
    return {f: int(getattr(out, f)) for f, _ in _PartitionSizes._fields_}


def tree_partition_plan(parent, seg_len, capacity: int) -> PartitionPlan:
    """Cuts the tree into partitions of at most `capacity` tokens and lays out everything the partitioned
    attention calls need (host only)."""
    parent, seg_len = _np(parent, np.int32), _np(seg_len, np.int32)
    if len(parent) != len(seg_len):
        raise ValueError("parent and seg_len differ in length")
    sz = tree_partition_sizes(parent, seg_len, capacity)
    n, npart, ntok = len(parent), sz["n_parts"], sz["n_tokens"]
    arr = dict(
        part_of_node=np.zeros(n, np.int32), part_node_off=np.zeros(npart + 1, np.int32), part_nodes=np.zeros(n, np.int32),
        part_parent=np.zeros(npart, np.int32), part_cut_node=np.zeros(npart, np.int32),
        part_pos_offset=np.zeros(npart, np.int32), part_tok_off=np.zeros(npart + 1, np.int32),
        own_tok=np.zeros(ntok, np.int32), part_prefix_off=np.zeros(npart + 1, np.int64),
        prefix_tok=np.zeros(sz["sum_prefix"], np.int32), prefix_visible=np.zeros(sz["sum_prefix"], np.uint8),
        kend=np.zeros(sz["sum_prefix"] + ntok, np.int32), part_ktile_off=np.zeros(npart + 1, np.int64),
        kt_min=np.zeros(sz["sum_ktiles"], np.int32), kt_max=np.zeros(sz["sum_ktiles"], np.int32),
        part_own_start=np.zeros(npart, np.int32), part_prefix_start=np.zeros(npart, np.int32))
    _check(_lib().tt_tree_partition_plan(n, _hp(parent), _hp(seg_len), int(capacity), *(_hp(a) for a in arr.values())))
    return PartitionPlan(n_parts=npart, n_tokens=ntok, capacity=int(capacity), max_part_tokens=sz["max_part_tokens"],
                         max_prefix=sz["max_prefix"], **arr)


# ---- device calls -----------------------------------------------------------------------------

def _torch():
    import torch
    return torch


def _dp(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _desc(q, k, v, n_prefix: int, scale, reference_kernels: bool) -> _AttnDesc:
    torch = _torch()
    if q.dim() != 3 or k.dim() != 3 or v.dim() != 3:
        raise ValueError("q, k, v must be [tokens, heads, d]")
    if q.dtype not in (torch.bfloat16, torch.float32) or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v must share dtype bf16 or fp32")
    for t in (q, k, v):
        if t.numel() > 0 and (t.stride(2) != 1 or t.stride(1) != t.shape[2]):
            raise ValueError("heads and d must be contiguous (only the token stride is free)")
    n_q, hq, d = q.shape
    if k.shape[0] != n_q or v.shape != k.shape or k.shape[2] != d:
        raise ValueError("k, v must be [n_q, hkv, d]")
    return _AttnDesc(n_q, n_prefix, hq, k.shape[1], d,
                     DTYPE_BF16 if q.dtype == torch.bfloat16 else DTYPE_FP32,
                     float(d) ** -0.5 if scale is None else float(scale),
                     FLAG_REFERENCE_KERNELS if reference_kernels else 0,
                     *(t.stride(0) if t.shape[0] > 1 else t.shape[1] * t.shape[2] for t in (q, k, v)))


def tree_attn_workspace(q, k, v, n_prefix: int = 0, backward: bool = False, scale=None,
                        reference_kernels: bool = False) -> int:
    d = _desc(q, k, v, n_prefix, scale, reference_kernels)
    return int(_lib().tt_tree_attn_workspace(ctypes.byref(d), 1 if backward else 0))


def _workspace(desc, backward, workspace, device):
    torch = _torch()
    need = int(_lib().tt_tree_attn_workspace(ctypes.byref(desc), 1 if backward else 0))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return workspace, workspace.numel() * workspace.element_size()


def tree_attn_fwd(q, k, v, kend, kt_min, kt_max, *, k_prefix=None, v_prefix=None, scale=None,
                  o=None, lse=None, workspace=None, stream=None, reference_kernels: bool = False):
    """q [N,hq,d]; k, v [N,hkv,d]; kend/kt_min/kt_max: int32 device tensors from tree_build_meta.
    Returns (o [N,hq,d], lse [hq,N] fp32)."""
    torch = _torch()
    n_prefix = 0 if k_prefix is None else k_prefix.shape[0]
    desc = _desc(q, k, v, n_prefix, scale, reference_kernels)
    if k_prefix is not None:
        k_prefix, v_prefix = k_prefix.contiguous(), v_prefix.contiguous()
    if o is None:
        o = torch.empty((desc.n_q, desc.hq, desc.d), dtype=q.dtype, device=q.device)
    if lse is None:
        lse = torch.empty((desc.hq, desc.n_q), dtype=torch.float32, device=q.device)
    workspace, ws_bytes = _workspace(desc, False, workspace, q.device)
    _check(_lib().tt_tree_attn_fwd(ctypes.byref(desc), _dp(q), _dp(k), _dp(v), _dp(k_prefix), _dp(v_prefix),
                                   _dp(kend), _dp(kt_min), _dp(kt_max), _dp(o), _dp(lse),
                                   _dp(workspace), ws_bytes, _stream_ptr(stream)))
    return o, lse


def tree_attn_bwd(q, k, v, kend, kt_min, kt_max, o, d_o, lse, *, k_prefix=None, v_prefix=None,
                  dk_prefix_acc=None, dv_prefix_acc=None, scale=None, dq=None, dk=None, dv=None,
                  workspace=None, stream=None, reference_kernels: bool = False):
    """Returns (dq [N,hq,d], dk [N,hkv,d], dv [N,hkv,d]); prefix gradients are added into the fp32
    accumulators dk_prefix_acc / dv_prefix_acc [P,hkv,d]."""
    torch = _torch()
    n_prefix = 0 if k_prefix is None else k_prefix.shape[0]
    desc = _desc(q, k, v, n_prefix, scale, reference_kernels)
    if k_prefix is not None:
        k_prefix, v_prefix = k_prefix.contiguous(), v_prefix.contiguous()
    if not (o.is_contiguous() and d_o.is_contiguous() and lse.is_contiguous()):
        raise ValueError("o, d_o, lse must be contiguous")
    if dq is None:
        dq = torch.empty((desc.n_q, desc.hq, desc.d), dtype=q.dtype, device=q.device)
    if dk is None:
        dk = torch.empty((desc.n_q, desc.hkv, desc.d), dtype=q.dtype, device=q.device)
    if dv is None:
        dv = torch.empty((desc.n_q, desc.hkv, desc.d), dtype=q.dtype, device=q.device)
    workspace, ws_bytes = _workspace(desc, True, workspace, q.device)
    _check(_lib().tt_tree_attn_bwd(ctypes.byref(desc), _dp(q), _dp(k), _dp(v), _dp(k_prefix), _dp(v_prefix),
                                   _dp(kend), _dp(kt_min), _dp(kt_max), _dp(o), _dp(d_o), _dp(lse),
                                   _dp(dq), _dp(dk), _dp(dv), _dp(dk_prefix_acc), _dp(dv_prefix_acc),
                                   _dp(workspace), ws_bytes, _stream_ptr(stream)))
    return dq, dk, dv


def tree_weighted_logprob(logits, target, weight=None, *, loss_acc=None, logp=None, lse=None,
                          want_lse: bool = True, stream=None):
    """logits [n, V] bf16/fp32 (row stride free), target [n] int32, weight [n] fp32 or None.
    Returns (logp [n], lse [n] or None, loss_acc [1]); loss_acc is added to (zeroed if created here)."""
    torch = _torch()
    if logits.dim() != 2 or logits.stride(1) != 1:
        raise ValueError("logits must be [rows, vocab] with contiguous vocab")
    if logits.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("logits must be bf16 or fp32")
    n, vocab = logits.shape
    if logp is None:
        logp = torch.empty(n, dtype=torch.float32, device=logits.device)
    if lse is None and want_lse:
        lse = torch.empty(n, dtype=torch.float32, device=logits.device)
    if loss_acc is None:
        loss_acc = torch.zeros(1, dtype=torch.float32, device=logits.device)
    _check(_lib().tt_tree_weighted_logprob(
        n, vocab, DTYPE_BF16 if logits.dtype == torch.bfloat16 else DTYPE_FP32, _dp(logits),
        logits.stride(0) if n > 1 else vocab, _dp(target), _dp(weight), _dp(logp), _dp(lse), _dp(loss_acc),
        _stream_ptr(stream)))
    return logp, lse, loss_acc


def tree_rope(x, tok_pos, *, theta_base: float = 1.0e6, inverse: bool = False, out=None, stream=None):
    """Rotary embedding of x [n, heads, d] (bf16/fp32, heads and d contiguous, free token stride) with the
    tree position ids tok_pos [n] int32; `inverse` undoes it / is its backward.  `out` may be x (in place)."""
    torch = _torch()
    if x.dim() != 3 or x.stride(2) != 1 or (x.shape[1] > 1 and x.stride(1) != x.shape[2]):
        raise ValueError("x must be [tokens, heads, d] with heads and d contiguous")
    if x.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("x must be bf16 or fp32")
    n, h, d = x.shape
    if out is None:
        out = torch.empty((n, h, d), dtype=x.dtype, device=x.device)
    if out.shape != x.shape or out.dtype != x.dtype or out.stride(2) != 1 or (h > 1 and out.stride(1) != d):
        raise ValueError("out must match x in shape and dtype, heads and d contiguous")
    _check(_lib().tt_tree_rope(n, h, d, DTYPE_BF16 if x.dtype == torch.bfloat16 else DTYPE_FP32, _dp(x),
                               x.stride(0) if n > 1 else h * d, _dp(tok_pos), float(theta_base), 1 if inverse else 0,
                               _dp(out), out.stride(0) if n > 1 else h * d, _stream_ptr(stream)))
    return out


def tree_weighted_logprob_bwd(logits, target, weight, lse, *, grad_scale: float = 1.0, out=None, stream=None):
    """dlogits = grad_scale * weight * (softmax(logits) - onehot(target)), same dtype and shape as logits
    (zero rows where target < 0); lse [n] fp32 is the one tree_weighted_logprob returned.  `out` may be
    the logits tensor itself (in place)."""
    torch = _torch()
    if logits.dim() != 2 or logits.stride(1) != 1:
        raise ValueError("logits must be [rows, vocab] with contiguous vocab")
    if logits.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("logits must be bf16 or fp32")
    n, vocab = logits.shape
    if out is None:
        out = torch.empty((n, vocab), dtype=logits.dtype, device=logits.device)
    if out.shape != logits.shape or out.dtype != logits.dtype or out.stride(1) != 1:
        raise ValueError("out must match logits in shape and dtype, with contiguous vocab")
    _check(_lib().tt_tree_weighted_logprob_bwd(
        n, vocab, DTYPE_BF16 if logits.dtype == torch.bfloat16 else DTYPE_FP32, _dp(logits),
        logits.stride(0) if n > 1 else vocab, _dp(target), _dp(weight), _dp(lse), float(grad_scale), _dp(out),
        out.stride(0) if n > 1 else vocab, _stream_ptr(stream)))
    return out


def tree_weighted_logprob_fwd_bwd(logits, target, weight=None, *, grad_scale: float = 1.0, loss_acc=None, logp=None,
                                  lse=None, out=None, stream=None):
    """tree_weighted_logprob and tree_weighted_logprob_bwd in one pass over the logits.  Returns (logp [n], lse [n],
    loss_acc [1] (added to; zeroed if created here), dlogits like logits); `out` may be the logits tensor itself."""
    torch = _torch()
    if logits.dim() != 2 or logits.stride(1) != 1:
        raise ValueError("logits must be [rows, vocab] with contiguous vocab")
    if logits.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("logits must be bf16 or fp32")
    n, vocab = logits.shape
    dev = logits.device
    if logp is None:
        logp = torch.empty(n, dtype=torch.float32, device=dev)
    if lse is None:
        lse = torch.empty(n, dtype=torch.float32, device=dev)
    if loss_acc is None:
        loss_acc = torch.zeros(1, dtype=torch.float32, device=dev)
    if out is None:
        out = torch.empty((n, vocab), dtype=logits.dtype, device=dev)
    if out.shape != logits.shape or out.dtype != logits.dtype or out.stride(1) != 1:
        raise ValueError("out must match logits in shape and dtype, with contiguous vocab")
    _check(_lib().tt_tree_weighted_logprob_fwd_bwd(
        n, vocab, DTYPE_BF16 if logits.dtype == torch.bfloat16 else DTYPE_FP32, _dp(logits),
        logits.stride(0) if n > 1 else vocab, _dp(target), _dp(weight), float(grad_scale), _dp(logp), _dp(lse), _dp(loss_acc),
        _dp(out), out.stride(0) if n > 1 else vocab, _stream_ptr(stream)))
    return logp, lse, loss_acc, out


def tree_attn_partitioned_workspace(q, k, v, plan: PartitionPlan, backward: bool = False, scale=None,
                                    reference_kernels: bool = False) -> int:
    d = _desc(q, k, v, 0, scale, reference_kernels)
    c = plan._c()
    return int(_lib().tt_tree_attn_partitioned_workspace(ctypes.byref(d), ctypes.byref(c), 1 if backward else 0))


def _part_workspace(desc, cplan, backward, workspace, device):
    torch = _torch()
    need = int(_lib().tt_tree_attn_partitioned_workspace(ctypes.byref(desc), ctypes.byref(cplan), 1 if backward else 0))
    if need == 0:
        raise TreeTrainError(-2, last_error())
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
    return workspace, workspace.numel() * workspace.element_size()


def tree_attn_partitioned_fwd(q, k, v, plan: PartitionPlan, *, scale=None, o=None, lse=None, workspace=None,
                              stream=None, reference_kernels: bool = False):
    """Whole-tree q [N,hq,d], k, v [N,hkv,d] in whole-tree DFS order; one attention pass per partition of
    `plan`.  Returns (o [N,hq,d], lse [hq,N])."""
    torch = _torch()
    desc = _desc(q, k, v, 0, scale, reference_kernels)
    cplan = plan._c()
    if o is None:
        o = torch.empty((desc.n_q, desc.hq, desc.d), dtype=q.dtype, device=q.device)
    if lse is None:
        lse = torch.empty((desc.hq, desc.n_q), dtype=torch.float32, device=q.device)
    workspace, ws_bytes = _part_workspace(desc, cplan, False, workspace, q.device)
    _check(_lib().tt_tree_attn_partitioned_fwd(ctypes.byref(desc), ctypes.byref(cplan), _dp(q), _dp(k), _dp(v),
                                               _dp(o), _dp(lse), _dp(workspace), ws_bytes, _stream_ptr(stream)))
    return o, lse


def tree_attn_partitioned_bwd(q, k, v, plan: PartitionPlan, o, d_o, lse, *, scale=None, dq=None, dk=None, dv=None,
                              workspace=None, stream=None, reference_kernels: bool = False):
    """Returns whole-tree (dq, dk, dv); cached-key gradients of all partitions are summed in fp32 inside."""
    torch = _torch()
    desc = _desc(q, k, v, 0, scale, reference_kernels)
    cplan = plan._c()
    if not (o.is_contiguous() and d_o.is_contiguous() and lse.is_contiguous()):
        raise ValueError("o, d_o, lse must be contiguous")
    if dq is None:
        dq = torch.empty((desc.n_q, desc.hq, desc.d), dtype=q.dtype, device=q.device)
    if dk is None:
        dk = torch.empty((desc.n_q, desc.hkv, desc.d), dtype=q.dtype, device=q.device)
    if dv is None:
        dv = torch.empty((desc.n_q, desc.hkv, desc.d), dtype=q.dtype, device=q.device)
    workspace, ws_bytes = _part_workspace(desc, cplan, True, workspace, q.device)
    _check(_lib().tt_tree_attn_partitioned_bwd(ctypes.byref(desc), ctypes.byref(cplan), _dp(q), _dp(k), _dp(v),
                                               _dp(o), _dp(d_o), _dp(lse), _dp(dq), _dp(dk), _dp(dv),
                                               _dp(workspace), ws_bytes, _stream_ptr(stream)))
    return dq, dk, dv


def _conv_check(x, weight, what="x"):
    torch = _torch()
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError(f"{what} must be [tokens, channels] with contiguous channels")
    if x.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError(f"{what} must be bf16 or fp32")
    if weight.dim() != 2 or weight.shape[0] != x.shape[1] or weight.dtype != torch.float32 or not weight.is_contiguous():
        raise ValueError("weight must be a contiguous fp32 [channels, K] tensor")
    return x.shape[0], x.shape[1], weight.shape[1], DTYPE_BF16 if x.dtype == torch.bfloat16 else DTYPE_FP32


def _row_stride(t):
    return t.stride(0) if t.shape[0] > 1 else t.shape[1]


def tree_conv_fwd(x, weight, bias, tok_pred, *, silu: bool = True, out=None, stream=None):
    """Tree-correct depthwise causal conv: x [n, C] bf16/fp32, weight [C, K] fp32, bias [C] fp32 or None,
    tok_pred [n] int32 (from tree_build_meta).  Returns y [n, C]."""
    torch = _torch()
    n, c, k, dt = _conv_check(x, weight)
    if out is None:
        out = torch.empty((n, c), dtype=x.dtype, device=x.device)
    _check(_lib().tt_tree_conv_fwd(n, c, k, dt, 1 if silu else 0, _dp(x), _row_stride(x), _dp(weight), _dp(bias), _dp(tok_pred),
                                   _dp(out), _row_stride(out), _stream_ptr(stream)))
    return out


def tree_conv_bwd(x, weight, bias, tok_pred, dy, plan: ConvPlan, *, silu: bool = True, want_dbias: bool = True,
                  workspace=None, stream=None):
    """Returns (dx [n, C] in x's dtype, dweight [C, K] fp32, dbias [C] fp32 or None)."""
    torch = _torch()
    n, c, k, dt = _conv_check(x, weight)
    _conv_check(dy, weight, "dy")
    if plan.kernel_size != k:
        raise ValueError(f"the plan was made for kernel size {plan.kernel_size}, weight has {k}")
    if plan.device is None:
        plan.to_device(x.device)
    dx = torch.empty((n, c), dtype=x.dtype, device=x.device)
    dw = torch.empty((c, k), dtype=torch.float32, device=x.device)
    db = torch.empty(c, dtype=torch.float32, device=x.device) if want_dbias else None
    need = int(_lib().tt_tree_conv_bwd_workspace(n, c, k, dt))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    d = plan.device
    _check(_lib().tt_tree_conv_bwd(n, c, k, dt, 1 if silu else 0, _dp(x), _row_stride(x), _dp(weight), _dp(bias), _dp(tok_pred),
                                   _dp(dy), _row_stride(dy), len(plan.fix_tok), _dp(d["fix_tok"]), _dp(d["fix_off"]),
                                   _dp(d["fix_t"]), _dp(d["fix_r"]), _dp(dx), _row_stride(dx), _dp(dw), _dp(db),
                                   _dp(workspace), workspace.numel(), _stream_ptr(stream)))
    return dx, dw, db


CONV_BWD_STATIC_SCRATCH_BYTES = 64 << 20


def tree_conv_bwd_static(x, weight, bias, tok_pred, dy, plan: ConvPlan, dx, dweight, dbias=None, *, silu: bool = True,
                         stream=None) -> None:
    """tree_conv_bwd for callers that may not allocate: every output is passed in (dx [n, C] in x's dtype,
    dweight [C, K] fp32, dbias [C] fp32 or None), the plan must already be on the device, and the scratch is the
    library's static array (shapes whose scratch exceeds CONV_BWD_STATIC_SCRATCH_BYTES are refused)."""
    n, c, k, dt = _conv_check(x, weight)
    _conv_check(dy, weight, "dy")
    if plan.kernel_size != k:
        raise ValueError(f"the plan was made for kernel size {plan.kernel_size}, weight has {k}")
    if plan.device is None:
        raise ValueError("move the plan to the device first (plan.to_device): this call does not allocate")
    if dx.shape != x.shape or dx.dtype != x.dtype or dweight.shape != weight.shape:
        raise ValueError("dx must match x, dweight must match weight")
    d = plan.device
    _check(_lib().tt_tree_conv_bwd_static(n, c, k, dt, 1 if silu else 0, _dp(x), _row_stride(x), _dp(weight), _dp(bias),
                                          _dp(tok_pred), _dp(dy), _row_stride(dy), len(plan.fix_tok), _dp(d["fix_tok"]),
                                          _dp(d["fix_off"]), _dp(d["fix_t"]), _dp(d["fix_r"]), _dp(dx), _row_stride(dx),
                                          _dp(dweight), _dp(dbias), _stream_ptr(stream)))


def tree_gdn_fwd(q, k, v, g, beta, plan: GdnPlan, *, scale=None, out=None, workspace=None, stream=None,
                 initial_state=None, return_states: bool = False):
    """Gated delta rule with tree state routing: q, k [n, hk, 128], v [n, hv, 128] bf16 contiguous; g, beta
    [n, hv] fp32 (g = log decay <= 0).  Returns o [n, hv, 128] bf16; with return_states also the end states
    [n_capture, hv, 128, 128] fp32 of the plan's capture nodes.  initial_state [hv, 128, 128] fp32: the state
    every root starts from."""
    torch = _torch()
    for t in (q, k, v):
        if t.dim() != 3 or t.dtype != torch.bfloat16 or not t.is_contiguous():
            raise ValueError("q, k, v must be contiguous bf16 [tokens, heads, dim]")
    n, hk, dk = q.shape
    hv, dv = v.shape[1], v.shape[2]
    if k.shape != q.shape or v.shape[0] != n:
        raise ValueError("k must match q, v must have the same token count")
    for t in (g, beta):
        if t.shape != (n, hv) or t.dtype != torch.float32 or not t.is_contiguous():
            raise ValueError("g, beta must be contiguous fp32 [tokens, hv]")
    if plan.device is None:
        plan.to_device(q.device)
    if out is None:
        out = torch.empty((n, hv, dv), dtype=torch.bfloat16, device=q.device)
    need = int(_lib().tt_tree_gdn_workspace(plan.n_chunks, plan.n_slots, hv))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    d = plan.device
    states = None
    if return_states:
        states = torch.empty((plan.n_capture, hv, dk, dv), dtype=torch.float32, device=q.device)
    if initial_state is not None and (initial_state.shape != (hv, dk, dv) or initial_state.dtype != torch.float32
                                      or not initial_state.is_contiguous()):
        raise ValueError("initial_state must be a contiguous fp32 [hv, dk, dv] tensor")
    _check(_lib().tt_tree_gdn_fwd(n, hk, hv, dk, dv, float(dk) ** -0.5 if scale is None else float(scale), _dp(q), _dp(k), _dp(v),
                                  _dp(g), _dp(beta), plan.n_chunks, _dp(d["chunk_tok0"]), _dp(d["chunk_len"]), _dp(d["chunk_src"]),
                                  _dp(d["chunk_dst"]), plan.n_slots, _dp(d["chunk_cap"]) if return_states and plan.n_capture else None,
                                  _sched_ref(plan), _dp(initial_state), _dp(states) if plan.n_capture else None, _dp(out), _dp(workspace), workspace.numel(),
                                  _stream_ptr(stream)))
    return (out, states) if return_states else out


def tree_gdn_bwd_workspace(n_tokens: int, hk: int, hv: int, plan: GdnPlan, smallest: bool = False) -> int:
    """Bytes of workspace with which tree_gdn_bwd takes all heads in one pass, or (smallest) the least it accepts:
    one key head with its value heads per pass.  Anything in between is used for as many key heads per pass as fit."""
    f = _lib().tt_tree_gdn_bwd_workspace_min if smallest else _lib().tt_tree_gdn_bwd_workspace
    return int(f(n_tokens, plan.n_chunks, plan.n_slots, plan.n_segments if plan._schedule() is not None else 0, hk, hv))


def tree_gdn_bwd(q, k, v, g, beta, d_o, plan: GdnPlan, *, scale=None, initial_state=None, d_state_out=None,
                 want_d_initial_state: bool = False, workspace=None, stream=None):
    """Backward of tree_gdn_fwd for upstream d_o [n, hv, 128] bf16.  Returns (dq, dk [n, hk, 128] bf16, dv [n, hv, 128]
    bf16, dg, dbeta [n, hv] fp32), plus d_initial_state [hv, 128, 128] fp32 when asked.  d_state_out
    [n_capture, hv, 128, 128] fp32: upstream gradient of the plan's captured end states.  workspace: a uint8 tensor of
    tree_gdn_bwd_workspace(...) bytes (default: allocated here, full size) or of any size down to its `smallest`."""
    torch = _torch()
    for t in (q, k, v, d_o):
        if t.dim() != 3 or t.dtype != torch.bfloat16 or not t.is_contiguous():
            raise ValueError("q, k, v, d_o must be contiguous bf16 [tokens, heads, dim]")
    n, hk, dk = q.shape
    hv, dv = v.shape[1], v.shape[2]
    if k.shape != q.shape or v.shape[0] != n or d_o.shape != v.shape:
        raise ValueError("k must match q, v must have the same token count, d_o must match v")
    for t in (g, beta):
        if t.shape != (n, hv) or t.dtype != torch.float32 or not t.is_contiguous():
            raise ValueError("g, beta must be contiguous fp32 [tokens, hv]")
    for t, shape, name in ((initial_state, (hv, dk, dv), "initial_state"), (d_state_out, (plan.n_capture, hv, dk, dv), "d_state_out")):
        if t is not None and (tuple(t.shape) != shape or t.dtype != torch.float32 or not t.is_contiguous()):
            raise ValueError(f"{name} must be a contiguous fp32 tensor of shape {shape}")
    if plan.device is None:
        plan.to_device(q.device)
    dev = q.device
    dq, dk_ = torch.empty_like(q), torch.empty_like(k)
    dv_ = torch.empty_like(v)
    dg, dbeta = torch.empty_like(g), torch.empty_like(beta)
    d_init = torch.empty((hv, dk, dv), dtype=torch.float32, device=dev) if want_d_initial_state else None
    need = tree_gdn_bwd_workspace(n, hk, hv, plan)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    d = plan.device
    use_cap = d_state_out is not None and plan.n_capture > 0
    _check(_lib().tt_tree_gdn_bwd(n, hk, hv, dk, dv, float(dk) ** -0.5 if scale is None else float(scale), _dp(q), _dp(k), _dp(v),
                                  _dp(g), _dp(beta), _dp(d_o), plan.n_chunks, _dp(d["chunk_tok0"]), _dp(d["chunk_len"]),
                                  _dp(d["chunk_src"]), _dp(d["chunk_dst"]), plan.n_slots, _dp(d["chunk_cap"]) if use_cap else None,
                                  _sched_ref(plan), _dp(initial_state), _dp(d_state_out) if use_cap else None, _dp(dq), _dp(dk_), _dp(dv_), _dp(dg),
                                  _dp(dbeta), _dp(d_init), _dp(workspace), workspace.numel(), _stream_ptr(stream)))
    out = (dq, dk_, dv_, dg, dbeta)
    return out + (d_init,) if want_d_initial_state else out
