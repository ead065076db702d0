"""CPU ORACLE (test infrastructure only) -- attention front ends.

branches():  per-branch recomputation (C, branch_attention.c) -- the authoritative reference:
             the paper's baseline of running all K paths independently (Eq. 1, 5, 6).
rows():      the same per-row arithmetic for a sample of outputs at sizes too big for branches().
dense():     softmax attention under an explicit boolean mask, numpy fp64, for tiny inputs;
             used to tie the per-branch oracle to the paper's mask statements.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

from . import build as _build
from . import meta as _meta

_LIBS: Dict[str, ctypes.CDLL] = {}


def _lib(real: str = "f64") -> ctypes.CDLL:
    if real not in _LIBS:
        path = _build.lib_path(real)
        if not os.path.exists(path):
            _build.build()
        lib = ctypes.CDLL(path)
        lib.oracle_real_bytes.restype = ctypes.c_int
        lib.oracle_max_threads.restype = ctypes.c_int
        assert lib.oracle_real_bytes() == (8 if real == "f64" else 4)
        _LIBS[real] = lib
    return _LIBS[real]


def n_threads() -> int:
    return int(_lib().oracle_max_threads())


def _f32(x) -> np.ndarray:
    """Inputs as contiguous float32 (bf16 inputs must be upcast by the caller: torch .float())."""
    if hasattr(x, "detach"):
        x = x.detach().cpu().float().numpy()
    return np.ascontiguousarray(x, dtype=np.float32)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def branches(meta, q, k, v, d_o=None, scale: Optional[float] = None, kv_heads: Optional[Sequence[int]] = None,
             real: str = "f64"):
    """Run every root-to-leaf branch as an independent causal sequence and scatter-sum.

    Returns dict(o [N,hq,d], lse [hq,N], dq, dk, dv, mismatch).  Only the query heads belonging to
    `kv_heads` (default: all) are filled; others stay zero.
    """
    q, k, v = _f32(q), _f32(k), _f32(v)
    n, hq, d = q.shape
    hkv = k.shape[1]
    assert k.shape == (n, hkv, d) and v.shape == k.shape and n == meta["n_tokens"]
    d_o = None if d_o is None else _f32(d_o)
    scale = float(d) ** -0.5 if scale is None else float(scale)
    dt = np.float64 if real == "f64" else np.float32
    pl = _meta.paths(meta)
    ptr = np.zeros(len(pl) + 1, dtype=np.int64)
    for i, p in enumerate(pl):
        ptr[i + 1] = ptr[i] + len(p)
    idx = np.ascontiguousarray(np.concatenate(pl) if pl else np.zeros(0), dtype=np.int32)
    g_tok = np.ascontiguousarray(meta["node_g"][meta["tok_node"]], dtype=np.int32)
    o = np.zeros((n, hq, d), dtype=dt)
    lse = np.zeros((hq, n), dtype=dt)
    dq = np.zeros((n, hq, d), dtype=dt)
    dk = np.zeros((n, hkv, d), dtype=dt)
    dv = np.zeros((n, hkv, d), dtype=dt)
    mism = ctypes.c_int64(0)
    groups = list(range(hkv)) if kv_heads is None else list(kv_heads)
    lib = _lib(real)
    for kvh in groups:
        rc = lib.oracle_attn_branches(
            ctypes.c_int64(n), hq, hkv, d, ctypes.c_double(scale),
            _p(q), _p(k), _p(v), _p(d_o),
            len(pl), _p(ptr), _p(idx), _p(g_tok), kvh, kvh + 1,
            _p(o), _p(lse), _p(dq), _p(dk), _p(dv), ctypes.byref(mism))
        assert rc == 0, "oracle_attn_branches failed"
        assert mism.value == 0, "forward equivalence (Eq. 6) violated inside the oracle"
    return dict(o=o, lse=lse, dq=dq, dk=dk, dv=dv, mismatch=0, n_paths=len(pl),
                n_lin=int(ptr[-1]))


def rows(meta, q, k, v, d_o, kvh: int, row_tokens: Sequence[int], key_tokens: Sequence[int] = (),
         scale: Optional[float] = None, real: str = "f64", complete_keys: bool = True):
    """Sampled outputs for key/value head `kvh` and its query heads.

    o/lse/dq are returned for `row_tokens`; dk/dv for `key_tokens`.  For dk/dv to be complete, every
    token that can see a wanted key is evaluated as well (all tokens from the key to the end of its
    node's subtree) -- they are appended to the evaluated rows automatically.

    complete_keys=False evaluates `row_tokens` only: dk/dv then hold the contributions of those query
    rows alone.  By Eq. 5 every term of dK_j / dV_j carries a factor dO_i (dV_j = sum_i P_ij dO_i,
    dS_ij = P_ij (dO_i . V_j - dO_i . O_i)), so this is the complete gradient whenever d_o is zero on
    every token outside `row_tokens` -- which makes a key near the root, seen by tens of thousands of
    queries, checkable at full size.
    """
    q, k, v = _f32(q), _f32(k), _f32(v)
    n, hq, d = q.shape
    hkv = k.shape[1]
    G = hq // hkv
    d_o = None if d_o is None else _f32(d_o)
    scale = float(d) ** -0.5 if scale is None else float(scale)
    dt = np.float64 if real == "f64" else np.float32
    row_tokens = [int(t) for t in row_tokens]
    need = list(row_tokens)
    have = set(need)
    for j in (key_tokens if complete_keys else ()):
        end = int(meta["subtree_end"][meta["tok_node"][int(j)]])
        for t in range(int(j), end):
            if t not in have:
                have.add(t)
                need.append(t)
    rb = [_meta.row_branch(meta, t) for t in need]
    ptr = np.zeros(len(rb) + 1, dtype=np.int64)
    for i, p in enumerate(rb):
        ptr[i + 1] = ptr[i] + len(p)
    idx = np.ascontiguousarray(np.concatenate(rb) if rb else np.zeros(0), dtype=np.int32)
    rows_arr = np.asarray(need, dtype=np.int32)
    keys_arr = np.asarray([int(j) for j in key_tokens], dtype=np.int32)
    nr, nk = len(need), len(keys_arr)
    o = np.zeros((nr, G, d), dtype=dt)
    lse = np.zeros((nr, G), dtype=dt)
    dq = np.zeros((nr, G, d), dtype=dt)
    dk = np.zeros((max(nk, 1), d), dtype=dt)
    dv = np.zeros((max(nk, 1), d), dtype=dt)
    rc = _lib(real).oracle_attn_rows(
        ctypes.c_int64(n), hq, hkv, d, ctypes.c_double(scale), _p(q), _p(k), _p(v), _p(d_o),
        kvh, nr, _p(rows_arr), _p(ptr), _p(idx), nk, _p(keys_arr),
        _p(o), _p(lse), _p(dq), _p(dk), _p(dv))
    assert rc == 0, "oracle_attn_rows failed"
    m = len(row_tokens)
    return dict(o=o[:m], lse=lse[:m], dq=dq[:m], dk=dk[:nk], dv=dv[:nk], n_rows_evaluated=nr)


def dense(mask: np.ndarray, q, k, v, d_o=None, scale: Optional[float] = None):
    """Masked softmax attention on the given token order, numpy fp64.  mask [nq, nk] bool.
    Gradients from the textbook formulas: P = softmax(S), dV = P^T dO, dP = dO V^T,
    dS = P o (dP - rowsum(dO o O)), dQ = scale dS K, dK = scale dS^T Q."""
    q, k, v = (np.asarray(_f32(x), dtype=np.float64) for x in (q, k, v))
    nq, hq, d = q.shape
    nk, hkv, _ = k.shape
    G = hq // hkv
    scale = float(d) ** -0.5 if scale is None else float(scale)
    o = np.zeros_like(q)
    lse = np.zeros((hq, nq))
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    if d_o is not None:
        d_o = np.asarray(_f32(d_o), dtype=np.float64)
    for h in range(hq):
        kh = h // G
        s = scale * (q[:, h, :] @ k[:, kh, :].T)
        s = np.where(mask, s, -np.inf)
        m = s.max(axis=1, keepdims=True)
        e = np.exp(s - m)
        l = e.sum(axis=1, keepdims=True)
        p = e / l
        o[:, h, :] = p @ v[:, kh, :]
        lse[h] = (m + np.log(l))[:, 0]
        if d_o is not None:
            g = d_o[:, h, :]
            dv[:, kh, :] += p.T @ g
            dp = g @ v[:, kh, :].T
            dd = (g * o[:, h, :]).sum(axis=1, keepdims=True)
            ds = p * (dp - dd)
            dq[:, h, :] = scale * (ds @ k[:, kh, :])
            dk[:, kh, :] += scale * (ds.T @ q[:, h, :])
    return dict(o=o, lse=lse, dq=dq, dk=dk, dv=dv)
