"""Small helpers shared by the tests: golden-file parsing, error norms and the error model of the attention parity
bounds (no arithmetic of the hot path itself)."""
import os

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _num(x):
    if "/" in x:
        a, b = x.split("/")
        return int(a) / int(b)
    if "." in x:
        return float(x)
    return int(x)


def read_golden(name):
    """Parse tests/golden/<name>: '#' comments; 'key: v v v' lines -> dict of lists of numbers."""
    out = {}
    with open(os.path.join(ROOT, "tests", "golden", name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            key, vals = line.split(":", 1)
            out[key.strip()] = [_num(x) for x in vals.split()]
    return out


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b.ravel())
    return float(np.linalg.norm((a - b).ravel()) / (den if den > 0 else 1.0))


def row_err(a, b, floor=0.05, budget=None):
    """Largest per-row error: rows are the vectors along the last axis (one token and head),
    err_r = max(0, |a_r - b_r| - budget_r) / max(|b_r|, floor * rms over rows of |b_r|).  The floor keeps
    rows whose reference is (nearly) zero by cancellation -- a query that sees one key has dQ = 0
    exactly -- from dividing rounding noise by nothing; a wrong row still reads O(1).  `budget`
    (one number per row, same units as the rows) is an absolute error the row may carry for a stated reason
    (saved_o_budget_dq / saved_o_budget_dk below)."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    if b.size == 0:
        return 0.0
    nb = np.linalg.norm(b, axis=-1)
    rms = float(np.sqrt(np.mean(nb ** 2)))
    den = np.maximum(nb, floor * rms if rms > 0 else 1.0)
    err = np.linalg.norm(a - b, axis=-1)
    if budget is not None:
        err = np.maximum(err - np.asarray(budget, dtype=np.float64), 0.0)
    return float((err / den).max())


def saved_o_rounding(d_o, o_ref, dtype):
    """The backward pass forms D_i = dO_i . O_i from the O tensor it is given.  That tensor has the I/O dtype: each
    element carries a rounding error of at most half a unit in the last place, |O| eps with eps = 2^-9 for bf16 (8
    significant bits) and 2^-24 for fp32, which the oracle's own fp64 O does not have.  D_i therefore moves by at
    most e_i = eps sum_c |dO_ic O_ic|.  d_o, o_ref [..., d]; returns e [...]."""
    eps = 2.0 ** -9 if dtype == "bf16" else 2.0 ** -24
    return eps * np.abs(np.asarray(d_o, dtype=np.float64) * np.asarray(o_ref, dtype=np.float64)).sum(axis=-1)


def dq_allowance(d_o, o_ref, k_norm_max, scale, dtype):
    """What the rounding of the saved O may add to a dQ row (an absolute budget for row_err).
    dQ_i = scale sum_j P_ij (dP_ij - D_i) K_j; a change dD_i of D_i moves it by -scale dD_i sum_j P_ij K_j, a
    vector no longer than scale e_i max_j |K_j| (a convex combination of keys; e_i from saved_o_rounding).
    For a query with many keys this is far below the other rounding noise; for one that sees few keys or whose
    softmax is concentrated dQ_i itself is small by cancellation and this term dominates -- in the fp32-arithmetic
    kernels exactly as in the MFMA kernels (measured over 1600 random trees: the error of such rows stays below
    0.3 of this bound in both).  d_o, o_ref [..., d]; k_norm_max broadcastable to their row shape."""
    return float(scale) * saved_o_rounding(d_o, o_ref, dtype) * np.asarray(k_norm_max, dtype=np.float64)


def dk_allowance(q, k, lse_ref, visible, d_o, o_ref, scale, dtype):
    """The same for dK rows: dK_j = scale sum_i P_ij (dP_ij - D_i) Q_i over the queries that see key j (all query
    heads of its kv head), so the rounding of the saved O may move it by up to scale sum_i P_ij e_i |Q_i|.  It
    matters for the keys of short nodes near a root, whose queries see one or two keys (P_ij near 1, dK_j small by
    cancellation).  Needs the softmax probabilities, formed here from the inputs and the reference LSE:
    q [n, hq, d], k [m, hkv, d], lse_ref [hq, n], visible [n, m] bool (query i sees key j), d_o, o_ref [n, hq, d];
    returns [m, hkv].  O(n m hq d): for the small cases only."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    lse_ref = np.asarray(lse_ref, dtype=np.float64)
    e = saved_o_rounding(d_o, o_ref, dtype)
    hq, hkv = q.shape[1], k.shape[1]
    qn = np.linalg.norm(q, axis=-1)
    out = np.zeros((k.shape[0], hkv))
    for h in range(hq):
        p = np.exp(float(scale) * q[:, h] @ k[:, h // (hq // hkv)].T - lse_ref[h][:, None]) * visible
        out[:, h // (hq // hkv)] += float(scale) * (p * (e[:, h] * qn[:, h])[:, None]).sum(axis=0)
    return out


def max_abs(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.abs(a - b).max()) if b.size else 0.0


# Attention parity bounds.  "l2": relative L2 over the whole tensor.  "row": largest per-row error
# (row_err: one query token and head for O and dQ, one key token and kv head for dK and dV), and for
# LSE the largest absolute difference.  The bf16 numbers follow from the rounding model of the MFMA
# path: P and dS are rounded to bf16 once (8 significant bits: relative error <= 2^-8 per element, about
# 1.7e-3 rms, independent between elements), Q (forward, dQ pass) or K (dK/dV pass) is re-rounded after the
# softmax scale is folded in, sums are fp32, outputs are rounded to bf16 once.  A row of 128 outputs then
# carries a relative error of about sqrt(2..3) x 1.7e-3 = 2.4e-3 - 3e-3 in L2 (measured: O, dK, dV rows
# <= 4.7e-3 over all cases); the row bounds leave a factor ~3.  A row that is wrong (a dropped tile, a wrong
# mask bit) reads O(1).  dQ and dK rows may in addition carry what the rounding of the saved O contributes
# (dq_allowance, dk_allowance: an absolute budget taken off the row's error before it is compared); with it
# the worst rows -- queries near the start of a root, which see one or two keys, and the keys they see --
# were measured at 5e-3 over 1600 random trees, like all others.
ATTN_TOL = {
    "fp32": {"l2": dict(o=1e-5, lse=1e-5, dq=1e-5, dk=1e-5, dv=1e-5),
             "row": dict(o=1e-5, lse=1e-5, dq=5e-4, dk=5e-5, dv=5e-5)},
    "bf16": {"l2": dict(o=1e-2, lse=1e-2, dq=2e-2, dk=2e-2, dv=2e-2),
             "row": dict(o=1.5e-2, lse=5e-3, dq=1.5e-2, dk=1.5e-2, dv=1.5e-2)},
}


def attention_errors(got, want, dq_allow=None, dk_allow=None):
    """got / want: dicts of arrays with the same shapes; keys among o, dq ([.., d] rows), lse, dk, dv
    (and dk_prefix / dv_prefix).  dq_allow / dk_allow: per-row budgets for dq / dk (a dict may give one per key of
    `want`, e.g. dk and dk_prefix).  Returns (whole-tensor rel-L2, per-row error) per key."""
    budgets = {}
    if dq_allow is not None:
        budgets["dq"] = dq_allow
    if isinstance(dk_allow, dict):
        budgets.update(dk_allow)
    elif dk_allow is not None:
        budgets["dk"] = dk_allow
    l2, row = {}, {}
    for key, ref in want.items():
        l2[key] = rel_l2(got[key], ref)
        if key == "lse":
            row[key] = max_abs(got[key], ref)
        else:
            row[key] = row_err(got[key], ref, budget=budgets.get(key))
    return l2, row


def assert_attention_close(got, want, dtype, label="", dq_allow=None, dk_allow=None):
    """dq_allow: per-row budget for dQ (dq_allowance), same leading shape as want["dq"] without d; dk_allow: the same
    for dK (dk_allowance), or a dict of budgets by output name."""
    l2, row = attention_errors(got, want, dq_allow, dk_allow)
    print(f"   {label} rel-L2:", {k_: f"{e:.2e}" for k_, e in l2.items()}, flush=True)
    print(f"   {label} per-row:", {k_: f"{e:.2e}" for k_, e in row.items()}, flush=True)
    tol = ATTN_TOL[dtype]
    for key in want:
        base = key.split("_")[0]
        assert l2[key] <= tol["l2"][base], ("rel-L2", key, l2[key])
        assert row[key] <= tol["row"][base], ("per-row", key, row[key])
    return l2, row
