"""CPU ORACLE (test infrastructure only) -- weighted log-prob loss in numpy fp64.

Per-token objective of the paper's "Derivation" section: l_t = -log p(y_t | x_<=t); the tree loss
is sum_t (g_t / K) l_t (Eq. 4), algebraically the same as the mean over the K branches of each
branch's summed loss (Eq. 1).
"""
from __future__ import annotations

import numpy as np


def _f64(x) -> np.ndarray:
    if hasattr(x, "detach"):
        x = x.detach().cpu().float().numpy()
    return np.asarray(x, dtype=np.float64)


def _used(target, vocab):
    """Rows that enter the loss: the target names a vocabulary entry.  A negative target is the usual
    "ignore" marker; a target >= vocab names no class either and is read the same way (the paper's
    objective, "Derivation" section, is only defined for y_t in the vocabulary)."""
    return (target >= 0) & (target < vocab)


def log_softmax_gather(logits, target):
    """Per row: lse = log sum_v exp(z_v); logp = z[target] - lse (0 on ignored rows, see _used)."""
    z = _f64(logits)
    target = np.asarray(target).astype(np.int64)
    used = _used(target, z.shape[1])
    m = z.max(axis=1)
    lse = m + np.log(np.exp(z - m[:, None]).sum(axis=1))
    safe = np.where(used, target, 0)
    logp = z[np.arange(z.shape[0]), safe] - lse
    logp = np.where(used, logp, 0.0)
    return logp, lse


def loss_tree(logp, weight) -> float:
    """Eq. 4: sum_t lambda_t * (-logp_t)."""
    return float(np.sum(_f64(weight) * (-_f64(logp))))


def loss_sep_avg(paths, logp, trained_tok, adv=None) -> float:
    """Eq. 1: (1/K) sum over branches of the branch's summed per-token loss, every branch
    evaluated on its own token list (shared tokens are counted once per branch)."""
    logp = _f64(logp)
    tr = _f64(trained_tok)
    a = np.ones_like(logp) if adv is None else _f64(adv)
    total = 0.0
    for p in paths:
        branch = 0.0
        for t in p:
            branch += tr[t] * a[t] * (-logp[t])
        total += branch
    return total / len(paths)


def dlogits(logits, target, weight, lse=None, grad_scale: float = 1.0) -> np.ndarray:
    """Gradient of grad_scale * sum_r weight_r * (-logp_r) with respect to the logits:
    d/dz_rv = grad_scale * weight_r * (softmax(z_r)_v - [v == target_r]); ignored rows (_used)
    contribute nothing to the loss and get a zero gradient.  (Derivative of Eq. 4 through
    l_t = -log softmax; `lse` may be passed in, it is what the forward pass saved.)"""
    z = _f64(logits)
    target = np.asarray(target).astype(np.int64)
    w = np.ones(z.shape[0]) if weight is None else _f64(weight)
    if lse is None:
        _, lse = log_softmax_gather(z, target)
    p = np.exp(z - _f64(lse)[:, None])
    g = p.copy()
    used = _used(target, z.shape[1])
    rows = np.nonzero(used)[0]
    g[rows, target[rows]] -= 1.0
    g *= (grad_scale * w)[:, None]
    g[~used] = 0.0
    return g
