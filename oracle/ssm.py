"""Oracle for the SSM-layer adaptations (Section "Implementation", paragraph "SSM Layers (GDN)";
Appendix "Tree-Correct Causal Convolution", "Tree-Aware SSM State Routing").

TEST INFRASTRUCTURE ONLY: plain numpy in fp64, no relation to the HIP library's code.

Both adaptations have a plain definition, which is what is written here: every token sees, as its
left context / incoming recurrent state, exactly what it would see in a standalone forward over its
own root-to-token sequence.  With `tok_pred[t]` = the token that precedes t on that sequence
(t-1 inside a node, the last token of the nearest non-empty ancestor at a node's first token, -1 at
the start of a branch) the causal convolution and the recurrence simply follow `tok_pred` instead
of t-1.  The paper's chunk-per-node procedures (parent's saved conv context, parent's end state)
compute the same thing node by node.
"""
from typing import Optional

import numpy as np


def _f64(x) -> np.ndarray:
    if hasattr(x, "detach"):
        x = x.detach().cpu().float().numpy()
    return np.asarray(x, dtype=np.float64)


def pred_chain(tok_pred, depth: int) -> np.ndarray:
    """P[m][t] = the m-th predecessor of t along its own sequence (P[0][t] = t), -1 if there is none."""
    tok_pred = np.asarray(tok_pred, dtype=np.int64)
    n = len(tok_pred)
    P = np.full((depth, n), -1, dtype=np.int64)
    if depth:
        P[0] = np.arange(n)
    for m in range(1, depth):
        prev = P[m - 1]
        P[m] = np.where(prev >= 0, tok_pred[np.maximum(prev, 0)], -1)
    return P


def _silu(z):
    return z / (1.0 + np.exp(-z))


def _dsilu(z):
    s = 1.0 / (1.0 + np.exp(-z))
    return s * (1.0 + z * (1.0 - s))


def tree_conv(x, weight, bias, tok_pred, activation: Optional[str] = "silu"):
    """Depthwise causal convolution along every token's own sequence.
    x [N, C]; weight [C, K] (weight[c, K-1] multiplies the token itself, weight[c, 0] the token K-1
    steps back -- the layout of a depthwise conv1d with left padding K-1); bias [C] or None;
    positions before the start of a branch contribute zero.  Returns (y [N, C], pre-activation)."""
    x, w = _f64(x), _f64(weight)
    n, c = x.shape
    K = w.shape[1]
    P = pred_chain(tok_pred, K)
    pre = np.zeros((n, c)) if bias is None else np.tile(_f64(bias), (n, 1))
    for m in range(K):
        ok = P[m] >= 0
        pre[ok] += w[:, K - 1 - m][None, :] * x[P[m][ok]]
    if activation == "silu":
        return _silu(pre), pre
    assert activation is None
    return pre, pre


def tree_conv_bwd(x, weight, bias, tok_pred, dy, activation: Optional[str] = "silu"):
    """Vector-Jacobian product of tree_conv: (dx [N, C], dweight [C, K], dbias [C]) for upstream dy."""
    x, w, dy = _f64(x), _f64(weight), _f64(dy)
    n, c = x.shape
    K = w.shape[1]
    P = pred_chain(tok_pred, K)
    _, pre = tree_conv(x, w, bias, tok_pred, activation)
    g = dy * _dsilu(pre) if activation == "silu" else dy
    dx = np.zeros((n, c))
    dw = np.zeros((c, K))
    for m in range(K):
        ok = P[m] >= 0
        np.add.at(dx, P[m][ok], w[:, K - 1 - m][None, :] * g[ok])
        dw[:, K - 1 - m] = (g[ok] * x[P[m][ok]]).sum(axis=0)
    return dx, dw, g.sum(axis=0)


def gdn_tree(q, k, v, g, beta, tok_pred, scale: Optional[float] = None, return_states: bool = False):
    """Gated delta rule with tree state routing (Section "Implementation", "SSM Layers (GDN)" (i);
    Appendix "Tree-Aware SSM State Routing"), as the token-by-token recurrence it is defined by.

    Per value head h (key head h // (Hv // Hk)), state S in R^{Dk x Dv}, token t with predecessor
    p = tok_pred[t] on its own sequence (S_p = 0 where p = -1: the start of a branch):
        S~  = exp(g_t) * S_p                         decay
        d   = beta_t * (v_t - S~^T k_t)              delta-rule correction of the value
        S_t = S~ + k_t d^T
        o_t = scale * S_t^T q_t
    Reading the state of the PREDECESSOR ON THE TOKEN'S OWN SEQUENCE -- the end state of the parent
    node at a node's first token -- instead of the previous token in DFS order is the whole
    adaptation; the paper's node-per-chunk procedure computes exactly this.
    q, k [N, Hk, Dk]; v [N, Hv, Dv]; g, beta [N, Hv] (g <= 0 is the log of the decay).
    Returns o [N, Hv, Dv] (and the state after every token if asked; small inputs only)."""
    q, k, v, g, beta = _f64(q), _f64(k), _f64(v), _f64(g), _f64(beta)
    n, hk, dk = q.shape
    hv, dv = v.shape[1], v.shape[2]
    rep = hv // hk
    scale = float(dk) ** -0.5 if scale is None else float(scale)
    tok_pred = np.asarray(tok_pred, dtype=np.int64)
    states = np.zeros((n, hv, dk, dv))
    o = np.zeros((n, hv, dv))
    for t in range(n):
        p = tok_pred[t]
        for h in range(hv):
            kt, qt = k[t, h // rep], q[t, h // rep]
            s = np.exp(g[t, h]) * (states[p, h] if p >= 0 else np.zeros((dk, dv)))
            d = beta[t, h] * (v[t, h] - s.T @ kt)
            s = s + np.outer(kt, d)
            states[t, h] = s
            o[t, h] = scale * (s.T @ qt)
    return (o, states) if return_states else o


def gdn_tree_bwd(q, k, v, g, beta, tok_pred, d_o, scale: Optional[float] = None):
    """Vector-Jacobian product of gdn_tree for upstream d_o [N, Hv, Dv]: (dq, dk [N, Hk, Dk], dv [N, Hv, Dv],
    dg, dbeta [N, Hv]).  The recurrence run backwards: dL/dS_t collects scale * q_t d_o_t^T and what every
    successor of t on any branch sends back (several successors at a branch point: their contributions
    add, which is the gradient accumulation at the shared parent state of the paper's "SSM Layers"
    paragraph).  Per token, with S~ = e^g S_p, r = v - S~^T k, d = beta r, S_t = S~ + k d^T, R = dL/dS_t:
        dq = scale S_t d_o;   dd = R^T k;   dv = beta dd;   dbeta = dd . r
        dS~ = R - beta k dd^T;   dk = R d - beta S~ dd;   dg = <dS~, S~>;   dL/dS_p += e^g dS~
    Small inputs only (keeps every state)."""
    q, k, v, g, beta, d_o = _f64(q), _f64(k), _f64(v), _f64(g), _f64(beta), _f64(d_o)
    n, hk, dk = q.shape
    hv, dv = v.shape[1], v.shape[2]
    rep = hv // hk
    scale = float(dk) ** -0.5 if scale is None else float(scale)
    tok_pred = np.asarray(tok_pred, dtype=np.int64)
    _, states = gdn_tree(q, k, v, g, beta, tok_pred, scale, return_states=True)
    dS = np.zeros_like(states)
    dq, dkk, dvv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    dg, dbeta = np.zeros_like(g), np.zeros_like(beta)
    for t in range(n - 1, -1, -1):               # successors always come later in DFS order
        p = tok_pred[t]
        for h in range(hv):
            kh = h // rep
            kt, qt = k[t, kh], q[t, kh]
            s_t = states[t, h]
            s_dec = np.exp(g[t, h]) * (states[p, h] if p >= 0 else np.zeros((dk, dv)))
            r = v[t, h] - s_dec.T @ kt
            d = beta[t, h] * r
            R = dS[t, h] + scale * np.outer(qt, d_o[t, h])
            dq[t, kh] += scale * (s_t @ d_o[t, h])
            dd = R.T @ kt
            dvv[t, h] = beta[t, h] * dd
            dbeta[t, h] = dd @ r
            ds_dec = R - beta[t, h] * np.outer(kt, dd)
            dkk[t, kh] += R @ d - beta[t, h] * (s_dec @ dd)
            dg[t, h] = float(np.sum(ds_dec * s_dec))
            if p >= 0:
                dS[p, h] += np.exp(g[t, h]) * ds_dec
    return dq, dkk, dvv, dg, dbeta
