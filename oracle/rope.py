"""CPU ORACLE (test infrastructure only) -- rotary position embedding in numpy fp64.

The tree position ids of Eq. 9 (depth-based positions: a token's position is the number of tokens on
its root-to-token path before it) are what a RoPE model rotates Q and K with; tokens of different
branches at the same depth get the same rotation.  The paper does not restate the rotation itself;
the reading used here is the rotate-half convention of the Qwen family it trains: for a head vector
x of even length d and i in [0, d/2),

    angle_i = pos * base^(-2 i / d)
    y[i]       = x[i] cos(angle_i) - x[i + d/2] sin(angle_i)
    y[i + d/2] = x[i + d/2] cos(angle_i) + x[i] sin(angle_i)

`inverse` rotates by -angle: it undoes the rotation and is also the backward pass (the rotation is
orthogonal, so the gradient of the input is the inverse rotation of the gradient of the output).
"""
from __future__ import annotations

import numpy as np


def _f64(x) -> np.ndarray:
    if hasattr(x, "detach"):
        x = x.detach().cpu().float().numpy()
    return np.asarray(x, dtype=np.float64)


def rope(x, pos, base: float = 1.0e6, inverse: bool = False) -> np.ndarray:
    """x [n, heads, d], pos [n] integer positions -> rotated array of the same shape (fp64)."""
    x = _f64(x)
    n, h, d = x.shape
    assert d % 2 == 0
    half = d // 2
    pos = np.asarray(pos).astype(np.float64)
    inv_freq = base ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = pos[:, None] * inv_freq[None, :]                   # [n, half]
    if inverse:
        ang = -ang
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)
