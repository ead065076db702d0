"""Small helpers shared by the tests (no method arithmetic)."""
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
