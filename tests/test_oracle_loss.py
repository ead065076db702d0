"""Pins for oracle/loss.py: closed forms, a library routine, and the Eq. 1 == Eq. 4 identity."""
import numpy as np
import torch

import workloads as W
from oracle import loss as L
from oracle import meta as M


def test_closed_forms():
    V = 1024
    z = np.full((3, V), 0.25)
    logp, lse = L.log_softmax_gather(z, [0, 5, V - 1])
    assert np.allclose(logp, -np.log(V), atol=1e-14) and np.allclose(lse, 0.25 + np.log(V), atol=1e-14)
    z = np.zeros((2, V))
    z[0, 7] = 80.0
    z[1, 9] = 80.0
    logp, _ = L.log_softmax_gather(z, [7, 3])
    assert abs(logp[0]) < 1e-30 + V * np.exp(-80.0) * 1.01 and abs(logp[1] + 80.0) < 1e-12
    logp, _ = L.log_softmax_gather(z, [-1, 9])
    assert logp[0] == 0.0


def test_against_library_log_softmax():
    logits, target = W.loss_inputs(64, 777, 3, std=2.0)
    logp, lse = L.log_softmax_gather(logits, target.numpy())
    ref = torch.log_softmax(logits.double(), dim=-1)
    want = ref[torch.arange(64), target.long()].numpy()
    assert np.allclose(logp, want, atol=1e-13)
    assert np.allclose(lse, torch.logsumexp(logits.double(), dim=-1).numpy(), atol=1e-13)


def test_sep_avg_equals_tree_loss():
    for seed in range(10):
        t = W.random_tree(seed, n_nodes=2 + seed, lo=1, hi=6, n_roots=1 + seed % 2, p_zero=0.1)
        m = M.dfs_meta(t.parent, t.seg_len, t.trained)
        n = m["n_tokens"]
        if n == 0:
            continue
        logits, target = W.loss_inputs(n, 50, seed)
        logp, _ = L.log_softmax_gather(logits, target.numpy())
        trained_tok = np.asarray(t.trained)[m["dfs_order"]][m["tok_node"]]
        a = L.loss_sep_avg(M.paths(m), logp, trained_tok)
        b = L.loss_tree(logp, m["tok_weight"])
        assert abs(a - b) <= 1e-6 * max(1.0, abs(a))
        # with exact (fp64) weights the two forms agree to rounding
        w64 = trained_tok * (m["node_g"][m["tok_node"]] / m["K"])
        assert abs(a - L.loss_tree(logp, w64)) <= 1e-13 * max(1.0, abs(a))


def test_single_chain_is_plain_nll_sum():
    c = W.chain_tree([4, 5])
    m = M.dfs_meta(c.parent, c.seg_len, c.trained)
    logits, target = W.loss_inputs(9, 31, 5)
    logp, _ = L.log_softmax_gather(logits, target.numpy())
    assert np.all(m["tok_weight"] == 1.0)
    nll = torch.nn.functional.cross_entropy(logits.double(), target.long(), reduction="sum").item()
    assert abs(L.loss_tree(logp, m["tok_weight"]) - nll) < 1e-12


def _rand_case(seed, rows=7, vocab=23):
    rng = np.random.default_rng(seed)
    z = rng.normal(size=(rows, vocab)) * 3.0
    y = rng.integers(0, vocab, size=rows)
    y[1] = -1                                   # an ignored row
    w = rng.uniform(0.1, 2.0, size=rows)
    return z, y, w


def test_dlogits_matches_finite_differences():
    z, y, w = _rand_case(3)
    g = L.dlogits(z, y, w, grad_scale=0.7)
    f = lambda zz: 0.7 * L.loss_tree(L.log_softmax_gather(zz, y)[0], w)
    h = 1e-6
    for (r, v) in [(0, 0), (0, int(y[0])), (2, 5), (3, int(y[3])), (6, 22), (1, 4)]:
        zp, zm = z.copy(), z.copy()
        zp[r, v] += h
        zm[r, v] -= h
        fd = (f(zp) - f(zm)) / (2 * h)
        assert abs(fd - g[r, v]) <= 1e-7 * max(1.0, abs(fd)), (r, v, fd, g[r, v])


def test_dlogits_closed_forms():
    # uniform logits: softmax = 1/V everywhere
    V = 16
    z = np.full((2, V), 1.25)
    g = L.dlogits(z, [3, -1], [2.0, 5.0])
    want = np.full(V, 2.0 / V)
    want[3] -= 2.0
    assert np.allclose(g[0], want, rtol=0, atol=1e-15)
    assert np.all(g[1] == 0.0)                    # ignored row
    # every row with a valid target sums to zero (softmax sums to one)
    z, y, w = _rand_case(5, rows=9, vocab=31)
    g = L.dlogits(z, y, w)
    assert np.abs(g[y >= 0].sum(axis=1)).max() <= 1e-14
    # a saved lse gives the same result as recomputing it
    _, lse = L.log_softmax_gather(z, y)
    assert np.array_equal(L.dlogits(z, y, w, lse=lse), g)


def test_dlogits_against_library_autograd():
    z, y, w = _rand_case(11, rows=12, vocab=40)
    zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    yt = torch.tensor(np.where(y >= 0, y, 0))
    nll = torch.nn.functional.cross_entropy(zt, yt, reduction="none")
    loss = (torch.tensor(w * (y >= 0)) * nll).sum()
    loss.backward()
    assert np.allclose(zt.grad.numpy(), L.dlogits(z, y, w), rtol=1e-12, atol=1e-14)


def test_ignored_rows_against_library_ignore_index():
    """A negative target and a target >= vocab are both ignored rows: zero loss term, zero gradient.
    Pinned to the library's cross entropy with ignore_index (sum reduction) and its autograd."""
    V = 50
    logits, target = W.loss_inputs(12, V, 5, std=2.0)
    target = target.clone().long()
    target[3] = -1
    target[7] = V            # first value outside the vocabulary
    target[9] = V + 1000
    w = np.linspace(0.5, 1.5, 12)
    logp, _ = L.log_softmax_gather(logits, target.numpy())
    assert logp[3] == 0.0 and logp[7] == 0.0 and logp[9] == 0.0
    z = logits.double().clone().requires_grad_(True)
    lib_t = target.clone()
    lib_t[(lib_t < 0) | (lib_t >= V)] = -100
    per_row = torch.nn.functional.cross_entropy(z, lib_t, ignore_index=-100, reduction="none")
    loss = (torch.from_numpy(w) * per_row).sum()
    loss.backward()
    assert abs(L.loss_tree(logp, w) - float(loss.detach())) < 1e-12
    g = L.dlogits(logits, target.numpy(), w)
    assert np.allclose(g, z.grad.numpy(), atol=1e-13)
    assert np.all(g[[3, 7, 9]] == 0.0)
