"""GPU parity: fused weighted log-prob kernel against the numpy fp64 oracle (loss within 1e-3
relative, per-row values to float32 rounding)."""
import numpy as np
import pytest
import torch

import paper_2511_00413_amd as T
import workloads as W
from oracle import loss as L
from oracle import meta as M

pytestmark = pytest.mark.gpu


def _run(logits, target, weight, **kw):
    logp, lse, loss = T.tree_weighted_logprob(logits.cuda(), target.cuda(),
                                              None if weight is None else torch.from_numpy(weight).cuda(), **kw)
    torch.cuda.synchronize()
    return logp.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64), float(loss.item())


def _check(logits, target, weight, atol):
    print(f"[case] loss rows={logits.shape[0]} vocab={logits.shape[1]} {logits.dtype}", flush=True)
    logp, lse, loss = _run(logits, target, weight)
    wl, wlse = L.log_softmax_gather(logits, target.numpy())
    assert np.abs(lse - wlse).max() <= atol
    assert np.abs(logp - wl).max() <= atol
    w = np.ones(len(wl)) if weight is None else weight
    want = L.loss_tree(wl, w)
    assert abs(loss - want) <= 1e-3 * max(abs(want), 1e-6)
    return loss, want


def test_cfg1_fp32():
    t = W.tree_cfg1()
    m = T.tree_build_meta(t.parent, t.seg_len, t.trained)
    d = W.DIMS[1]
    logits, target = W.loss_inputs(m.n_tokens, d.vocab, 1, d.logit_std, d.logit_dtype)
    loss, want = _check(logits, target, m.tok_weight, 2e-6)
    # Eq. 1 form over the branches agrees too
    om = M.dfs_meta(t.parent, t.seg_len, t.trained)
    wl, _ = L.log_softmax_gather(logits, target.numpy())
    trained_tok = np.asarray(t.trained)[om["dfs_order"]][om["tok_node"]]
    sep = L.loss_sep_avg(M.paths(om), wl, trained_tok)
    assert abs(loss - sep) <= 1e-3 * abs(sep)


@pytest.mark.parametrize("rows,vocab,dtype", [(37, 32768, "bf16"), (5, 151936, "bf16"), (64, 777, "bf16"),
                                              (33, 1001, "fp32"), (3, 8, "fp32"), (9, 1, "bf16"), (300, 5000, "bf16")])
def test_shapes_and_misaligned_rows(rows, vocab, dtype):
    logits, target = W.loss_inputs(rows, vocab, rows + vocab, 2.0, dtype)
    w = np.random.default_rng(rows).random(rows).astype(np.float32)
    _check(logits, target, w, 4e-6 * max(1.0, np.log(vocab)))


def test_strided_rows_and_chunked_accumulation():
    logits, target = W.loss_inputs(48, 2048, 7, 2.0, "bf16")
    w = np.random.default_rng(1).random(48).astype(np.float32)
    _, _, whole = _run(logits, target, w)
    acc = torch.zeros(1, dtype=torch.float32, device="cuda")
    ld, td, wd = logits.cuda(), target.cuda(), torch.from_numpy(w).cuda()
    for lo in range(0, 48, 16):
        T.tree_weighted_logprob(ld[lo:lo + 16], td[lo:lo + 16], wd[lo:lo + 16], loss_acc=acc)
    assert abs(acc.item() - whole) <= 1e-5 * abs(whole)
    # a view with a wider row stride (vocab-padded buffer)
    wide = torch.zeros(48, 2048 + 24, dtype=torch.bfloat16, device="cuda")
    wide[:, :2048] = ld
    logp_a, _, _ = T.tree_weighted_logprob(ld, td, wd)
    logp_b, _, _ = T.tree_weighted_logprob(wide[:, :2048], td, wd)
    assert torch.equal(logp_a, logp_b)


def test_special_rows():
    V = 4096
    z = torch.zeros(6, V)
    z[0, 5] = 80.0                       # one dominant logit
    z[1] = 0.25                          # uniform: logp = -ln V
    z[2] = -1e4; z[2, 9] = -9990.0       # far-negative row
    z[3, :100] = float("-inf")           # masked vocabulary entries
    z[4] = 3e4                           # large magnitude, uniform
    tgt = torch.tensor([5, 17, 9, 200, 0, -1], dtype=torch.int32)
    logp, lse, loss = _run(z, tgt, None)
    wl, wlse = L.log_softmax_gather(z, tgt.numpy())
    assert np.allclose(logp, wl, rtol=1e-6, atol=1e-5) and logp[5] == 0.0
    assert abs(logp[1] + np.log(V)) < 1e-5
    assert np.isfinite(loss)
    # deterministic
    logp2, _, loss2 = _run(z, tgt, None)
    assert np.array_equal(logp, logp2) and loss == loss2


# ---- backward: gradient with respect to the logits ------------------------------------------------
# bf16 output: one round-to-nearest-even of each element (relative 2^-9) on top of fp32 arithmetic ->
# rel-L2 <= 4e-3 and every element within 2^-8 relative + a small absolute floor; fp32 output: 1e-5.

def _grad_elem_bound(logits, weight, grad_scale, want):
    """Element-wise bound of a bf16 gradient: one rounding of the output (2^-8 of the value), plus the fp32 evaluation
    of the softmax value behind it -- exp(z - lse) carries a relative error of about 1e-5 + 2^-23 max|z| (lse is an
    fp32 number of the logits' magnitude; its rounding is a relative error of every exponential of the row).  That
    second term is relative to the softmax value p, not to p - 1: at the target of a confident row (p near 1, the
    gradient w (p - 1) small by cancellation) it is what is left, and with a vocabulary of a handful of entries every
    row of a test can be such a row."""
    z = logits.float().numpy().astype(np.float64)
    w = np.ones(z.shape[0]) if weight is None else np.asarray(weight, dtype=np.float64)
    zmax = z.max(axis=1, keepdims=True)
    e = np.exp(z - zmax)
    prob = e / e.sum(axis=1, keepdims=True)
    mag = np.abs(z).max(axis=1, keepdims=True)
    return 2.0 ** -8 * np.abs(want) + np.abs(grad_scale * w)[:, None] * prob * (1e-5 + 2.0 ** -23 * mag)


def _check_bwd(logits, target, weight, grad_scale=1.0, inplace=False):
    print(f"[case] loss bwd rows={logits.shape[0]} vocab={logits.shape[1]} {logits.dtype} inplace={inplace}", flush=True)
    lg = logits.cuda()
    tg = target.cuda()
    wt = None if weight is None else torch.from_numpy(weight).cuda()
    _, lse, _ = T.tree_weighted_logprob(lg, tg, wt)
    src = lg.clone() if inplace else lg
    got = T.tree_weighted_logprob_bwd(src, tg, wt, lse, grad_scale=grad_scale, out=src if inplace else None)
    torch.cuda.synchronize()
    got = got.float().cpu().numpy().astype(np.float64)
    want = L.dlogits(logits, target.numpy(), weight, grad_scale=grad_scale)
    num = np.sqrt(((got - want) ** 2).sum())
    den = max(np.sqrt((want ** 2).sum()), 1e-30)
    if logits.dtype == torch.bfloat16:
        assert num / den <= 4e-3, num / den
        assert np.all(np.abs(got - want) <= _grad_elem_bound(logits, weight, grad_scale, want))
    else:
        assert num / den <= 1e-5, num / den
    # ignored rows (target negative or not below the vocabulary size) are exactly zero
    ign = (target.numpy() < 0) | (target.numpy() >= logits.shape[1])
    assert np.all(got[ign] == 0.0)
    return got


@pytest.mark.parametrize("rows,vocab,dtype", [(37, 32768, "bf16"), (5, 151936, "bf16"), (64, 777, "bf16"),
                                              (33, 1001, "fp32"), (3, 8, "fp32"), (9, 1, "bf16"), (300, 5000, "bf16"),
                                              (16, 4096, "fp32"), (196, 8, "bf16"), (131, 7, "bf16")])
def test_bwd_shapes_and_misaligned_rows(rows, vocab, dtype):
    logits, target = W.loss_inputs(rows, vocab, rows + 3 * vocab, 2.0, dtype)
    target = target.clone()
    if rows > 2:
        target[1] = -1
    w = (np.random.default_rng(rows).random(rows) + 0.25).astype(np.float32)
    _check_bwd(logits, target, w, grad_scale=0.5)


@pytest.mark.parametrize("rows,vocab,seed", [(196, 8, 3100021), (131, 7, 3101361)])
def test_confident_rows_of_a_small_vocabulary(rows, vocab, seed):
    """Wide logits over a handful of entries: nearly every row puts p close to 1 on one entry, so the gradient at a
    hit target, w (p - 1), is small by cancellation and no element of the test is large.  (Shapes from a randomized
    sweep; they need the softmax-relative term of _grad_elem_bound.)"""
    logits, target = W.loss_inputs(rows, vocab, seed % 100000, 6.0, "bf16")
    w = (np.random.default_rng(rows).random(rows) + 0.25).astype(np.float32)
    _check_bwd(logits, target, w, grad_scale=0.5)
    _check_fused(logits, target, w, grad_scale=1.0 / 64, stride_pad=8)


def test_out_of_range_target_is_an_ignored_row():
    """target >= vocab: forward gives logp = 0 and adds nothing, backward gives an exactly zero row -- also
    when the logits are large and the lse entry of that row holds garbage."""
    V = 1000
    logits, target = W.loss_inputs(8, V, 31, 2.0, "bf16")
    logits = logits.clone()
    logits[2] = 300.0                      # exp(300) overflows fp32: must not turn 0 * inf into NaN
    target = target.clone()
    target[2] = V
    target[5] = V + 12345
    target[6] = -7
    w = np.linspace(0.5, 2.0, 8).astype(np.float32)
    logp, lse, loss = _run(logits, target, w)
    wl, _ = L.log_softmax_gather(logits, target.numpy())
    assert logp[2] == 0.0 and logp[5] == 0.0 and logp[6] == 0.0
    assert np.allclose(logp, wl, rtol=1e-6, atol=4e-5)
    assert abs(loss - L.loss_tree(wl, w)) <= 1e-5 * abs(L.loss_tree(wl, w))
    got = _check_bwd(logits, target, w, grad_scale=2.0)
    assert np.all(got[[2, 5, 6]] == 0.0) and np.isfinite(got).all()
    # garbage in the saved lse of the ignored rows changes nothing
    lg, tg, wt = logits.cuda(), target.cuda(), torch.from_numpy(w).cuda()
    _, lse_d, _ = T.tree_weighted_logprob(lg, tg, wt)
    lse_d = lse_d.clone()
    lse_d[[2, 5, 6]] = float("nan")
    again = T.tree_weighted_logprob_bwd(lg, tg, wt, lse_d, grad_scale=2.0)
    torch.cuda.synchronize()
    assert np.array_equal(again.float().cpu().numpy(), got.astype(np.float32))


def test_bwd_in_place_and_no_weight():
    logits, target = W.loss_inputs(24, 2048, 19, 2.0, "bf16")
    a = _check_bwd(logits, target, None)
    b = _check_bwd(logits, target, None, inplace=True)
    assert np.array_equal(a, b)


def test_bwd_strided_rows():
    logits, target = W.loss_inputs(20, 1024, 23, 2.0, "bf16")
    wide = torch.zeros(20, 1536, dtype=torch.bfloat16)
    wide[:, :1024] = logits
    lg = wide.cuda()[:, :1024]
    _, lse, _ = T.tree_weighted_logprob(lg, target.cuda(), None)
    out_wide = torch.full((20, 1280), 7.0, dtype=torch.bfloat16, device="cuda")
    T.tree_weighted_logprob_bwd(lg, target.cuda(), None, lse, out=out_wide[:, :1024])
    torch.cuda.synchronize()
    want = L.dlogits(logits, target.numpy(), None)
    got = out_wide[:, :1024].float().cpu().numpy()
    assert np.sqrt(((got - want) ** 2).sum()) / np.sqrt((want ** 2).sum()) <= 4e-3
    assert float((out_wide[:, 1024:] - 7.0).abs().max()) == 0.0       # nothing written past the row


@pytest.mark.parametrize("scheme", ["path_sum", "token_mean", "uniform"])
def test_general_path_weights_against_branch_by_branch_loss(scheme):
    """"Derivation", general path weights: the GPU's single weighted sum over unique tokens with
    lambda from tt_tree_path_weights equals the loss evaluated branch by branch, each branch on its
    own token list with its own weight (and advantages for the policy-gradient form)."""
    t = W.random_tree(91, n_nodes=14, lo=3, hi=40, shuffle=True)
    m = M.dfs_meta(t.parent, t.seg_len, t.trained)
    n, K = m["n_tokens"], m["K"]
    rng = np.random.default_rng(3)
    adv = rng.normal(size=n).astype(np.float32)
    logits, target = W.loss_inputs(n, 4096, 17, 2.0, "bf16")
    wl, _ = L.log_softmax_gather(logits, target.numpy())
    tr = m["tok_trained"].astype(np.float64)
    paths = M.paths(m)
    if scheme == "path_sum":
        w = rng.uniform(0.1, 2.0, K).astype(np.float32)
        lam, _ = T.tree_path_weights(t.parent, t.seg_len, t.trained, path_weight=w, advantage=adv)
        want = sum(float(w[k]) * sum(tr[i] * adv[i] * -wl[i] for i in p) for k, p in enumerate(paths))
    elif scheme == "token_mean":
        lam, _ = T.tree_path_weights(t.parent, t.seg_len, t.trained, scheme=T.WEIGHT_PATH_TOKEN_MEAN)
        want = sum(sum(tr[i] * -wl[i] for i in p) / tr[p].sum() for p in paths if tr[p].sum()) / K
    else:
        lam, _ = T.tree_path_weights(t.parent, t.seg_len, t.trained, scheme=T.WEIGHT_UNIFORM)
        want = float((tr * -wl).sum())
    print(f"[case] loss with general path weights, scheme {scheme}, N={n}, K={K}", flush=True)
    _, _, loss = _run(logits, target, lam)
    assert abs(loss - want) <= 1e-3 * max(abs(want), 1e-6), (loss, want)


# ---- forward and backward in one pass over the logits ---------------------------------------------
# Same bounds as the two separate calls: the one-pass kernel does the same arithmetic per element and only
# adds the row's partial sums in another order (512 instead of 256 threads), so lse / logp may differ from
# the separate call's in the last bit.

def _check_fused(logits, target, weight, grad_scale=1.0, inplace=False, stride_pad=0):
    rows, vocab = logits.shape
    print(f"[case] loss fwd+bwd rows={rows} vocab={vocab} {logits.dtype} inplace={inplace} pad={stride_pad}", flush=True)
    if stride_pad:
        buf = torch.zeros(rows, vocab + stride_pad, dtype=logits.dtype, device="cuda")
        buf[:, :vocab] = logits.cuda()
        lg = buf[:, :vocab]
    else:
        lg = logits.cuda()
    tg = target.cuda()
    wt = None if weight is None else torch.from_numpy(weight).cuda()
    sep_logp, sep_lse, sep_loss = T.tree_weighted_logprob(lg, tg, wt)
    sep_grad = T.tree_weighted_logprob_bwd(lg, tg, wt, sep_lse, grad_scale=grad_scale)
    src = lg.clone() if inplace else lg
    logp, lse, loss, got = T.tree_weighted_logprob_fwd_bwd(src, tg, wt, grad_scale=grad_scale, out=src if inplace else None)
    torch.cuda.synchronize()
    atol = (4e-6 if logits.dtype == torch.bfloat16 else 2e-6) * max(1.0, np.log(vocab))
    wl, wlse = L.log_softmax_gather(logits, target.numpy())
    assert np.abs(lse.cpu().numpy().astype(np.float64) - wlse).max() <= atol
    assert np.abs(logp.cpu().numpy().astype(np.float64) - wl).max() <= atol
    w = np.ones(rows) if weight is None else weight
    want_loss = L.loss_tree(wl, w)
    assert abs(float(loss.item()) - want_loss) <= 1e-3 * max(abs(want_loss), 1e-6)
    g = got.float().cpu().numpy().astype(np.float64)
    want = L.dlogits(logits, target.numpy(), weight, grad_scale=grad_scale)
    num, den = np.sqrt(((g - want) ** 2).sum()), max(np.sqrt((want ** 2).sum()), 1e-30)
    if logits.dtype == torch.bfloat16:
        assert num / den <= 4e-3, num / den
        assert np.all(np.abs(g - want) <= _grad_elem_bound(logits, weight, grad_scale, want))
    else:
        assert num / den <= 1e-5, num / den
    ign = (target.numpy() < 0) | (target.numpy() >= vocab)
    assert np.all(g[ign] == 0.0) and np.all(logp.cpu().numpy()[ign] == 0.0)
    # against the two separate calls: statistics to the last bits, gradient to one rounding of the output
    assert torch.allclose(lse, sep_lse, rtol=0, atol=atol) and torch.allclose(logp, sep_logp, rtol=0, atol=atol)
    assert abs(float(loss.item()) - float(sep_loss.item())) <= 1e-5 * max(abs(want_loss), 1e-6)
    gs = sep_grad.float().cpu().numpy().astype(np.float64)
    assert np.all(np.abs(g - gs) <= (2 * _grad_elem_bound(logits, weight, grad_scale, want) if logits.dtype == torch.bfloat16
                                     else 2.0 ** -7 * np.abs(gs) + 1e-7 * np.abs(gs).max()))


@pytest.mark.parametrize("rows,vocab,dtype", [(37, 32768, "bf16"),      # a row fills the LDS copy exactly
                                              (5, 151936, "bf16"),      # longer than the copy: the rest is read twice
                                              (21, 40000, "bf16"), (64, 777, "bf16"), (300, 5000, "bf16"), (9, 1, "bf16"),
                                              (103, 8, "bf16"), (132, 7, "bf16"),   # a handful of entries: confident rows
                                              (33, 1001, "fp32"), (3, 8, "fp32"), (16, 4096, "fp32"), (6, 20000, "fp32")])
def test_fwd_bwd_one_pass(rows, vocab, dtype):
    logits, target = W.loss_inputs(rows, vocab, 5 * rows + vocab, 2.0, dtype)
    target = target.clone()
    if rows > 2:
        target[1] = -1
        target[2] = vocab            # out of range: ignored as well
    w = (np.random.default_rng(rows).random(rows) + 0.25).astype(np.float32)
    _check_fused(logits, target, w, grad_scale=0.5)


def test_fwd_bwd_one_pass_in_place_and_strides():
    logits, target = W.loss_inputs(40, 4096, 77, 2.0, "bf16")
    w = (np.random.default_rng(3).random(40) + 0.25).astype(np.float32)
    _check_fused(logits, target, w, inplace=True)
    _check_fused(logits, target, None, stride_pad=24)        # rows stay on the 16-byte grid: one-pass kernel
    _check_fused(logits, target, w, stride_pad=3)            # rows off the grid: the call runs the two passes
    logits, target = W.loss_inputs(12, 1000, 78, 1.0, "fp32")
    _check_fused(logits, target, w[:12], inplace=True, grad_scale=2.0)


def test_fwd_bwd_one_pass_special_rows_and_chunks():
    V = 4096
    z = torch.zeros(6, V)
    z[0, 5] = 80.0
    z[1] = 0.25
    z[2] = -1e4; z[2, 9] = -9990.0
    z[3, :100] = float("-inf")
    z[4] = 3e4
    tgt = torch.tensor([5, 17, 9, 200, 0, -1], dtype=torch.int32)
    logp, lse, loss, grad = T.tree_weighted_logprob_fwd_bwd(z.cuda(), tgt.cuda())
    torch.cuda.synchronize()
    wl, _ = L.log_softmax_gather(z, tgt.numpy())
    assert np.allclose(logp.cpu().numpy(), wl, rtol=1e-6, atol=1e-5) and np.isfinite(grad.cpu().numpy()).all()
    want = L.dlogits(z, tgt.numpy(), None)
    # lse is an fp32 number of the logits' magnitude: its rounding (|lse| 2^-24) is a relative error of every
    # exponential of the row, on top of the fp32 arithmetic
    zn = z.numpy()
    mag = np.where(np.isfinite(zn), np.abs(zn), 0.0).max(axis=1, keepdims=True)
    gnp = grad.cpu().numpy().astype(np.float64)
    onehot = np.zeros_like(want)
    for r_, y_ in enumerate(tgt.numpy()):
        if 0 <= y_ < V:
            onehot[r_, y_] = 1.0
    prob = want + onehot                       # the error is relative to the softmax value, not to softmax - 1
    bad = np.argwhere(np.abs(gnp - want) > (1e-5 + 2.0 ** -23 * mag) * np.abs(prob) + 1e-7)
    assert len(bad) == 0, [(int(r), int(c), gnp[r, c], want[r, c]) for r, c in bad[:5]]
    # loss accumulated over row chunks; reproducible
    logits, target = W.loss_inputs(48, 2048, 7, 2.0, "bf16")
    ld, td = logits.cuda(), target.cuda()
    whole = T.tree_weighted_logprob_fwd_bwd(ld, td)
    acc = torch.zeros(1, dtype=torch.float32, device="cuda")
    parts = [T.tree_weighted_logprob_fwd_bwd(ld[lo:lo + 16], td[lo:lo + 16], loss_acc=acc)[3] for lo in range(0, 48, 16)]
    assert abs(acc.item() - whole[2].item()) <= 1e-5 * abs(whole[2].item())
    assert torch.equal(torch.cat(parts), whole[3])
    again = T.tree_weighted_logprob_fwd_bwd(ld, td)
    assert all(torch.equal(a, b) for a, b in zip(whole, again))
