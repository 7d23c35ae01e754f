"""Pins for the oracle's gather and multi-head attention (Eq. 3) -- CPU only."""
import numpy as np
import pytest
import torch

from oracle import attention


def make(seed, B=2, n=7, d=12, bias=True):
    rng = np.random.default_rng(seed)
    xs = rng.standard_normal((B, n, d))
    W = [rng.standard_normal((d, d)) / np.sqrt(d) for _ in range(4)]
    b = [0.1 * rng.standard_normal(d) for _ in range(4)] if bias else [None] * 4
    dy = rng.standard_normal((B, n, d))
    return xs, W, b, dy


def torch_mha(xs, W, b, H):
    """Same expression through torch's library SDPA on CPU in float64."""
    B, n, d = xs.shape
    dk = d // H
    proj = lambda w, bb: xs @ w + (bb if bb is not None else 0)
    q, k, v = (proj(W[i], b[i]).reshape(B, n, H, dk).transpose(1, 2) for i in range(3))
    o = torch.nn.functional.scaled_dot_product_attention(q, k, v)
    o = o.transpose(1, 2).reshape(B, n, d)
    return o @ W[3] + (b[3] if b[3] is not None else 0)


@pytest.mark.parametrize("H,bias", [(1, False), (3, True), (4, False)])
def test_forward_matches_library_sdpa(H, bias):
    xs, W, b, _ = make(H, bias=bias)
    y, cache = attention.mha_forward(xs, *W, H, *b)
    tb = [torch.from_numpy(v) if v is not None else None for v in b]
    ref = torch_mha(torch.from_numpy(xs), [torch.from_numpy(w) for w in W], tb, H)
    assert np.allclose(y, ref.numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(cache["p"].sum(axis=-1), 1.0, rtol=1e-14)      # softmax rows


def test_single_head_is_eq_3_written_out():
    xs, W, _, _ = make(5, B=1, n=5, d=8, bias=False)
    y, _ = attention.mha_forward(xs, *W, 1)
    q, k, v = xs[0] @ W[0], xs[0] @ W[1], xs[0] @ W[2]
    out = np.zeros_like(q)
    for i in range(5):
        s = np.array([q[i] @ k[j] / np.sqrt(8.0) for j in range(5)])
        p = np.exp(s) / np.exp(s).sum()
        out[i] = sum(p[j] * v[j] for j in range(5))
    assert np.allclose(y[0], out @ W[3], rtol=1e-12)


@pytest.mark.parametrize("H,bias", [(2, True), (3, False)])
def test_backward_matches_autograd(H, bias):
    xs, W, b, dy = make(10 + H, bias=bias)
    y, cache = attention.mha_forward(xs, *W, H, *b)
    g = attention.mha_backward(dy, cache)
    txs = torch.from_numpy(xs).requires_grad_()
    tW = [torch.from_numpy(w).requires_grad_() for w in W]
    tb = [torch.from_numpy(v).requires_grad_() if v is not None else None for v in b]
    ref = torch_mha(txs, tW, tb, H)
    ref.backward(torch.from_numpy(dy))
    assert np.allclose(g["dxs"], txs.grad.numpy(), rtol=1e-10, atol=1e-12)
    for name, t in zip(("dWq", "dWk", "dWv", "dWo"), tW):
        assert np.allclose(g[name], t.grad.numpy(), rtol=1e-10, atol=1e-12), name
    if bias:
        for name, t in zip(("dbq", "dbk", "dbv", "dbo"), tb):
            assert np.allclose(g[name], t.grad.numpy(), rtol=1e-10, atol=1e-12), name


def test_backward_matches_central_finite_differences():
    H = 2
    xs, W, b, dy = make(21, B=1, n=4, d=6)
    _, cache = attention.mha_forward(xs, *W, H, *b)
    g = attention.mha_backward(dy, cache)
    loss = lambda xs_, W_, b_: float((attention.mha_forward(xs_, *W_, H, *b_)[0] * dy).sum())
    eps = 1e-6
    rng = np.random.default_rng(0)
    for _ in range(12):                                               # sampled coordinates of every operand
        i = tuple(rng.integers(0, s) for s in xs.shape)
        xp, xm = xs.copy(), xs.copy()
        xp[i] += eps
        xm[i] -= eps
        assert (loss(xp, W, b) - loss(xm, W, b)) / (2 * eps) == pytest.approx(g["dxs"][i], rel=1e-6, abs=1e-8)
    for wi, name in enumerate(("dWq", "dWk", "dWv", "dWo")):
        for _ in range(6):
            i = tuple(rng.integers(0, s) for s in W[wi].shape)
            Wp = [w.copy() for w in W]
            Wm = [w.copy() for w in W]
            Wp[wi][i] += eps
            Wm[wi][i] -= eps
            fd = (loss(xs, Wp, b) - loss(xs, Wm, b)) / (2 * eps)
            assert fd == pytest.approx(g[name][i], rel=1e-6, abs=1e-8), name
    for bi, name in enumerate(("dbq", "dbk", "dbv", "dbo")):
        bp = [v.copy() for v in b]
        bm = [v.copy() for v in b]
        bp[bi][2] += eps
        bm[bi][2] -= eps
        fd = (loss(xs, W, bp) - loss(xs, W, bm)) / (2 * eps)
        assert fd == pytest.approx(g[name][2], rel=1e-6, abs=1e-8), name


def test_gather_and_its_adjoint():
    rng = np.random.default_rng(1)
    tok = rng.standard_normal((3, 10, 4))
    sel = np.array([0, 3, 4, 9])
    xs = attention.gather(tok, sel)
    assert xs.shape == (3, 4, 4)
    for b in range(3):
        for i, n in enumerate(sel):
            assert np.array_equal(xs[b, i], tok[b, n])
    g = rng.standard_normal(xs.shape)
    back = attention.scatter_add(g, sel, 10)
    assert (xs * g).sum() == pytest.approx((tok * back).sum(), rel=1e-13)   # <gather t, g> = <t, scatter g>
    assert np.all(back[:, [1, 2, 5, 6, 7, 8]] == 0)


def test_identity_selection_is_dense_attention():
    xs, W, b, _ = make(2, B=2, n=9, d=8)
    dense, _ = attention.mha_forward(xs, *W, 2, *b)
    sub, _ = attention.mha_forward(attention.gather(xs, np.arange(9)), *W, 2, *b)
    assert np.array_equal(dense, sub)


def test_attention_is_permutation_equivariant_over_tokens():
    xs, W, b, _ = make(3, B=1, n=6, d=8)
    perm = np.array([3, 1, 5, 0, 2, 4])
    y, _ = attention.mha_forward(xs, *W, 2, *b)
    yp, _ = attention.mha_forward(xs[:, perm], *W, 2, *b)
    assert np.allclose(yp, y[:, perm], rtol=1e-12, atol=1e-13)
