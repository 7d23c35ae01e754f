"""Pins for the oracle's embedding of the kept variates -- CPU only."""
import numpy as np
import pytest
import torch

from oracle import attention, embedding


def make(seed, B=3, N=9, L=10, d=6):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B, N, L)) * rng.uniform(0.1, 10, (1, N, 1)) + rng.uniform(-5, 5, (1, N, 1))
    We = rng.standard_normal((L, d))
    be = rng.standard_normal(d)
    sel = np.sort(rng.choice(N, 4, replace=False))
    return x, sel, We, be


def test_one_hot_windows_pick_rows_of_the_weight():
    """Without standardisation a window that is 1 at time t and 0 elsewhere embeds to row t of We (+ be)."""
    L, d = 7, 5
    rng = np.random.default_rng(0)
    We, be = rng.standard_normal((L, d)), rng.standard_normal(d)
    x = np.eye(L)[None]                                                  # variate n is the one-hot window at t = n
    sel = np.array([1, 4, 6])
    xs = embedding.embed_forward(x, sel, We, be, standardise=False)
    assert np.allclose(xs[0], We[sel] + be, atol=1e-15)
    assert np.allclose(embedding.embed_forward(x, sel, We, None, standardise=False)[0], We[sel], atol=1e-15)


def test_identity_weight_returns_the_standardised_window():
    x, sel, _, _ = make(1)
    L = x.shape[-1]
    z = embedding.embed_forward(x, sel, np.eye(L), None, standardise=True)
    assert np.allclose(z.mean(axis=-1), 0, atol=1e-12)
    assert np.allclose((z ** 2).mean(axis=-1), 1, atol=1e-12)
    # standardisation removes offset and positive scale of the window
    z2 = embedding.embed_forward(3.5 * x - 2.0, sel, np.eye(L), None, standardise=True)
    assert np.allclose(z, z2, atol=1e-10)
    # a constant window becomes zeros, not NaN
    xc = np.full((1, 2, L), 4.25)
    assert np.array_equal(embedding.embed_forward(xc, [0, 1], np.eye(L), None), np.zeros((1, 2, L)))


@pytest.mark.parametrize("standardise", [False, True])
def test_forward_is_the_library_matmul_of_the_gathered_windows(standardise):
    x, sel, We, be = make(2)
    z = attention.gather(x, sel)
    if standardise:
        z = (z - z.mean(-1, keepdims=True)) / z.std(-1, keepdims=True)
    want = np.einsum("bil,ld->bid", z, We) + be
    assert np.allclose(embedding.embed_forward(x, sel, We, be, standardise), want, rtol=1e-12, atol=1e-12)


def test_kept_only_equals_embedding_everything_then_gathering():
    """Embedding the kept variates gives the rows that a gather of the all-variate embedding would give."""
    x, sel, We, be = make(3)
    full = embedding.embed_forward(x, np.arange(x.shape[1]), We, be)
    assert np.array_equal(embedding.embed_forward(x, sel, We, be), attention.gather(full, sel))


@pytest.mark.parametrize("standardise", [False, True])
def test_backward_against_autograd_and_finite_differences(standardise):
    x, sel, We, be = make(4)
    rng = np.random.default_rng(9)
    dxs = rng.standard_normal((x.shape[0], len(sel), We.shape[1]))
    dWe, dbe = embedding.embed_backward(x, sel, dxs, standardise)
    # torch autograd of the same expression in float64
    z = torch.from_numpy(embedding.kept_windows(x, sel, standardise))
    Wt = torch.from_numpy(We).requires_grad_()
    bt = torch.from_numpy(be).requires_grad_()
    ((z @ Wt + bt) * torch.from_numpy(dxs)).sum().backward()
    assert np.allclose(dWe, Wt.grad.numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(dbe, bt.grad.numpy(), rtol=1e-12, atol=1e-12)
    # central differences on a few entries
    f = lambda W, b: float((embedding.embed_forward(x, sel, W, b, standardise) * dxs).sum())
    for (t, j) in [(0, 0), (3, 2), (9, 5)]:
        Wp, Wm = We.copy(), We.copy()
        Wp[t, j] += 1e-6
        Wm[t, j] -= 1e-6
        assert abs((f(Wp, be) - f(Wm, be)) / 2e-6 - dWe[t, j]) < 1e-6 * max(1.0, abs(dWe[t, j]))
    bp, bm = be.copy(), be.copy()
    bp[1] += 1e-6
    bm[1] -= 1e-6
    assert abs((f(We, bp) - f(We, bm)) / 2e-6 - dbe[1]) < 1e-6 * max(1.0, abs(dbe[1]))


def test_adjoint_identity():
    """<xs, dxs> = <We, dWe> + <be, dbe>: the backward is the adjoint of the (linear in We, be) forward."""
    x, sel, We, be = make(5)
    rng = np.random.default_rng(3)
    dxs = rng.standard_normal((x.shape[0], len(sel), We.shape[1]))
    xs = embedding.embed_forward(x, sel, We, be)
    dWe, dbe = embedding.embed_backward(x, sel, dxs)
    assert np.isclose((xs * dxs).sum(), (We * dWe).sum() + (be * dbe).sum(), rtol=1e-12)
