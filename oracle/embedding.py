"""Token embedding of the kept variates only (Sec. 3.1, Sec. 3.3: the reduction works "directly from raw
variates", so the embedding of the dropped ones is never formed), forward and backward, in fp64.
Test infrastructure.

Conventions (the paper defers the tokenisation to its variate-tokenised backbone, Sec. 4.1): a token is a
shared linear map R^L -> R^d of one variate's whole lookback window, xs = z We + be with We [L, d]; with
`standardise` the window is first brought to zero mean and unit (population) variance over time, a constant
window becoming all zeros; the windows themselves are data, so the backward pass has only the gradients of
We and be.
"""
import numpy as np


def kept_windows(x, sel, standardise=True):
    """z[b, i, :] = window sel[i] of batch element b, standardised over time if asked."""
    x = np.asarray(x, dtype=np.float64)
    z = x[:, np.asarray(sel, dtype=np.int64), :]
    if standardise:
        mu = z.mean(axis=-1, keepdims=True)
        sd = np.sqrt(((z - mu) ** 2).mean(axis=-1, keepdims=True))
        z = (z - mu) / np.where(sd > 0, sd, 1.0)
    return z


def embed_forward(x, sel, We, be=None, standardise=True):
    """x [B, N, L], sel [n'] -> xs [B, n', d] = z We (+ be)."""
    z = kept_windows(x, sel, standardise)
    We = np.asarray(We, dtype=np.float64)
    B, n, L = z.shape
    xs = np.zeros((B, n, We.shape[1]))
    for b in range(B):
        for i in range(n):
            acc = np.zeros(We.shape[1])
            for t in range(L):
                acc += z[b, i, t] * We[t]
            xs[b, i] = acc
    if be is not None:
        xs = xs + np.asarray(be, dtype=np.float64)
    return xs


def embed_backward(x, sel, dxs, standardise=True):
    """Gradients of sum(xs * dxs): dWe[t, :] = sum_{b,i} z[b, i, t] dxs[b, i, :], dbe = sum_{b,i} dxs[b, i, :]."""
    z = kept_windows(x, sel, standardise)
    dxs = np.asarray(dxs, dtype=np.float64)
    B, n, L = z.shape
    dWe = np.zeros((L, dxs.shape[-1]))
    for b in range(B):
        for i in range(n):
            dWe += np.outer(z[b, i], dxs[b, i])
    dbe = dxs.sum(axis=(0, 1))
    return dWe, dbe
