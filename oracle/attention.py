"""Gather of the kept variate tokens and multi-head scaled dot-product attention
(Eq. 3: softmax(Q K^T / sqrt(d_k)) V), forward and backward, in fp64.
Test infrastructure.

Conventions (the paper prints the single-head formula only): tokens are rows,
projections are y = x W with W [d, d] (+ optional bias), the model width d is
cut into H contiguous chunks of d_k = d/H, one per head; no mask, no dropout.
The backward is the analytic derivative of exactly that expression.
"""
import numpy as np


def gather(tokens, sel):
    """xs[b, i, :] = tokens[b, sel[i], :]."""
    return np.asarray(tokens)[:, np.asarray(sel, dtype=np.int64), :]


def scatter_add(dxs, sel, N):
    """Adjoint of gather: zeros at dropped variates."""
    B, _, d = dxs.shape
    out = np.zeros((B, N, d), dtype=dxs.dtype)
    out[:, np.asarray(sel, dtype=np.int64), :] = dxs
    return out


def _split(t, H):
    B, n, d = t.shape
    return t.reshape(B, n, H, d // H).transpose(0, 2, 1, 3)      # [B, H, n, dk]


def _merge(t):
    B, H, n, dk = t.shape
    return t.transpose(0, 2, 1, 3).reshape(B, n, H * dk)


def mha_forward(xs, Wq, Wk, Wv, Wo, H, bq=None, bk=None, bv=None, bo=None):
    """Returns (y [B, n, d], cache) with cache holding what the backward needs."""
    xs, Wq, Wk, Wv, Wo = (np.asarray(a, dtype=np.float64) for a in (xs, Wq, Wk, Wv, Wo))
    d = xs.shape[-1]
    if d % H:
        raise ValueError("d must be a multiple of H")
    dk = d // H
    q = xs @ Wq
    k = xs @ Wk
    v = xs @ Wv
    if bq is not None:
        q = q + np.asarray(bq, dtype=np.float64)
    if bk is not None:
        k = k + np.asarray(bk, dtype=np.float64)
    if bv is not None:
        v = v + np.asarray(bv, dtype=np.float64)
    qh, kh, vh = _split(q, H), _split(k, H), _split(v, H)
    s = np.einsum("bhid,bhjd->bhij", qh, kh) / np.sqrt(float(dk))
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    p = e / e.sum(axis=-1, keepdims=True)
    oh = np.einsum("bhij,bhjd->bhid", p, vh)
    o = _merge(oh)
    y = o @ Wo
    if bo is not None:
        y = y + np.asarray(bo, dtype=np.float64)
    cache = dict(xs=xs, Wq=Wq, Wk=Wk, Wv=Wv, Wo=Wo, H=H, qh=qh, kh=kh, vh=vh, p=p, o=o)
    return y, cache


def mha_backward(dy, cache):
    """Gradients of sum(dy * y).  Returns dict dxs, dWq, dWk, dWv, dWo, dbq, dbk, dbv, dbo."""
    dy = np.asarray(dy, dtype=np.float64)
    xs, Wq, Wk, Wv, Wo, H = (cache[n] for n in ("xs", "Wq", "Wk", "Wv", "Wo", "H"))
    qh, kh, vh, p, o = (cache[n] for n in ("qh", "kh", "vh", "p", "o"))
    d = xs.shape[-1]
    dk = d // H
    flat = lambda t: t.reshape(-1, d)
    dWo = flat(o).T @ flat(dy)
    dbo = flat(dy).sum(axis=0)
    do = dy @ Wo.T
    doh = _split(do, H)
    dvh = np.einsum("bhij,bhid->bhjd", p, doh)
    dp = np.einsum("bhid,bhjd->bhij", doh, vh)
    ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
    dqh = np.einsum("bhij,bhjd->bhid", ds, kh) / np.sqrt(float(dk))
    dkh = np.einsum("bhij,bhid->bhjd", ds, qh) / np.sqrt(float(dk))
    dq, dk_, dv = _merge(dqh), _merge(dkh), _merge(dvh)
    dWq = flat(xs).T @ flat(dq)
    dWk = flat(xs).T @ flat(dk_)
    dWv = flat(xs).T @ flat(dv)
    dxs = dq @ Wq.T + dk_ @ Wk.T + dv @ Wv.T
    return dict(dxs=dxs, dWq=dWq, dWk=dWk, dWv=dWv, dWo=dWo,
                dbq=flat(dq).sum(axis=0), dbk=flat(dk_).sum(axis=0),
                dbv=flat(dv).sum(axis=0), dbo=dbo)
