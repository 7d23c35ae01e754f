"""Shared helpers of the GPU parity tests (not a test module)."""
import functools

import numpy as np
import torch

import workloads as wl
from oracle import attention as o_attn
from oracle import kdfh as o_kdfh
from oracle import sampling as o_samp

TOL = {"bf16": 2e-2, "fp32": 1e-5}      # max|gpu - oracle| / max|oracle|, per tensor
SEED, STEP = 0x5EED5EED1234, 7


def torch_dtype(name):
    return torch.bfloat16 if name == "bf16" else torch.float32


def to_dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return t if dtype is None else t.to(dtype)


def rel_err(got, want):
    got = got.detach().float().cpu().numpy().astype(np.float64) if isinstance(got, torch.Tensor) else np.asarray(got)
    scale = np.abs(want).max()
    return float(np.abs(got - want).max() / (scale if scale > 0 else 1.0))


@functools.lru_cache(maxsize=None)
def workload_inputs(name, screened=True):
    """Windows of a workload, screened with the oracle's amplitude-gap rule, plus the oracle's k-DFH output."""
    w = wl.WORKLOADS[name]
    accept = None
    if screened:
        accept = lambda x: o_kdfh.gap_ok(o_kdfh.batch_mean(o_kdfh.amplitudes(x, 1, w.eps)), w.k)
    x, info = wl.make_signals(w, seed=0, accept=accept)
    topk, hsh, abar = o_kdfh.kdfh(x, w.k)
    return w, x, info, topk, hsh, abar


@functools.lru_cache(maxsize=None)
def workload_selection(name):
    w, x, info, topk, hsh, abar = workload_inputs(name)
    gid, sel, G = o_samp.stratified_sample(hsh, 0, w.ratio[0], w.ratio[1], SEED, STEP)
    return gid, sel, G


def oracle_attention(xs, W, H, dy, biases=(None, None, None, None)):
    """Oracle forward + backward, one batch element at a time (weight gradients summed over the batch)."""
    B = xs.shape[0]
    ys, dxs = [], []
    acc = None
    for b in range(B):
        y, cache = o_attn.mha_forward(xs[b:b + 1], *W, H, *biases)
        g = o_attn.mha_backward(dy[b:b + 1], cache)
        ys.append(y)
        dxs.append(g.pop("dxs"))
        if acc is None:
            acc = g
        else:
            for key in acc:
                acc[key] = acc[key] + g[key]
    acc["y"] = np.concatenate(ys)
    acc["dxs"] = np.concatenate(dxs)
    return acc
