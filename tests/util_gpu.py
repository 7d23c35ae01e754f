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


# Element-wise bounds for the attention tensors, relative to the RMS of the oracle's tensor rather than to its largest
# element.  bf16: every intermediate (Q, K, V, P, O, y; dO, dP, dS, dQ, dK, dV, the gradients) is rounded to 8
# significant bits, a relative error of at most 2^-9 on every term of the sums that follow; per stage that is about
# 2^-9 / sqrt(3) = 1.1e-3 of the result's RMS, six to eight stages in quadrature 3-4e-3 (measured 2.2e-3 .. 4.6e-3, and
# 8.9e-3 for the two-token case whose score gradients nearly cancel), and the worst of ~10^6 elements lies 5-6 sigma
# out (measured up to 3.7e-2 of the RMS, 6.5e-2 with two tokens).  fp32: 4e-7 and 3e-6 measured.
#   rms(gpu - oracle) <= RMS_TOL * rms(oracle)   and   |gpu - oracle|_i <= ELEM_REL * |oracle_i| + ELEM_ABS * rms(oracle)
RMS_TOL = {"bf16": 1.5e-2, "fp32": 4e-6}
ELEM_REL = {"bf16": 2.0 ** -7, "fp32": 1e-6}
ELEM_ABS = {"bf16": 8e-2, "fp32": 3e-5}


def elem_err(got, want, dtype):
    """(rms(diff) / rms(want) / RMS_TOL, max_i |diff_i| / (ELEM_REL |want_i| + ELEM_ABS rms(want))): both must be <= 1.
    None for a tensor that is identically zero in the oracle (no scale of its own)."""
    got = got.detach().float().cpu().numpy().astype(np.float64) if isinstance(got, torch.Tensor) else np.asarray(got)
    rms = float(np.sqrt(np.mean(want * want)))
    if rms == 0.0:
        return None
    diff = np.abs(got - want)
    return (float(np.sqrt(np.mean(diff * diff))) / rms / RMS_TOL[dtype],
            float((diff / (ELEM_REL[dtype] * np.abs(want) + ELEM_ABS[dtype] * rms)).max()))


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
