"""Seeded synthetic inputs shaped like the paper's workloads.

This module only makes inputs: periodic multivariate windows, token embeddings,
projection weights and upstream gradients.  It holds none of the method's
arithmetic (no spectrum, no ranking, no hashing, no sampling, no attention) and
is the one module that both the CPU oracle's tests and the GPU path's tests and
benchmark draw from.

The paper evaluates on Electricity (321 variates), Traffic (862), Weather and
Solar-Energy with lookback 96 and batch 32 (App. D, App. E).  Those datasets are
not available here; the generators below stand in for them with sums of
sinusoids at daily / half-daily / weekly periods (hourly sampling), per-variate
scale and phase, additive Gaussian noise, and most variates drawn from a small
set of shared templates so that groups of redundant variates exist.

Signal model for variate n at absolute time tau:
    s_n(tau) = c_n + scale_n * ( sum_m A_nm sin(2 pi tau / p_nm + phi_nm) + sigma * noise )
Window b of a batch covers tau_b .. tau_b + L - 1 with tau_b uniform in [0, 10 L).
A template fixes the periods and a well separated amplitude vector (adjacent
ratios >= 1.25); phases, scale and offset are per variate; noise is fresh per
(window, variate, time).
"""
from dataclasses import dataclass
import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    N: int
    L: int
    k: int
    ratio: tuple          # per-group keep ratio (num, den)
    d: int
    H: int
    dtype: str            # "fp32" or "bf16": arithmetic type of tokens / weights
    periods: tuple        # candidate periods (in samples)
    n_templates: int
    template_frac: float  # fraction of variates that follow a template
    sigma: float
    amp: tuple            # amplitude range U(lo, hi)
    scale: tuple = ("const", 1.0, 1.0)   # ("uniform"|"loguniform"|"const", lo, hi)
    minmax: bool = False  # rescale each variate to [0, 1] before adding noise
    noise_frac: float = 0.0   # fraction of variates that are pure noise
    n_sin: tuple = (1, 3)     # sinusoids per template (inclusive range)
    key: int = 0

    @property
    def eps(self):
        R = self.L // 2 + 1
        return (R + 1) // 2


WORKLOADS = {
    "tiny": Workload("tiny", B=4, N=32, L=96, k=3, ratio=(1, 4), d=64, H=2, dtype="fp32",
                     periods=(24.0, 12.0, 168.0 / 7.0, 8.0), n_templates=4, template_frac=1.0,
                     sigma=0.05, amp=(0.5, 2.0), n_sin=(3, 3), key=1),
    "electricity": Workload("electricity", B=32, N=321, L=96, k=3, ratio=(1, 5), d=512, H=8, dtype="bf16",
                            periods=(24.0, 168.0, 12.0, 8.0, 6.0), n_templates=20, template_frac=0.8,
                            sigma=0.1, amp=(0.5, 2.0), scale=("uniform", 0.1, 10.0), n_sin=(3, 4), key=2),
    "traffic": Workload("traffic", B=32, N=862, L=96, k=3, ratio=(1, 10), d=512, H=8, dtype="bf16",
                        periods=(24.0, 12.0, 168.0, 8.0, 6.0), n_templates=30, template_frac=0.95,
                        sigma=0.02, amp=(0.5, 2.0), minmax=True, n_sin=(3, 4), key=3),
    "long": Workload("long", B=16, N=2048, L=336, k=4, ratio=(1, 10), d=512, H=8, dtype="bf16",
                     periods=(24.0, 48.0, 168.0, 336.0 / 2.0, 12.0, 8.0, 84.0, 56.0), n_templates=64,
                     template_frac=1.0, sigma=0.1, amp=(0.5, 3.0), n_sin=(4, 5), key=4),
    "stress": Workload("stress", B=8, N=8192, L=512, k=5, ratio=(1, 20), d=768, H=12, dtype="bf16",
                       periods=tuple(float(p) for p in range(4, 257)), n_templates=256, template_frac=1.0,
                       sigma=0.1, amp=(0.5, 2.0), scale=("loguniform", 0.01, 100.0),
                       noise_frac=0.1, n_sin=(5, 6), key=5),
}
ORDER = ("tiny", "electricity", "traffic", "long", "stress")


def _rng(w, seed, *stream):
    return np.random.default_rng([0x5EED0000 + w.key, int(seed), *[int(s) for s in stream]])


def _separated_amplitudes(rng, m, lo, hi):
    """m amplitudes, descending, adjacent ratio >= 1.25, the largest in [lo, hi]."""
    a = [rng.uniform(lo, hi)]
    for _ in range(1, m):
        a.append(a[-1] / rng.uniform(1.25, 1.8))
    return np.asarray(a)


def _templates(w, seed):
    rng = _rng(w, seed, 1)
    distinct = sorted(set(w.periods))
    out = []
    seen = set()
    for _ in range(w.n_templates):
        for _attempt in range(32):               # prefer templates whose ordered period tuples differ
            m = int(rng.integers(w.n_sin[0], min(w.n_sin[1], len(distinct)) + 1))
            per = rng.choice(np.asarray(distinct), size=m, replace=False)
            if tuple(per.tolist()) not in seen:
                break
        seen.add(tuple(per.tolist()))
        out.append((per, _separated_amplitudes(rng, m, *w.amp)))
    return out


def _draw_scale(w, rng, n):
    kind, lo, hi = w.scale
    if kind == "uniform":
        return rng.uniform(lo, hi, size=n)
    if kind == "loguniform":
        return np.exp(rng.uniform(np.log(lo), np.log(hi), size=n))
    return np.full(n, float(lo))


def make_signals(w, seed=0, accept=None, max_tries=64):
    """Windows x float32 [B, N, L] plus bookkeeping.

    accept: optional callable(x float32 [B, n, L]) -> bool [n]; variates it
    rejects get fresh noise (next noise stream) up to max_tries times.  The
    caller decides what "acceptable" means (the tests pass a screen on the
    separation of the leading amplitudes); this module does not look at spectra.
    Returns (x, info) with info = dict(template [N] (-1: none, -2: pure noise),
    redrawn: number of variates whose noise was redrawn, unresolved: still rejected).
    """
    B, N, L = w.B, w.N, w.L
    templates = _templates(w, seed)
    rng = _rng(w, seed, 2)
    tau0 = rng.integers(0, 10 * L, size=B)
    tau = tau0[:, None] + np.arange(L)[None, :]                       # [B, L]
    n_noise = int(round(w.noise_frac * N))
    n_tmpl = int(round(w.template_frac * (N - n_noise)))
    kind = np.full(N, -1, dtype=np.int64)
    perm = rng.permutation(N)
    kind[perm[:n_noise]] = -2
    kind[perm[n_noise:n_noise + n_tmpl]] = rng.integers(0, len(templates), size=n_tmpl)
    scale = _draw_scale(w, rng, N)
    offset = np.zeros(N)
    distinct = sorted(set(w.periods))
    clean = np.zeros((B, N, L))
    for n in range(N):
        if kind[n] == -2:
            continue
        if kind[n] >= 0:
            per, amp = templates[kind[n]]
        else:
            m = int(rng.integers(w.n_sin[0], min(w.n_sin[1], len(distinct)) + 1))
            per = rng.choice(np.asarray(distinct), size=m, replace=False)
            amp = _separated_amplitudes(rng, m, *w.amp)
        phi = rng.uniform(0.0, 2.0 * np.pi, size=len(per))
        for p, a, ph in zip(per, amp, phi):
            clean[:, n, :] += a * np.sin(2.0 * np.pi * tau / p + ph)
    if w.minmax:
        lo = clean.min(axis=(0, 2), keepdims=True)
        hi = clean.max(axis=(0, 2), keepdims=True)
        span = np.where(hi > lo, hi - lo, 1.0)
        clean = (clean - lo) / span
        scale = np.ones(N)

    def noisy(idx, attempt):
        out = np.empty((B, len(idx), L))
        for j, n in enumerate(idx):
            g = _rng(w, seed, 3, n, attempt)
            out[:, j, :] = offset[n] + scale[n] * (clean[:, n, :] + w.sigma * g.standard_normal((B, L)))
        return out.astype(np.float32)

    x = noisy(np.arange(N), 0)
    redrawn = 0
    unresolved = 0
    if accept is not None:
        bad = np.nonzero(~np.asarray(accept(x), dtype=bool))[0]
        redrawn = len(bad)
        attempt = 1
        while len(bad) and attempt < max_tries:
            x[:, bad, :] = noisy(bad, attempt)
            still = ~np.asarray(accept(x[:, bad, :]), dtype=bool)
            bad = bad[still]
            attempt += 1
        unresolved = len(bad)
    return x, dict(template=kind, redrawn=redrawn, unresolved=unresolved, tau0=tau0)


def round_bf16(a):
    """Round float64/float32 values to the nearest bfloat16 (ties to even), returned as float32."""
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    u = a32.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a32.shape)


def quantise(a, dtype):
    """Values representable in the workload's arithmetic type, as float32."""
    if dtype == "bf16":
        return round_bf16(a)
    return np.ascontiguousarray(a, dtype=np.float32)


def make_tokens(w, x, seed=0):
    """Variate tokens float32 [B, N, d] (already representable in w.dtype).

    A seeded shared linear embedding R^L -> R^d of each window after per-window
    standardisation (zero mean, unit variance over time), which is what the
    variate-tokenised backbone the paper builds on does before embedding.
    """
    rng = _rng(w, seed, 4)
    We = rng.standard_normal((w.L, w.d)) / np.sqrt(w.L)
    be = 0.1 * rng.standard_normal(w.d)
    xd = x.astype(np.float64)
    mu = xd.mean(axis=-1, keepdims=True)
    sd = xd.std(axis=-1, keepdims=True)
    z = (xd - mu) / np.where(sd > 0, sd, 1.0)
    tok = z.reshape(-1, w.L) @ We + be
    return quantise(tok.reshape(w.B, w.N, w.d), w.dtype)


def make_weights(w, seed=0):
    """Wq, Wk, Wv, Wo float32 [d, d], entries N(0, 1/d), representable in w.dtype."""
    rng = _rng(w, seed, 5)
    return tuple(quantise(rng.standard_normal((w.d, w.d)) / np.sqrt(w.d), w.dtype) for _ in range(4))


def make_biases(w, seed=0):
    rng = _rng(w, seed, 7)
    return tuple(quantise(0.1 * rng.standard_normal(w.d), w.dtype) for _ in range(4))


def make_upstream(w, n_sel, seed=0):
    """dy float32 [B, n_sel, d], N(0, 1), representable in w.dtype."""
    rng = _rng(w, seed, 6)
    return quantise(rng.standard_normal((w.B, n_sel, w.d)), w.dtype)
