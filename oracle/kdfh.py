"""k-dominant frequency hashing (Alg. 1, Def. 1) in fp64.  Test infrastructure.

Steps, in the algorithm's order:
  1. amplitude spectrum of every (window, variate) series  -- Alg. 1 step 1
  2. keep only the candidate bins f_min..f_max (low-pass)   -- Alg. 1 step 2
  3. mean of the amplitudes over the batch                  -- Alg. 1 step 3
  4. the k largest bins, ranked by descending amplitude     -- Alg. 1 step 4, Def. 1
  5. a hash of that ordered tuple                           -- Alg. 1 step 5

Readings of what the paper leaves open (conventions of this repository):
  * bin 0 (the mean) is not a candidate: the printed hash of a flat variate is
    "1-2-3" (App. G text), so the default first candidate is bin 1;
  * the cut-off is a count of candidate bins ("there are epsilon frequencies in
    the averaged spectrum", complexity paragraph); epsilon = 25 for T = 96,
    "half the number of positive frequencies" (App. E), generalised as
    ceil((floor(L/2)+1)/2);
  * amplitudes are unnormalised |X_f|; the mean is a mean of amplitudes;
  * equal amplitudes rank the lower bin first;
  * the hash is the ordered tuple written in radix R = floor(L/2)+1, first
    rank most significant, so equal tuples <=> equal hashes and "4-12-8" and
    "12-4-8" (Fig. 5 text) differ.
"""
import numpy as np


def num_bins(L):
    """R: number of bins of a real DFT of length L."""
    return L // 2 + 1


def default_cutoff(L):
    """epsilon: half the non-negative-frequency bins, rounded up (25 at L = 96, App. E)."""
    R = num_bins(L)
    return (R + 1) // 2


def dft(x, bins):
    """Real and imaginary part of X_f = sum_t x[t] exp(-2 pi i f t / L) for f in bins.

    x: [..., L] (converted to float64).  Returns (Re, Im), each [..., len(bins)].
    The angle is reduced in integers, (f*t mod L)/L, before cos/sin are taken.
    """
    x = np.asarray(x, dtype=np.float64)
    L = x.shape[-1]
    f = np.asarray(bins, dtype=np.int64)
    t = np.arange(L, dtype=np.int64)
    m = (f[:, None] * t[None, :]) % L                   # [F, L]
    ang = 2.0 * np.pi * m.astype(np.float64) / float(L)
    re = x @ np.cos(ang).T
    im = -(x @ np.sin(ang).T)
    return re, im


def amplitudes(x, f_min, f_max):
    """A[b, n, f - f_min] = |X_f| of window b, variate n, for f_min <= f <= f_max (steps 1-2)."""
    re, im = dft(x, np.arange(f_min, f_max + 1))
    return np.sqrt(re * re + im * im)


def batch_mean(A):
    """Mean over the leading (batch) axis, summed in ascending b (step 3)."""
    acc = np.zeros(A.shape[1:], dtype=np.float64)
    for b in range(A.shape[0]):
        acc = acc + A[b]
    return acc / float(A.shape[0])


def ranked_topk(abar, k, f_min):
    """Step 4: for every variate the k bins of largest mean amplitude, largest first.

    abar: [N, F].  Ties: the lower bin ranks first.  Returns int64 [N, k] of bin indices.
    """
    N, F = abar.shape
    if not 1 <= k <= F:
        raise ValueError("k must lie in 1..number of candidate bins")
    out = np.empty((N, k), dtype=np.int64)
    f = np.arange(F)
    for n in range(N):
        order = sorted(f.tolist(), key=lambda j: (-abar[n, j], j))
        out[n] = np.asarray(order[:k]) + f_min
    return out


def hash_values(topk, R):
    """Step 5: sum_j topk[n, j] * R**(k-1-j), as Python-int exact arithmetic, returned uint64."""
    N, k = topk.shape
    if R ** k >= 2 ** 63:
        raise ValueError("R**k must stay below 2**63")
    out = np.empty(N, dtype=np.uint64)
    for n in range(N):
        h = 0
        for j in range(k):
            h = h * R + int(topk[n, j])
        out[n] = h
    return out


def decode_hash(h, k, R):
    """Inverse of hash_values for one hash: the ordered tuple of bins."""
    h = int(h)
    digits = []
    for _ in range(k):
        digits.append(h % R)
        h //= R
    return tuple(reversed(digits))


def kdfh(x, k, f_min=1, f_max=None):
    """Whole of Alg. 1.  x: [B, N, L].  Returns (topk int64 [N,k], hash uint64 [N], abar float64 [N,F])."""
    x = np.asarray(x)
    L = x.shape[-1]
    if f_max is None:
        f_max = default_cutoff(L)
    if not (0 <= f_min <= f_max <= L // 2):
        raise ValueError("candidate bins must satisfy 0 <= f_min <= f_max <= floor(L/2)")
    A = amplitudes(x, f_min, f_max)
    abar = batch_mean(A)
    topk = ranked_topk(abar, k, f_min)
    return topk, hash_values(topk, num_bins(L)), abar


def gap_ok(abar, k, rel=1e-3):
    """Input screen used when comparing an fp32 implementation with this fp64 one.

    True for a variate whose k+1 largest mean amplitudes a_1 >= ... >= a_{k+1}
    satisfy a_j - a_{j+1} >= rel * a_j for j = 1..k, i.e. whose ranked top-k
    cannot change under a perturbation much smaller than rel.
    """
    s = -np.sort(-abar, axis=1)[:, :k + 1]
    if s.shape[1] < k + 1:                       # k == F: only k values exist
        s = np.concatenate([s, np.zeros((s.shape[0], 1))], axis=1)
    return np.all(s[:, :k] - s[:, 1:k + 1] >= rel * s[:, :k], axis=1)
