"""Grouping by hash and stratified sampling (Sec. "Sparse Attention via Stratified
Sampling", Eq. 1-2, and the reduction ratio delta of the following paragraph).
Test infrastructure.

The paper fixes: variates with the same hash form a group G_i; from each group
|S_i| = min(|G_i|, gs) members are retained, chosen at random; S is the union.
Left open by the paper and fixed here as repository conventions:
  * group ids number the distinct hashes in ascending order, from 0;
  * the retained count also supports a per-group keep ratio num/den:
        n_i = min(|G_i|, gs', max(1, ceil(|G_i| * num / den))),
    gs' = gs, or no cap when gs == 0; num/den = 1/1 switches the ratio off and
    leaves Eq. 1 as printed;
  * "random": every variate n draws a 64-bit key u[n] from Philox4x32-10 with
    counter (n, 0, step_lo, step_hi) and key (seed_lo, seed_hi), u = r0<<32 | r1;
    a group keeps its n_i members with the smallest (u[n], n).  Smallest-key
    selection is a uniform sample without replacement;
  * S is listed in ascending variate index;
  * a second, deterministic sampler (the paper: "not limited to any specific sampling
    method"): a group keeps the members whose mean amplitude spectrum is closest to the
    group's mean spectrum (representative_sample below), distances in float64, ties to
    the lower variate index.
"""
import numpy as np

from .philox import philox4x32_10_array


def group_ids(hashes):
    """Dense group id per variate: rank of its hash among the sorted distinct hashes."""
    hashes = np.asarray(hashes, dtype=np.uint64)
    distinct = sorted(set(int(h) for h in hashes))
    rank = {h: i for i, h in enumerate(distinct)}
    gid = np.asarray([rank[int(h)] for h in hashes], dtype=np.int64)
    return gid, len(distinct)


def keep_count(g, gs, num, den):
    """Members retained from a group of size g (Eq. 1 with the optional keep ratio)."""
    if den <= 0 or num < 0 or num > den:
        raise ValueError("keep ratio must satisfy 0 <= num <= den, den > 0")
    by_ratio = max(1, (g * num + den - 1) // den)
    n_i = min(g, by_ratio)
    if gs > 0:
        n_i = min(n_i, gs)
    return n_i


def random_keys(N, seed, step):
    """u[n] for n = 0..N-1 as uint64."""
    seed = int(seed)
    step = int(step)
    n = np.arange(N, dtype=np.uint64)
    r0, r1, _, _ = philox4x32_10_array(n, 0, step & 0xFFFFFFFF, (step >> 32) & 0xFFFFFFFF,
                                       seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    return (r0 << np.uint64(32)) | r1


def stratified_sample(hashes, gs, num, den, seed, step):
    """Returns (group_id int64 [N], sel int64 [N'] ascending, G)."""
    gid, G = group_ids(hashes)
    N = len(gid)
    u = random_keys(N, seed, step)
    kept = []
    for i in range(G):
        members = [n for n in range(N) if gid[n] == i] if N <= 64 else np.nonzero(gid == i)[0].tolist()
        n_i = keep_count(len(members), gs, num, den)
        members.sort(key=lambda n: (int(u[n]), n))
        kept.extend(members[:n_i])
    sel = np.asarray(sorted(kept), dtype=np.int64)
    return gid, sel, G


def reduction_ratio(N, n_sel):
    """delta = 1 - N'/N."""
    return 1.0 - float(n_sel) / float(N)


def spectrum_distances(abar, gid, G):
    """Squared Euclidean distance of every variate's mean amplitude spectrum to the mean spectrum of its group:

        mean_g[f] = (1 / |g|) sum_{n in g} abar[n, f],      d[n] = sum_f (abar[n, f] - mean_{gid[n]}[f])^2,

    the plain definition in float64 (the inputs are converted exactly).  Returns d as float64 [N].
    """
    A = np.asarray(abar, dtype=np.float64)
    gid = np.asarray(gid)
    d = np.zeros(A.shape[0], dtype=np.float64)
    for g in range(G):
        members = np.nonzero(gid == g)[0]
        mean = A[members].sum(axis=0) / float(len(members))
        d[members] = ((A[members] - mean) ** 2).sum(axis=1)
    return d


def representative_sample(hashes, abar, gs, num, den):
    """Deterministic per-group sampler (Sec. 3.3 leaves the sampling method open): a group keeps the members whose
    spectrum lies closest to the group's mean spectrum, ties to the lower variate index.
    Returns (group_id int64 [N], sel int64 [N'] ascending, G)."""
    gid, G = group_ids(hashes)
    N = len(gid)
    d = spectrum_distances(abar, gid, G)
    kept = []
    for i in range(G):
        members = np.nonzero(gid == i)[0].tolist()
        n_i = keep_count(len(members), gs, num, den)
        members.sort(key=lambda n: (float(d[n]), n))
        kept.extend(members[:n_i])
    sel = np.asarray(sorted(kept), dtype=np.int64)
    return gid, sel, G

