"""Pins for the oracle's grouping and stratified sampling (Eq. 1-2, reduction ratio) -- CPU only."""
import itertools
import math

import numpy as np
import pytest

from oracle import philox, sampling
from conftest import read_golden


def random_hashes(rng, N, n_distinct):
    pool = rng.integers(0, 2 ** 62, size=n_distinct, dtype=np.uint64)
    return pool[rng.integers(0, n_distinct, size=N)]


# ---------------------------------------------------------------- grouping
def test_grouping_against_brute_force_equality():
    rng = np.random.default_rng(1)
    h = random_hashes(rng, 60, 9)
    gid, G = sampling.group_ids(h)
    for a in range(60):
        for b in range(60):
            assert (gid[a] == gid[b]) == (h[a] == h[b])
    assert sorted(set(gid.tolist())) == list(range(G))                # dense
    for a in range(60):
        for b in range(60):
            if h[a] < h[b]:
                assert gid[a] < gid[b]                                # numbered in ascending hash


def test_grouping_handles_large_hash_values():
    h = np.array([2 ** 63 - 1, 5, 2 ** 63 - 2, 5], dtype=np.uint64)   # would lose bits in float64
    gid, G = sampling.group_ids(h)
    assert G == 3 and gid.tolist() == [2, 0, 1, 0]


# ---------------------------------------------------------------- retained counts (Eq. 1)
@pytest.mark.parametrize("gs", [1, 5, 10, 20])
def test_counts_follow_eq_1(gs):
    rng = np.random.default_rng(gs)
    h = random_hashes(rng, 300, 17)
    gid, sel, G = sampling.stratified_sample(h, gs, 1, 1, seed=3, step=4)
    sizes = np.bincount(gid, minlength=G)
    kept = np.bincount(gid[sel], minlength=G)
    assert kept.tolist() == [min(int(g), gs) for g in sizes]
    assert len(sel) == sum(min(int(g), gs) for g in sizes)            # S is the union (Eq. 2)
    assert np.all(kept >= 1)
    delta = sampling.reduction_ratio(300, len(sel))
    assert delta == pytest.approx(1 - sum(min(int(g), gs) for g in sizes) / 300)


def test_gs_one_keeps_one_per_group_and_large_gs_keeps_all():
    rng = np.random.default_rng(9)
    h = random_hashes(rng, 200, 23)
    gid, sel, G = sampling.stratified_sample(h, 1, 1, 1, 0, 0)
    assert len(sel) == G and sorted(gid[sel].tolist()) == list(range(G))
    _, sel, _ = sampling.stratified_sample(h, 10 ** 6, 1, 1, 0, 0)
    assert sel.tolist() == list(range(200))
    _, sel, _ = sampling.stratified_sample(h, 0, 1, 1, 0, 0)          # no cap, ratio off
    assert sel.tolist() == list(range(200))


@pytest.mark.parametrize("num,den", [(1, 4), (1, 5), (1, 10), (1, 20), (3, 7)])
def test_keep_ratio_rule(num, den):
    for g in range(1, 200):
        n_i = sampling.keep_count(g, 0, num, den)
        assert n_i == max(1, math.ceil(g * num / den - 1e-12)) and 1 <= n_i <= g
        assert sampling.keep_count(g, 3, num, den) == min(n_i, 3)
    rng = np.random.default_rng(den)
    h = random_hashes(rng, 500, 31)
    gid, sel, G = sampling.stratified_sample(h, 0, num, den, 5, 6)
    sizes = np.bincount(gid, minlength=G)
    kept = np.bincount(gid[sel], minlength=G)
    assert kept.tolist() == [sampling.keep_count(int(g), 0, num, den) for g in sizes]


def test_keep_count_rejects_bad_ratios():
    for num, den in [(2, 1), (1, 0), (-1, 3)]:
        with pytest.raises(ValueError):
            sampling.keep_count(5, 0, num, den)


def test_reduction_ratio_reproduces_table_3():
    rows = [line.split()[1:] for line in read_golden("paper_facts.txt") if line.startswith("delta")]
    assert len(rows) == 4
    for used, n, pct in rows:
        assert 100 * sampling.reduction_ratio(int(n), float(used)) == pytest.approx(float(pct), abs=0.03)


# ---------------------------------------------------------------- which members are retained
def test_selection_against_brute_force_rank_counting():
    rng = np.random.default_rng(2)
    N = 80
    h = random_hashes(rng, N, 6)
    seed, step = 0xDEADBEEFCAFE, 2 ** 40 + 17
    gid, sel, G = sampling.stratified_sample(h, 4, 1, 2, seed, step)
    u = []
    for n in range(N):                                               # keys straight from the scalar generator
        r = philox.philox4x32_10((n, 0, step & 0xFFFFFFFF, step >> 32), (seed & 0xFFFFFFFF, seed >> 32))
        u.append((r[0] << 32) | r[1])
    want = []
    for n in range(N):
        members = [m for m in range(N) if h[m] == h[n]]
        rank = sum(1 for m in members if (u[m], m) < (u[n], n))
        if rank < min(4, max(1, -(-len(members) // 2))):
            want.append(n)
    assert sel.tolist() == want
    assert sel.tolist() == sorted(set(sel.tolist()))                  # ascending, no repeats


def test_selection_depends_on_seed_and_step_only():
    h = random_hashes(np.random.default_rng(4), 120, 5)
    a = sampling.stratified_sample(h, 3, 1, 1, 1, 1)[1]
    assert np.array_equal(a, sampling.stratified_sample(h, 3, 1, 1, 1, 1)[1])
    assert not np.array_equal(a, sampling.stratified_sample(h, 3, 1, 1, 1, 2)[1])
    assert not np.array_equal(a, sampling.stratified_sample(h, 3, 1, 1, 2, 1)[1])


def test_random_sampling_is_uniform_over_subsets():
    # one group of 5 and one of 3, keep 2 of each: all C(5,2)=10 and C(3,2)=3 subsets equally likely
    h = np.array([7, 7, 9, 7, 9, 7, 9, 7], dtype=np.uint64)
    g5 = [0, 1, 3, 5, 7]
    g3 = [2, 4, 6]
    c5 = {s: 0 for s in itertools.combinations(g5, 2)}
    c3 = {s: 0 for s in itertools.combinations(g3, 2)}
    trials = 6000
    for step in range(trials):
        sel = sampling.stratified_sample(h, 2, 1, 1, seed=12345, step=step)[1].tolist()
        c5[tuple(n for n in sel if n in g5)] += 1
        c3[tuple(n for n in sel if n in g3)] += 1
    chi5 = sum((c - trials / 10) ** 2 / (trials / 10) for c in c5.values())
    chi3 = sum((c - trials / 3) ** 2 / (trials / 3) for c in c3.values())
    assert chi5 < 33.7      # chi-square, 9 dof, p = 1e-4
    assert chi3 < 18.4      # 2 dof, p = 1e-4
    member = np.zeros(8)
    for s, c in c5.items():
        for n in s:
            member[n] += c
    assert np.allclose(member[g5] / trials, 2 / 5, atol=0.03)         # membership probability n_i/g


# ---------------------------------------------------------------- deterministic representatives
def spectra(rng, N, F, n_distinct):
    """Hashes with n_distinct groups and spectra that scatter around one centre per group."""
    h = random_hashes(rng, N, n_distinct)
    centres = {int(v): rng.uniform(0.5, 5.0, F) for v in set(h.tolist())}
    A = np.stack([centres[int(v)] + 0.2 * rng.standard_normal(F) for v in h])
    return h, np.abs(A)


def test_representative_is_the_member_closest_to_the_group_mean():
    """gs = 1: brute force in float64 over every group, wherever the two best candidates are clearly apart."""
    rng = np.random.default_rng(21)
    h, A = spectra(rng, 120, 9, 11)
    gid, sel, G = sampling.representative_sample(h, A, 1, 1, 1)
    assert len(sel) == G
    for g in range(G):
        members = np.nonzero(gid == g)[0]
        mean = A[members].mean(axis=0)
        d = ((A[members] - mean) ** 2).sum(axis=1)
        order = np.argsort(d, kind="stable")
        if len(members) == 1 or d[order[1]] - d[order[0]] > 1e-4 * d[order[1]]:
            assert members[order[0]] in sel
        assert len(set(members.tolist()) & set(sel.tolist())) == 1


@pytest.mark.parametrize("gs,num,den", [(0, 1, 4), (3, 1, 1), (2, 1, 2), (0, 1, 1)])
def test_representative_counts_and_order(gs, num, den):
    rng = np.random.default_rng(22)
    h, A = spectra(rng, 200, 6, 17)
    gid, sel, G = sampling.representative_sample(h, A, gs, num, den)
    assert np.all(np.diff(sel) > 0)
    for g in range(G):
        members = np.nonzero(gid == g)[0]
        kept = [n for n in members if n in set(sel.tolist())]
        assert len(kept) == sampling.keep_count(len(members), gs, num, den)
        # the kept members are the closest ones: no dropped member is strictly closer than a kept one
        d = sampling.spectrum_distances(A, gid, G)
        dropped = [n for n in members if n not in kept]
        if dropped:
            assert max(d[n] for n in kept) <= min(d[n] for n in dropped)


def test_representative_ties_go_to_the_lower_index_and_scaling_is_irrelevant():
    h = np.array([7, 7, 7, 7, 9, 9], dtype=np.uint64)
    A = np.array([[1.0, 2.0]] * 4 + [[3.0, 1.0], [5.0, 1.0]])          # identical members; a pair equidistant from its mean
    gid, sel, G = sampling.representative_sample(h, A, 2, 1, 1)
    assert sel.tolist() == [0, 1, 4, 5]
    gid, sel, G = sampling.representative_sample(h, A, 1, 1, 1)
    assert sel.tolist() == [0, 4]
    rng = np.random.default_rng(23)
    h, A = spectra(rng, 90, 5, 8)
    base = sampling.representative_sample(h, A.astype(np.float32), 2, 1, 1)[1]
    for p in (-3, 4):                                                   # a power of two scales every float32 operation exactly
        assert np.array_equal(sampling.representative_sample(h, (A.astype(np.float32) * np.float32(2.0 ** p)), 2, 1, 1)[1], base)


def test_distances_hand_computed_example():
    """Two groups; every number below is worked out by hand from the definition."""
    h = np.array([5, 9, 5, 5, 9], dtype=np.uint64)
    A = np.array([[1.0, 2.0], [10.0, 0.0], [3.0, 2.0], [2.0, 5.0], [10.0, 4.0]])
    gid, G = sampling.group_ids(h)
    # group of hash 5 = variates 0, 2, 3: mean (2, 3); distances 1 + 1, 1 + 1, 0 + 4
    # group of hash 9 = variates 1, 4: mean (10, 2); distances 4, 4
    assert sampling.spectrum_distances(A, gid, G).tolist() == [2.0, 4.0, 2.0, 4.0, 4.0]
    assert sampling.representative_sample(h, A, 1, 1, 1)[1].tolist() == [0, 1]        # ties: the lower index
    assert sampling.representative_sample(h, A, 2, 1, 1)[1].tolist() == [0, 1, 2, 4]


def test_distances_brute_force_and_variance_identity():
    """Pure-Python loops over a small input, and sum_{n in g} d[n] = sum_f (sum_n a^2 - |g| mean_f^2)."""
    rng = np.random.default_rng(24)
    h, A = spectra(rng, 60, 7, 6)
    gid, G = sampling.group_ids(h)
    d = sampling.spectrum_distances(A, gid, G)
    for n in range(60):
        members = [m for m in range(60) if gid[m] == gid[n]]
        want = 0.0
        for f in range(7):
            mean = sum(float(A[m, f]) for m in members) / len(members)
            want += (float(A[n, f]) - mean) ** 2
        assert abs(d[n] - want) <= 1e-12 * max(want, 1.0)
    for g in range(G):
        members = np.nonzero(gid == g)[0]
        total = sum(float(A[m, f]) ** 2 for m in members for f in range(7))
        total -= len(members) * sum((sum(float(A[m, f]) for m in members) / len(members)) ** 2 for f in range(7))
        assert abs(d[members].sum() - total) <= 1e-10 * max(total, 1.0)


def test_distances_invariances_and_special_cases():
    rng = np.random.default_rng(25)
    h, A = spectra(rng, 80, 5, 9)
    gid, G = sampling.group_ids(h)
    d = sampling.spectrum_distances(A, gid, G)
    # a shift common to all members of a group moves its mean along: distances unchanged
    shift = rng.uniform(1.0, 2.0, (G, 5))
    assert np.allclose(sampling.spectrum_distances(A + shift[gid], gid, G), d, rtol=1e-9, atol=1e-12)
    # a permutation of the variates permutes the distances
    perm = rng.permutation(80)
    gid_p, _ = sampling.group_ids(h[perm])
    assert np.allclose(sampling.spectrum_distances(A[perm], gid_p, G), d[perm], rtol=1e-12, atol=0)
    # a group of one, and a group of identical members, sit on their mean
    h1 = np.array([3, 4, 4, 4], dtype=np.uint64)
    A1 = np.array([[1.5, 2.5], [0.25, 0.75], [0.25, 0.75], [0.25, 0.75]])
    assert sampling.spectrum_distances(A1, *sampling.group_ids(h1)).tolist() == [0.0, 0.0, 0.0, 0.0]
    # float32 inputs are taken exactly: the same values as float64 give the same distances
    A32 = A.astype(np.float32)
    assert np.array_equal(sampling.spectrum_distances(A32, gid, G), sampling.spectrum_distances(A32.astype(np.float64), gid, G))
