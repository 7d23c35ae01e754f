"""Pins for the oracle's k-DFH (Alg. 1, Def. 1, Theorem 1) -- CPU only.

Each test checks the oracle against something fixed outside of it: a closed
form, an identity, a library routine, or a fact the paper prints.
"""
import itertools

import numpy as np
import pytest

from oracle import kdfh
from conftest import read_golden


def facts(key):
    return [line.split()[1:] for line in read_golden("paper_facts.txt") if line.split()[0] == key]


def sinusoid(L, A, f, phi):
    t = np.arange(L)
    return A * np.sin(2 * np.pi * f * t / L + phi)


# ---------------------------------------------------------------- spectrum
@pytest.mark.parametrize("L,f0", [(96, 4), (96, 25), (336, 14), (512, 100), (97, 7)])
def test_pure_sinusoid_closed_form(L, f0):
    # x = A sin(2 pi f0 t / L + phi), integer 0 < f0 < L/2  =>  |X_f0| = A L / 2, every other bin 0
    A, phi = 1.7, 0.3
    x = sinusoid(L, A, f0, phi)[None, None, :]
    amp = kdfh.amplitudes(x, 0, L // 2)[0, 0]
    assert amp[f0] == pytest.approx(A * L / 2, rel=1e-12)
    others = np.delete(amp, f0)
    assert np.all(others < 1e-10 * A * L)


def test_dc_and_nyquist_bins():
    L = 96
    x = np.full((1, 1, L), 2.5)
    amp = kdfh.amplitudes(x, 0, L // 2)[0, 0]
    assert amp[0] == pytest.approx(2.5 * L, rel=1e-13)
    assert np.all(amp[1:] < 1e-10)
    alt = ((-1.0) ** np.arange(L))[None, None, :]
    amp = kdfh.amplitudes(alt, 0, L // 2)[0, 0]
    assert amp[L // 2] == pytest.approx(L, rel=1e-13)


@pytest.mark.parametrize("L", [96, 97, 336, 512])
def test_parseval(L):
    rng = np.random.default_rng(L)
    x = rng.standard_normal((2, 3, L))
    amp = kdfh.amplitudes(x, 0, L // 2)
    w = np.full(L // 2 + 1, 2.0)
    w[0] = 1.0
    if L % 2 == 0:
        w[-1] = 1.0
    lhs = (x ** 2).sum(axis=-1)
    rhs = (amp ** 2 * w).sum(axis=-1) / L
    assert np.allclose(lhs, rhs, rtol=1e-12)


@pytest.mark.parametrize("L", [96, 336, 512, 101])
def test_matches_library_rfft_real_and_imaginary(L):
    rng = np.random.default_rng(L + 1)
    x = rng.standard_normal((2, 4, L))
    re, im = kdfh.dft(x, np.arange(0, L // 2 + 1))
    ref = np.fft.rfft(x, axis=-1)
    assert np.allclose(re, ref.real, atol=1e-11)
    assert np.allclose(im, ref.imag, atol=1e-11)          # sign of the imaginary part included


def test_low_pass_keeps_exactly_the_candidate_bins():
    L = 96
    x = np.random.default_rng(0).standard_normal((2, 3, L))
    full = kdfh.amplitudes(x, 0, L // 2)
    part = kdfh.amplitudes(x, 3, 17)
    assert part.shape == (2, 3, 15)
    assert np.allclose(part, full[..., 3:18], rtol=0, atol=1e-12)


def test_default_cutoff_matches_the_paper():
    for L, eps in facts("cutoff"):
        assert kdfh.default_cutoff(int(L)) == int(eps)
    assert kdfh.default_cutoff(336) == 85
    assert kdfh.default_cutoff(512) == 129
    assert kdfh.num_bins(96) == 49 and kdfh.num_bins(97) == 49


# ---------------------------------------------------------------- batch mean
def test_batch_mean_is_a_mean_of_amplitudes_not_the_amplitude_of_a_mean():
    L = 96
    a = sinusoid(L, 1.0, 4, 0.0)
    x = np.stack([a, -a])[:, None, :]                     # two windows in anti-phase
    A = kdfh.amplitudes(x, 1, 25)
    abar = kdfh.batch_mean(A)
    assert abar[0, 3] == pytest.approx(L / 2, rel=1e-12)  # bin 4 survives the average
    assert np.allclose(kdfh.amplitudes(x.mean(axis=0, keepdims=True), 1, 25), 0, atol=1e-10)


def test_batch_mean_value():
    rng = np.random.default_rng(3)
    A = rng.random((5, 4, 7))
    assert np.allclose(kdfh.batch_mean(A), A.sum(axis=0) / 5, rtol=1e-15)


# ---------------------------------------------------------------- ranked top-k and hash
def test_planted_sinusoids_hash_to_their_frequencies_in_amplitude_order():
    L, k = 96, 3
    freqs = (4, 12, 8)
    amps = (3.0, 2.0, 1.0)
    rng = np.random.default_rng(0)
    x = np.zeros((4, 2, L))
    for b in range(4):
        for n in range(2):
            for f, a in zip(freqs, amps):
                x[b, n] += sinusoid(L, a, f, rng.uniform(0, 2 * np.pi))
    topk, h, _ = kdfh.kdfh(x, k)
    assert topk.tolist() == [list(freqs)] * 2
    assert h[0] == h[1] == (4 * 49 + 12) * 49 + 8


def test_order_of_the_dominant_frequencies_distinguishes_hashes():
    L = 96
    for a, b in facts("distinct_hash"):
        ta = tuple(int(v) for v in a.split("-"))
        tb = tuple(int(v) for v in b.split("-"))
        assert sorted(ta) == sorted(tb)
        k = len(ta)
        amps = [2.0 ** (-j) for j in range(k)]
        xs = []
        for tup in (ta, tb):
            xs.append(sum(sinusoid(L, amp, f, 0.1 * f) for f, amp in zip(tup, amps)))
        x = np.stack(xs)[None, :, :]
        topk, h, _ = kdfh.kdfh(x, k)
        assert tuple(topk[0]) == ta and tuple(topk[1]) == tb
        assert h[0] != h[1]
        assert kdfh.decode_hash(h[0], k, 49) == ta and kdfh.decode_hash(h[1], k, 49) == tb


def test_flat_variate_gets_the_lowest_bins():
    (label,) = facts("flat_hash")[0]
    want = [int(v) for v in label.split("-")]
    x = np.zeros((3, 1, 96))
    topk, h, _ = kdfh.kdfh(x, len(want))
    assert topk[0].tolist() == want
    # a constant offset changes nothing because bin 0 is not a candidate and all other bins stay ~0;
    # exact ties only exist for the all-zero window, which is what is asserted above
    topk5, _, _ = kdfh.kdfh(np.zeros((1, 1, 512)), 5)
    assert topk5[0].tolist() == [1, 2, 3, 4, 5]


def test_ties_rank_the_lower_bin_first_and_order_is_descending():
    abar = np.array([[1.0, 5.0, 5.0, 0.5, 5.0, 7.0]])
    assert kdfh.ranked_topk(abar, 4, f_min=1)[0].tolist() == [6, 2, 3, 5]
    assert kdfh.ranked_topk(abar, 6, f_min=0)[0].tolist() == [5, 1, 2, 4, 0, 3]


def test_ranked_topk_against_brute_force():
    rng = np.random.default_rng(11)
    abar = rng.integers(0, 6, size=(40, 9)).astype(np.float64)        # many ties
    got = kdfh.ranked_topk(abar, 4, f_min=2)
    for n in range(40):
        remaining = list(range(9))
        want = []
        for _ in range(4):                                           # repeated arg-max, first maximum wins
            best = remaining[0]
            for j in remaining:
                if abar[n, j] > abar[n, best]:
                    best = j
            want.append(best + 2)
            remaining.remove(best)
        assert got[n].tolist() == want


def test_hash_is_injective_and_ordered_like_the_tuples():
    R, k = 7, 3
    tuples = list(itertools.product(range(R), repeat=k))
    h = kdfh.hash_values(np.asarray(tuples), R)
    assert len(set(h.tolist())) == len(tuples)
    assert h.tolist() == sorted(h.tolist())                           # product() is lexicographic
    for tup, hv in zip(tuples, h):
        assert kdfh.decode_hash(hv, k, R) == tup


def test_hash_range_check():
    with pytest.raises(ValueError):
        kdfh.hash_values(np.zeros((1, 8), dtype=np.int64), 257)       # 257**8 > 2**63
    assert int(kdfh.hash_values(np.full((1, 5), 256), 257)[0]) == 257 ** 5 - 1


def test_argument_checks():
    x = np.zeros((1, 1, 96))
    with pytest.raises(ValueError):
        kdfh.kdfh(x, 3, f_min=1, f_max=49)
    with pytest.raises(ValueError):
        kdfh.kdfh(x, 30, f_min=1, f_max=25)


# ---------------------------------------------------------------- Theorem 1
def test_theorem_1_reconstruction_error_is_half_the_dropped_energy():
    # n sinusoids on integer bins; rebuild the signal from the oracle's k dominant bins
    # (their real/imaginary parts); the mean squared error must equal 1/2 sum_{i>k} A_i^2.
    L, k = 96, 3
    freqs = [4, 8, 12, 20, 7, 16]
    amps = [2.0, 1.5, 1.1, 0.7, 0.4, 0.2]
    phis = [0.3, 1.0, 2.0, 4.0, 5.0, 0.7]
    x = sum(sinusoid(L, a, f, p) for f, a, p in zip(freqs, amps, phis))
    topk, _, _ = kdfh.kdfh(x[None, None, :], k)
    assert topk[0].tolist() == freqs[:k]
    re, im = kdfh.dft(x, topk[0])
    t = np.arange(L)
    recon = sum((2.0 / L) * (re[j] * np.cos(2 * np.pi * f * t / L) - im[j] * np.sin(2 * np.pi * f * t / L))
                for j, f in enumerate(topk[0]))
    mse = np.mean((x - recon) ** 2)
    assert mse == pytest.approx(0.5 * sum(a * a for a in amps[k:]), rel=1e-10)


# ---------------------------------------------------------------- invariances
def _noisy_batch(seed, B=6, N=5, L=96):
    rng = np.random.default_rng(seed)
    x = 0.05 * rng.standard_normal((B, N, L))
    for n in range(N):
        fs = rng.choice(np.arange(1, 25), size=4, replace=False)
        for j, f in enumerate(fs):
            for b in range(B):
                x[b, n] += sinusoid(L, 2.0 / (1.5 ** j), f, rng.uniform(0, 6.28))
    return x


def test_hash_invariant_under_window_permutation_and_positive_scaling():
    x = _noisy_batch(5)
    t0, h0, a0 = kdfh.kdfh(x, 3)
    t1, h1, a1 = kdfh.kdfh(x[::-1], 3)
    assert np.array_equal(h0, h1) and np.allclose(a0, a1, rtol=1e-13)
    scale = np.array([0.01, 0.5, 1.0, 30.0, 1e4])[None, :, None]
    t2, h2, a2 = kdfh.kdfh(x * scale, 3)
    assert np.array_equal(t0, t2) and np.array_equal(h0, h2)
    assert np.allclose(a2, a0 * scale[0], rtol=1e-12)


def test_circular_shift_leaves_amplitudes_unchanged():
    x = _noisy_batch(6)
    a0 = kdfh.amplitudes(x, 1, 25)
    a1 = kdfh.amplitudes(np.roll(x, 17, axis=-1), 1, 25)
    assert np.allclose(a0, a1, rtol=1e-10, atol=1e-10)


def test_one_hash_per_variate_shared_by_the_batch():
    x = _noisy_batch(7, B=4, N=9)
    topk, h, abar = kdfh.kdfh(x, 3)
    assert topk.shape == (9, 3) and h.shape == (9,) and abar.shape == (9, 25)
    assert h.dtype == np.uint64


# ---------------------------------------------------------------- screening helper
def test_gap_screen():
    abar = np.array([[10.0, 5.0, 2.0, 1.0, 0.1],
                     [10.0, 9.9999, 2.0, 1.0, 0.1],       # ranks 1/2 too close
                     [10.0, 5.0, 2.0, 1.9995, 0.1]])      # ranks 3/4 too close
    assert kdfh.gap_ok(abar, 3).tolist() == [True, False, False]
    assert kdfh.gap_ok(abar, 2).tolist() == [True, False, True]
