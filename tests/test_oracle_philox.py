"""Pins for the oracle's Philox4x32-10 against the generator's published known answers."""
import numpy as np

from oracle import philox
from conftest import read_golden


def _kat():
    rows = []
    for line in read_golden("philox4x32_10_kat.txt"):
        w = [int(t, 16) for t in line.split()]
        rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_known_answers_scalar():
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, out in rows:
        assert list(philox.philox4x32_10(ctr, key)) == out


def test_known_answers_array():
    for ctr, key, out in _kat():
        r = philox.philox4x32_10_array([ctr[0]], ctr[1], ctr[2], ctr[3], key[0], key[1])
        assert [int(v[0]) for v in r] == out


def test_array_equals_scalar_on_random_counters():
    rng = np.random.default_rng(7)
    c = rng.integers(0, 2 ** 32, size=(4, 50), dtype=np.uint64)
    k = rng.integers(0, 2 ** 32, size=2, dtype=np.uint64)
    r = philox.philox4x32_10_array(c[0], c[1], c[2], c[3], int(k[0]), int(k[1]))
    for i in range(50):
        assert tuple(int(v[i]) for v in r) == philox.philox4x32_10(c[:, i].tolist(), k.tolist())


def test_is_a_bijection_of_the_counter_on_a_small_slice():
    # distinct counters under one key never collide (the generator is a keyed permutation)
    r = philox.philox4x32_10_array(np.arange(4096), 0, 5, 0, 99, 1)
    words = set(zip(*(v.tolist() for v in r)))
    assert len(words) == 4096
