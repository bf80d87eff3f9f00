"""Pins for the oracle's counter-based generator (CPU only).

The paper says nothing about random numbers; the build draws them from
Philox4x32-10, so the oracle's implementation is pinned to the publication's
known-answer vectors and to an independent pure-Python-integer implementation."""
import os
import random

import numpy as np

from philox_ref import accept_words, gumbel_word, philox4x32_10

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat():
    rows = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(t, 16) for t in line.split()]
        rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_known_answer_vectors(oracle):
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, out in rows:
        assert list(oracle.philox(ctr, key)) == out
        assert philox4x32_10(ctr, key) == out


def test_matches_python_integers_on_random_counters(oracle):
    rng = random.Random(1234)
    for _ in range(500):
        ctr = [rng.getrandbits(32) for _ in range(4)]
        key = [rng.getrandbits(32) for _ in range(2)]
        assert list(oracle.philox(ctr, key)) == philox4x32_10(ctr, key)


def test_single_bit_of_counter_or_key_changes_output(oracle):
    base = list(oracle.philox([1, 2, 3, 4], [5, 6]))
    for word in range(4):
        c = [1, 2, 3, 4]
        c[word] ^= 1
        assert list(oracle.philox(c, [5, 6])) != base
    assert list(oracle.philox([1, 2, 3, 4], [5, 7])) != base
    assert list(oracle.philox([1, 2, 3, 4], [4, 6])) != base


def test_word_layout_of_the_draws(oracle):
    rng = random.Random(7)
    for _ in range(200):
        seed = rng.getrandbits(64)
        seq, rnd, pos, v = rng.getrandbits(32), rng.getrandbits(32), rng.randrange(21), \
            rng.randrange(152064)
        assert oracle.accept_words(seed, seq, rnd, pos) == accept_words(seed, seq, rnd, pos)
        assert oracle.gumbel_word(seed, seq, rnd, pos, v) == gumbel_word(seed, seq, rnd, pos, v)
    # acceptance and Gumbel streams never share a counter block (bit 16 of word 1 differs)
    assert oracle.gumbel_word(9, 1, 2, 3, 0) != oracle.accept_words(9, 1, 2, 3)[0]


def test_uniform_maps_are_open_interval_and_exact(oracle):
    assert oracle.uniform24(0) == 0.5 / 2 ** 24
    assert oracle.uniform24(0xFFFFFFFF) == 1.0 - 0.5 / 2 ** 24
    assert oracle.uniform24(0x000001FF) == 1.5 / 2 ** 24  # low 8 bits are dropped
    assert oracle.uniform32(0) == 0.5 / 2 ** 32
    assert oracle.uniform32(0xFFFFFFFF) == 1.0 - 0.5 / 2 ** 32
    assert oracle.uniform32(12345) == 12345.5 / 2 ** 32


def test_uniformity_of_draws(oracle):
    # 64 K words of one Gumbel stream: mean 1/2, variance 1/12, chi-square over 64 bins
    n = 1 << 16
    u = np.array([oracle.uniform32(oracle.gumbel_word(42, 3, 5, 2, v)) for v in range(n)])
    assert abs(u.mean() - 0.5) < 4 * (1 / 12 / n) ** 0.5
    assert abs(u.var() - 1 / 12) < 2e-3
    counts, _ = np.histogram(u, bins=64, range=(0, 1))
    chi2 = ((counts - n / 64) ** 2 / (n / 64)).sum()
    assert chi2 < 120.0  # 63 dof: P(chi2 > 120) ~ 2e-5
