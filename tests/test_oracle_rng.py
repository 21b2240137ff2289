"""Pins for the oracle's random direction z (run without a GPU)."""
import os

import numpy as np
import pytest
from scipy import stats

from oracle import philox

HERE = os.path.dirname(os.path.abspath(__file__))


def _kat():
    rows = []
    with open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([int(x, 16) for x in line.split()])
    return rows


def test_philox_known_answers():
    rows = _kat()
    assert len(rows) == 3
    for r in rows:
        out = philox.philox4x32_10(r[0], r[1], r[2], r[3], r[4], r[5])
        assert [int(np.asarray(x).reshape(-1)[0]) for x in out] == r[6:10]


def test_philox_vectorised_matches_scalar():
    c0 = np.array([0, 0xFFFFFFFF, 0x243F6A88, 7], dtype=np.uint32)
    out = philox.philox4x32_10(c0, 5, 9, 0, 0xDEADBEEF, 0x12345678)
    for i, c in enumerate(c0):
        one = philox.philox4x32_10(int(c), 5, 9, 0, 0xDEADBEEF, 0x12345678)
        assert [int(o[i]) for o in out] == [int(np.asarray(x).reshape(-1)[0]) for x in one]


def test_word_addressing():
    """Stream word j is output j&3 of call j>>2 with counter (lo(q), hi(q), tensor, 0) and
    key (lo(seed), hi(seed)); the 64-bit word index and seed really use both halves."""
    seed = (0xABCDEF01 << 32) | 0x13572468
    e0 = (1 << 34) + 6
    w = philox.random_words(seed, 77, e0, 9)
    for i in range(9):
        e = e0 + i
        q = e >> 2
        x = philox.philox4x32_10(q & 0xFFFFFFFF, q >> 32, 77, 0, seed & 0xFFFFFFFF, seed >> 32)
        assert int(w[i]) == int(np.asarray(x[e & 3]).reshape(-1)[0])
    # a different tensor id, seed half or high index word changes the stream
    assert not np.array_equal(w, philox.random_words(seed, 78, e0, 9))
    assert not np.array_equal(w, philox.random_words(seed ^ (1 << 40), 77, e0, 9))
    assert not np.array_equal(w, philox.random_words(seed, 77, e0 - (1 << 34), 9))


def test_gaussian_window_invariance():
    """z depends on (seed, tensor, e) only: any window / piece cut gives the same values."""
    full = philox.gaussian(42, 3, 0, 5000)
    for e0, n in ((0, 1), (1, 7), (2, 4), (3, 1001), (4093, 907)):
        assert np.array_equal(full[e0:e0 + n], philox.gaussian(42, 3, e0, n))
    big = philox.gaussian(7, 1, 5, (1 << 21) + 3)            # crosses the threaded path's cuts
    assert np.array_equal(big, philox._gaussian_piece(7, 1, 5, (1 << 21) + 3))
    assert np.array_equal(philox.gaussian(42, 3, 0, 64), philox.gaussian(42, 3, 0, 64))


def test_gaussian_box_muller_structure():
    """Elements (2j, 2j+1) come from stream word j: they share the radius
    rho = sqrt(-2 ln u1) set by the word's high half and the angle set by its low half."""
    w = philox.random_words(9, 4, 0, 2048).astype(np.int64)
    z = philox.gaussian(9, 4, 0, 4096).astype(np.float64).reshape(-1, 2)
    u1 = ((w >> 16) + 1) / 2.0 ** 16
    u2 = (w & 0xFFFF) / 2.0 ** 16
    r2 = z[:, 0] ** 2 + z[:, 1] ** 2
    assert np.allclose(r2, -2 * np.log(u1), rtol=1e-5, atol=1e-6)
    ang = np.mod(np.arctan2(z[:, 1], z[:, 0]) / (2 * np.pi), 1.0)
    ok = r2 > 1e-3
    d = np.abs(ang - u2)[ok]
    assert np.all(np.minimum(d, 1 - d) < 1e-5)
    # a window that starts in the middle of a Philox call (element 8q + 5) lines up with the same words
    z5 = philox.gaussian(9, 4, 8 * 37 + 5, 3).astype(np.float64)
    assert np.array_equal(z5, z.reshape(-1)[8 * 37 + 5: 8 * 37 + 8])


def test_gaussian_distribution():
    n = 1 << 20
    z = philox.gaussian(42, 2, 0, n).astype(np.float64)
    assert abs(z.mean()) < 4 / np.sqrt(n)
    assert abs(z.var() - 1) < 4 * np.sqrt(2 / n)
    assert abs(stats.skew(z)) < 0.02 and abs(stats.kurtosis(z)) < 0.03
    assert stats.kstest(z, "norm").pvalue > 1e-3
    assert np.abs(z).max() <= np.sqrt(-2 * np.log(2.0 ** -16)) + 1e-6      # 4.710
    assert np.abs(z).max() > 4.0                                           # the tail is there up to the cut
    # no linear correlation between neighbours, tensors, seeds (consecutive steps)
    z_t = philox.gaussian(42, 3, 0, n).astype(np.float64)
    z_s = philox.gaussian(43, 2, 0, n).astype(np.float64)
    lim = 5 / np.sqrt(n)
    assert abs(np.mean(z[:-1] * z[1:])) < lim
    assert abs(np.mean(z[0::4] * z[2::4])) < lim * 2
    assert abs(np.mean(z * z_t)) < lim
    assert abs(np.mean(z * z_s)) < lim


def test_rounding_bits_are_a_separate_uniform_stream():
    """The 16-bit rounding draws come from the same generator with the last counter word set to 1: halves of the
    words of call e >> 3, uniform, window-invariant, and unrelated to the words z is drawn from."""
    seed, tid = 1234567, 9
    r = philox.rounding_bits(seed, tid, 0, 1 << 16).astype(np.int64)
    for e in (0, 1, 6, 7, 8, 13, 4095):
        q = e >> 3
        x = philox.philox4x32_10(q, 0, tid, 1, seed & 0xFFFFFFFF, seed >> 32)
        w = int(np.asarray(x[(e >> 1) & 3]).reshape(-1)[0])
        assert int(r[e]) == (w >> (16 * (e & 1))) & 0xFFFF
    assert np.array_equal(r[100:177], philox.rounding_bits(seed, tid, 100, 77))
    assert abs(r.mean() / 65535 - 0.5) < 4 / np.sqrt(12 * r.size)
    assert stats.kstest(r / 65536.0, "uniform").pvalue > 1e-3
    zw = philox.random_words(seed, tid, 0, 1 << 15).astype(np.int64)             # the stream z uses (counter word 0)
    assert abs(np.corrcoef(r[0::2], zw & 0xFFFF)[0, 1]) < 5 / np.sqrt(zw.size)
