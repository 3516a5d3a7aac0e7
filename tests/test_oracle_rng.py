"""Pins of the oracle's counter-based generator and of the draws built on it."""
import os

import numpy as np
from scipy import stats

GOLD = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _draw(ora, seed, stream, blk, worker, it):
    key = [seed & 0xFFFFFFFF, ((seed >> 32) & 0xFFFFFFFF) ^ stream]
    return ora.philox4x32_10([blk, worker, it & 0xFFFFFFFF, it >> 32], key)


def test_philox_known_answers(ora):
    n = 0
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(t, 16) for t in line.split()]
        assert list(ora.philox4x32_10(v[0:4], v[4:6])) == v[6:10]
        n += 1
    assert n == 3


def test_philox_words_are_uniform(ora):
    words = np.concatenate([ora.philox4x32_10([c, 7, 0, 0], [123, 456]) for c in range(20000)])
    # byte histogram of every byte lane
    for sh in (0, 8, 16, 24):
        h = np.bincount((words >> sh) & 0xFF, minlength=256)
        assert stats.chisquare(h).pvalue > 1e-4
    assert abs(words.astype(np.float64).mean() / 2**32 - 0.5) < 0.01


def test_batch_indices_in_range_and_uniform(ora):
    M, B = 3, 64
    shard_off = np.array([0, 10, 17, 1017], dtype=np.int64)
    n = np.diff(shard_off)
    counts = [np.zeros(k, dtype=np.int64) for k in n]
    for it in range(400):
        idx = ora.sample_batch(M, B, shard_off, 99, it)
        for i in range(M):
            assert idx[i].min() >= 0 and idx[i].max() < n[i]
            counts[i] += np.bincount(idx[i], minlength=n[i])
    assert stats.chisquare(counts[0]).pvalue > 1e-4
    assert stats.chisquare(counts[1]).pvalue > 1e-4
    # the index is floor(u * n / 2^32) of word b%4 of block b/4, stream 1
    idx = ora.sample_batch(M, B, shard_off, 99, 5)
    for i in range(M):
        for b in (0, 1, 5, 63):
            u = int(_draw(ora, 99, 1, b // 4, i, 5)[b % 4])
            assert idx[i, b] == (u * int(n[i])) >> 32


def test_synthetic_gradient_moments(ora):
    M, D, ld, sigma = 2, 200_000, 200_000 + 64, 1e-3 ** 0.5
    g = ora.synth_grad(M, D, ld, sigma, 11, 3)
    assert np.all(g[:, D:] == 0.0)
    z = g[:, :D].astype(np.float64) / sigma
    n = z.size
    assert abs(z.mean()) < 5 / np.sqrt(n)
    assert abs(z.var() - 1.0) < 5 * np.sqrt(2.0 / n)
    assert abs(stats.kurtosis(z.ravel())) < 5 * np.sqrt(24.0 / n)
    assert stats.kstest(z.ravel()[:50000], "norm").pvalue > 1e-4
    # successive elements (cos/sin branches of one pair, and neighbouring pairs) are uncorrelated
    for lag in (1, 2, 4):
        r = np.corrcoef(z[0, :-lag], z[0, lag:])[0, 1]
        assert abs(r) < 5 / np.sqrt(D)
    # different workers and iterations give different streams; the same counter the same values
    assert abs(np.corrcoef(z[0], z[1])[0, 1]) < 5 / np.sqrt(D)
    g2 = ora.synth_grad(M, D, ld, sigma, 11, 4)
    assert abs(np.corrcoef(g2[0, :D], g[0, :D])[0, 1]) < 5 / np.sqrt(D)
    assert np.array_equal(ora.synth_grad(M, D, ld, sigma, 11, 3), g)


def test_synthetic_gradient_follows_box_muller_of_the_words(ora):
    sigma = 0.25
    g = ora.synth_grad(1, 16, 64, sigma, 77, 9)
    for blk in range(4):
        r = _draw(ora, 77, 2, blk, 0, 9).astype(np.float64)
        u = (np.floor(r / 512.0) + 0.5) / 2**23
        assert np.all(u.astype(np.float32).astype(np.float64) == u) and np.all((u > 0) & (u < 1))
        for h in range(2):
            rad = np.sqrt(-2 * np.log(u[2 * h]))
            want = sigma * rad * np.array([np.cos(2 * np.pi * u[2 * h + 1]), np.sin(2 * np.pi * u[2 * h + 1])])
            np.testing.assert_allclose(g[0, 4 * blk + 2 * h: 4 * blk + 2 * h + 2], want, rtol=1e-6, atol=1e-9)
