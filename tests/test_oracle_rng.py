"""Pins for oracle.rng: the hash against the published SplitMix64 sequence, uniformity,
stream independence, and the Gumbel-argmax draw against the distribution it must follow."""
import numpy as np
from scipy import stats

from oracle import rng


def test_mix64_reproduces_published_splitmix64_sequence():
    # SplitMix64 (Steele, Lea, Flood 2014) seeded with 1234567: next() = mix64(state += golden)
    want = [6457827717110365317, 3203168211198807973, 9817491932198370423,
            4593380528125082431, 16408922859458223821]
    x = np.uint64(1234567)
    got = []
    with np.errstate(over="ignore"):
        for _ in want:
            x = x + np.uint64(0x9E3779B97F4A7C15)
            got.append(int(rng.mix64(x)))
    assert got == want


def test_uniform_range_and_float32_exact():
    u = rng.uniform(7, 3, 11, np.arange(200000))
    assert u.min() > 0.0 and u.max() < 1.0
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)


def test_uniform_is_uniform_chi_square():
    u = rng.uniform(123, 0, 5, np.arange(400000))
    counts, _ = np.histogram(u, bins=64, range=(0, 1))
    p = stats.chisquare(counts).pvalue
    assert p > 1e-4


def test_streams_positions_seeds_decorrelated():
    idx = np.arange(100000)
    base = rng.uniform(1, 0, 0, idx)
    for other in (rng.uniform(2, 0, 0, idx), rng.uniform(1, 1, 0, idx), rng.uniform(1, 0, 1, idx)):
        assert abs(np.corrcoef(base, other)[0, 1]) < 0.02
        assert not np.array_equal(base, other)


def test_gumbel_argmax_follows_softmax():
    logits = np.array([0.3, -1.0, 2.0, 0.0, 1.1])
    p = np.exp(logits) / np.exp(logits).sum()
    n = 40000
    counts = np.zeros(5)
    for pos in range(n):
        g = rng.gumbel(99, rng.stream_id(0, rng.STREAM_BONUS), pos, np.arange(5))
        counts[np.argmax(logits + g)] += 1
    assert stats.chisquare(counts, p * n).pvalue > 1e-4
