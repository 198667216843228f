"""Pins of the sampling oracle: each check compares it with something it does not contain."""
import numpy as np
import pytest
from scipy import special, stats

from oracle import sampling as smp


def test_tempered_is_the_library_softmax_of_the_scaled_logits():
    g = np.random.default_rng(0)
    l = g.standard_normal((3, 5, 257)) * 4
    for T in (1.0, 0.7, 2.5):
        z, lse, p = smp.tempered(l, T)
        np.testing.assert_allclose(p, special.softmax(l / T, axis=-1), rtol=1e-12, atol=0)
        np.testing.assert_allclose(lse, special.logsumexp(l / T, axis=-1), rtol=1e-13)
        np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-12)
    # T = 1 leaves the logits alone
    assert np.array_equal(smp.tempered(l, 1.0)[0], l)


def _unmix32(h):
    """The published inverse of the finaliser (each step is invertible modulo 2^32)."""
    h = np.asarray(h, dtype=np.uint64)
    m = np.uint64(0xFFFFFFFF)
    h ^= h >> np.uint64(16)
    h = (h * np.uint64(0x7ED1B41D)) & m          # inverse of 0xC2B2AE35 modulo 2^32
    h ^= (h >> np.uint64(13)) ^ (h >> np.uint64(26))
    h = (h * np.uint64(0xA5CB9243)) & m          # inverse of 0x85EBCA6B modulo 2^32
    h ^= h >> np.uint64(16)
    return h


def test_the_finaliser_is_the_published_bijection():
    assert (0x85EBCA6B * 0xA5CB9243) % 2 ** 32 == 1 and (0xC2B2AE35 * 0x7ED1B41D) % 2 ** 32 == 1
    x = np.concatenate([np.arange(100000, dtype=np.uint64), np.random.default_rng(1).integers(0, 2 ** 32, 100000, dtype=np.uint64)])
    y = smp.fmix32(x)
    assert np.array_equal(_unmix32(y), x)
    assert int(smp.fmix32(np.uint64(0))) == 0                       # the finaliser's fixed point
    assert len(np.unique(y)) == len(np.unique(x))


def test_uniform_numbers_are_uniform_and_independent_across_ids_rows_and_seeds():
    n = 200000
    u = smp.uniform(1234, 3, np.arange(n))
    assert 0.0 < u.min() and u.max() < 1.0
    assert np.array_equal(u.astype(np.float32).astype(np.float64), u)    # exact in float32
    assert abs(u.mean() - 0.5) < 4 * np.sqrt(1 / 12 / n) and abs(u.var() - 1 / 12) < 1e-3
    counts = np.bincount((u * 64).astype(int), minlength=64)
    assert stats.chisquare(counts).pvalue > 1e-4
    for other in (smp.uniform(1234, 4, np.arange(n)), smp.uniform(1235, 3, np.arange(n)),
                  smp.uniform(1234 + (1 << 32), 3, np.arange(n)), np.roll(u, 1)):
        assert abs(np.corrcoef(u, other)[0, 1]) < 5 / np.sqrt(n)
        assert not np.array_equal(u, other)


def _frequencies(z, draws, sampler):
    c = np.zeros(len(z))
    for s in range(draws):
        c[sampler(z, s)] += 1
    return c


def test_gumbel_max_draws_follow_the_softmax():
    g = np.random.default_rng(5)
    z = g.standard_normal(12) * 2.0
    _, _, p = smp.tempered(z, 1.0)
    draws = 40000
    c = _frequencies(z, draws, lambda zz, s: smp.gumbel_sample(zz, 1000 + s, 2)[0])
    assert stats.chisquare(c, p * draws).pvalue > 1e-4
    # an inversion sampler over the same probabilities gives statistically the same frequencies
    inv = np.bincount(np.searchsorted(np.cumsum(p), np.random.default_rng(6).random(draws)).clip(0, len(p) - 1), minlength=len(p))
    assert stats.chi2_contingency(np.stack([c, inv]))[1] > 1e-4
    # planted mistakes fail the same test: no minus sign in front of the outer logarithm; the wrong temperature
    wrong_sign = _frequencies(z, draws, lambda zz, s: int(np.argmax(zz + np.log(-np.log(smp.uniform(1000 + s, 2, np.arange(len(zz))))))))
    assert stats.chisquare(wrong_sign + 1e-9, p * draws).pvalue < 1e-12
    z_half, _, p_half = smp.tempered(z, 0.5)
    assert stats.chisquare(c, p_half * draws).pvalue < 1e-12
    c_half = _frequencies(z_half, draws, lambda zz, s: smp.gumbel_sample(zz, 5000 + s, 0)[0])
    assert stats.chisquare(c_half, p_half * draws).pvalue > 1e-4


def test_low_temperature_reproduces_the_argmax_and_ties_go_to_the_lower_id():
    g = np.random.default_rng(7)
    l = g.standard_normal(500)
    z, _, p = smp.tempered(l, 1e-3)
    assert all(smp.gumbel_sample(z, s, 0)[0] == int(np.argmax(l)) for s in range(50))
    # margin: distance of the winner's perturbed value to the runner-up
    best, val, margin = smp.gumbel_sample(l, 9, 1)
    v = l + smp.gumbel(9, 1, np.arange(500))
    assert best == int(np.argmax(v)) and val == v.max() and np.isclose(margin, np.sort(v)[-1] - np.sort(v)[-2])
    # one token in the vocabulary: always drawn
    assert smp.gumbel_sample(np.array([0.3]), 1, 0)[0] == 0
