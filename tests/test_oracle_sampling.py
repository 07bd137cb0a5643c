"""Pins for the oracle's speculative-sampling primitives (CPU only).

Section 2 / Eq. (1): accepting x ~ q with probability min(1, p[x]/q[x]) and otherwise drawing
from norm(max(0, p - q)) yields a token distributed exactly as p.  Closed forms used here:
output distribution == p; acceptance frequency == sum_k min(p_k, q_k).
"""
import math

import numpy as np
import pytest
from scipy import stats

from oracle import sampling


def _dists(v, seed):
    rng = np.random.default_rng(seed)
    p = rng.dirichlet(np.ones(v) * 0.7)
    q = rng.dirichlet(np.ones(v) * 0.7)
    return p, q


def test_probs_softmax_scale_temperature_and_greedy():
    x = np.array([[0.0, math.log(2.0), math.log(5.0)]])
    np.testing.assert_allclose(sampling.probs(x, 1.0), [[1 / 8, 2 / 8, 5 / 8]], rtol=1e-15)
    np.testing.assert_allclose(sampling.probs(x, 0.5), [[1 / 30, 4 / 30, 25 / 30]], rtol=1e-14)      # logits / T
    np.testing.assert_allclose(sampling.probs(x, 1.0, logit_scale=2.0), [[1 / 30, 4 / 30, 25 / 30]], rtol=1e-14)
    g = sampling.probs(np.array([[1.0, 7.0, 7.0, 2.0]]), 0.0)
    assert g.tolist() == [[0.0, 1.0, 0.0, 0.0]]                       # ties -> lowest id
    big = sampling.probs(np.array([[1000.0, 1001.0]], dtype=np.float32), 1.0)
    assert np.isfinite(big).all() and abs(big.sum() - 1) < 1e-6


def test_sample_is_inverse_cdf_in_ascending_id():
    w = [0.1, 0.0, 0.4, 0.5]
    assert sampling.sample(w, 0.0) == 0
    assert sampling.sample(w, 0.0999) == 0
    assert sampling.sample(w, 0.1) == 2            # cdf must exceed u strictly; id 1 has no mass
    assert sampling.sample(w, 0.4999) == 2
    assert sampling.sample(w, 0.5) == 3
    assert sampling.sample(w, 0.999999) == 3
    assert sampling.sample([3.0, 1.0], 0.74) == 0  # unnormalised weights
    assert sampling.sample([3.0, 1.0], 0.76) == 1
    assert sampling.sample([0.5, 0.5, 0.0], 0.9999999999999999) == 1   # never lands on a zero-mass tail
    with pytest.raises(ValueError):
        sampling.sample([0.0, 0.0], 0.3)


def test_accept_rule_and_residual():
    p = np.array([0.5, 0.3, 0.2]); q = np.array([0.2, 0.6, 0.2])
    assert sampling.accept(p, q, 0, 0.999)                 # p >= q: always
    assert sampling.accept(p, q, 1, 0.5)                   # r <= 0.3/0.6
    assert not sampling.accept(p, q, 1, 0.5000001)
    assert sampling.accept(p, q, 2, 0.999)                 # equality p == q accepts
    np.testing.assert_allclose(sampling.residual(p, q), [0.3, 0.0, 0.0], atol=1e-16)
    assert sampling.resample(p, q, 0.99) == 0
    assert sampling.resample(p, p, 0.6) == 1               # no residual mass -> falls back to p


def test_special_cases_identical_and_disjoint():
    p, _ = _dists(8, 1)
    rng = np.random.default_rng(2)
    for _ in range(200):
        x = sampling.sample(p, rng.random())
        assert sampling.accept(p, p, x, rng.random())      # p == q: always accepted
    a = np.array([0.5, 0.5, 0, 0]); b = np.array([0, 0, 0.25, 0.75])
    for _ in range(200):
        x = sampling.sample(b, rng.random())
        assert not sampling.accept(a, b, x, max(rng.random(), 1e-12))
    np.testing.assert_allclose(sampling.residual(a, b), a)   # disjoint supports: resample ~ p


def test_speculative_sampling_output_distribution_equals_target_chi_square():
    """Vocabulary 8, 1e6 seeded trials: chi-square of the emitted token against p."""
    v, n = 8, 1_000_000
    p, q = _dists(v, 11)
    rng = np.random.default_rng(12345)
    u = rng.random((n, 3))
    counts = np.zeros(v, dtype=np.int64)
    n_acc = 0
    for t in range(n):
        x = sampling.sample(q, u[t, 0])
        if sampling.accept(p, q, x, u[t, 1]):
            counts[x] += 1
            n_acc += 1
        else:
            counts[sampling.resample(p, q, u[t, 2])] += 1
    chi2 = float(((counts - n * p) ** 2 / (n * p)).sum())
    assert chi2 < stats.chi2.ppf(1 - 1e-4, v - 1), (chi2, counts)
    alpha = np.minimum(p, q).sum()                                     # closed-form acceptance rate
    assert abs(n_acc / n - alpha) < 5 * math.sqrt(alpha * (1 - alpha) / n)
    # a wrong residual (|p - q| instead of max(0, p - q)) must be detectable by the same test
    bad = np.abs(p - q) / np.abs(p - q).sum()
    mix = np.minimum(p, q) + (1 - alpha) * bad
    assert float((n * (mix - p) ** 2 / p).sum()) > 10 * stats.chi2.ppf(1 - 1e-4, v - 1)
