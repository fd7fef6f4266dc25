"""Pins for the oracle's gradient statistics (no GPU): the density measure of
equation (1) and Welford's single-pass mean / variance that Section 3 uses for
Figure 1 (arxiv 1802.04434)."""
import math
from fractions import Fraction

import numpy as np
import pytest

import exact
from test_oracle_pins import fr


def test_density_of_dense_and_sparse_vectors(oracle):
    # the two values the paper states: 1 for a fully dense vector, 1/d for a fully sparse one
    for d in (1, 7, 1000, 65_537):
        ones = np.ones(d, np.float32)
        assert oracle.density(ones)[2] == 1.0
        assert oracle.density(-3.5 * ones)[2] == 1.0
        signs = np.where(np.arange(d) % 3 == 0, -2.0, 2.0).astype(np.float32)
        assert oracle.density(signs)[2] == 1.0
        hot = np.zeros(d, np.float32)
        hot[d // 2] = -7.0
        l1, l2sq, phi = oracle.density(hot)
        assert (l1, l2sq) == (7.0, 49.0) and phi == pytest.approx(1.0 / d, rel=1e-15)
    assert oracle.density(np.zeros(5, np.float32)) == (0.0, 0.0, 0.0)
    assert oracle.density(np.zeros(0, np.float32)) == (0.0, 0.0, 0.0)


def test_density_closed_form_and_exact_rational(oracle):
    # v = (1, 2, ..., d): |v|_1 = d(d+1)/2, |v|_2^2 = d(d+1)(2d+1)/6, phi = 3(d+1) / (2(2d+1))
    for d in (1, 2, 10, 1000, 4000):
        v = np.arange(1, d + 1, dtype=np.float32)
        l1, l2sq, phi = oracle.density(v)
        assert l1 == d * (d + 1) / 2 and l2sq == d * (d + 1) * (2 * d + 1) / 6
        assert phi == pytest.approx(3 * (d + 1) / (2 * (2 * d + 1)), rel=1e-15)
    rng = np.random.default_rng(31)
    v = (rng.standard_normal(300) * 10.0 ** rng.integers(-3, 3, 300)).astype(np.float32)
    l1 = sum(abs(fr(t)) for t in v)
    l2sq = sum(fr(t) ** 2 for t in v)
    got = oracle.density(v)
    assert got[0] == pytest.approx(float(l1), rel=1e-15) and got[1] == pytest.approx(float(l2sq), rel=1e-15)
    assert got[2] == pytest.approx(float(l1 * l1 / (300 * l2sq)), rel=1e-14)
    # scale invariance, permutation invariance, and the bound |v|_1^2 <= phi d^2 |v|_inf^2
    assert oracle.density(np.float32(8.0) * v)[2] == pytest.approx(got[2], rel=1e-15)
    assert oracle.density(v[::-1].copy())[2] == pytest.approx(got[2], rel=1e-14)
    assert got[0] ** 2 <= got[2] * 300 ** 2 * float(np.max(np.abs(v))) ** 2 * (1 + 1e-12)
    assert 1.0 / 300 <= got[2] <= 1.0


def test_density_of_a_gaussian_vector_is_two_over_pi(oracle):
    # (E|z|)^2 / E z^2 = 2 / pi
    z = np.random.default_rng(32).standard_normal(1 << 21).astype(np.float32)
    assert oracle.density(z)[2] == pytest.approx(2 / math.pi, abs=2e-3)


def test_welford_hand_cases(oracle):
    # exact in binary: samples 1, 3 -> mean 2, sum of squared deviations 2; then 8 -> mean 4, m2 26
    mean = np.zeros(1, np.float32)
    m2 = np.zeros(1, np.float32)
    oracle.welford_update(np.array([1.0], np.float32), mean, m2, 1)
    assert (mean[0], m2[0]) == (1.0, 0.0)
    oracle.welford_update(np.array([3.0], np.float32), mean, m2, 2)
    assert (mean[0], m2[0]) == (2.0, 2.0)
    oracle.welford_update(np.array([8.0], np.float32), mean, m2, 3)
    assert (mean[0], m2[0]) == (4.0, 26.0)               # (1-4)^2 + (3-4)^2 + (8-4)^2
    assert oracle.welford_sigma(np.array([32.0], np.float32), 2)[0] == 4.0
    # identical samples: the mean is the sample, no spread, exactly
    g = np.random.default_rng(33).standard_normal(100).astype(np.float32)
    mean = np.zeros(100, np.float32)
    m2 = np.zeros(100, np.float32)
    for n in range(1, 6):
        oracle.welford_update(g, mean, m2, n)
    assert np.array_equal(mean, g) and not m2.any()


def test_welford_exact_rational_operation_order(oracle):
    rng = np.random.default_rng(34)
    d, steps = 60, 7
    mean = np.zeros(d, np.float32)
    m2 = np.zeros(d, np.float32)
    mean_q = [Fraction(0)] * d
    m2_q = [Fraction(0)] * d
    for n in range(1, steps + 1):
        g = (rng.standard_normal(d) * 3 + 1).astype(np.float32)
        oracle.welford_update(g, mean, m2, n)
        for i in range(d):
            gi = fr(g[i])
            delta = exact.round_f32(gi - mean_q[i])
            mean_q[i] = exact.round_f32(mean_q[i] + exact.round_f32(delta / n))
            m2_q[i] = exact.round_f32(m2_q[i] + exact.round_f32(delta * exact.round_f32(gi - mean_q[i])))
            assert fr(mean[i]) == mean_q[i] and fr(m2[i]) == m2_q[i], (n, i)
    sigma = oracle.welford_sigma(m2, steps)
    for i in range(d):
        var = exact.round_f32(m2_q[i] / steps)
        s = fr(sigma[i])
        # correctly rounded square root: s is the fp32 nearest to sqrt(var)
        ulp = Fraction(float(np.spacing(sigma[i])))
        assert (s - ulp / 2) ** 2 <= var <= (s + ulp / 2) ** 2


def test_welford_matches_two_pass_statistics(oracle):
    rng = np.random.default_rng(35)
    d, steps = 2000, 200
    mu = rng.standard_normal(d)
    sd = np.abs(rng.standard_normal(d)) + 0.1
    samples = (mu + sd * rng.standard_normal((steps, d))).astype(np.float32)
    mean = np.zeros(d, np.float32)
    m2 = np.zeros(d, np.float32)
    for n in range(steps):
        oracle.welford_update(samples[n], mean, m2, n + 1)
    ref_mean = samples.astype(np.float64).mean(axis=0)
    ref_sigma = samples.astype(np.float64).std(axis=0)           # population: divide by n
    assert np.allclose(mean, ref_mean, rtol=0, atol=2e-5)
    assert np.allclose(oracle.welford_sigma(m2, steps), ref_sigma, rtol=2e-5)
    # bf16 samples are widened exactly
    bf = (samples[0].view(np.uint32) >> 16).astype(np.uint16)
    mean_b = np.zeros(d, np.float32)
    m2_b = np.zeros(d, np.float32)
    oracle.welford_update(bf, mean_b, m2_b, 1)
    assert np.array_equal(mean_b.view(np.uint32), bf.astype(np.uint32) << 16)
