"""Pins for the oracle's two variants of the step (no GPU): Theorem 3's warm-up
(length C(beta) and the warm-up iteration) and Section 4's "(good)" update
x <- x - delta * sum_m sign(g_m)  (arxiv 1802.04434)."""
from fractions import Fraction

import numpy as np
import pytest

import exact
from test_oracle_pins import fr, paper_constants, rand_grad


def warmup_conditions(beta, C):
    """both conditions of Theorem 3, in exact rational arithmetic"""
    first = Fraction(C, 2) * beta ** C <= 1 / (1 - beta ** 2) / (C + 1)
    second = beta ** (C + 1) <= Fraction(1, 2)
    return first, second


def test_warmup_length_value_printed_in_the_paper(oracle):
    c = paper_constants()
    assert oracle.warmup_length(c["warmup_beta"]) == int(c["warmup_C"]) == 54
    beta = Fraction(9, 10)
    assert warmup_conditions(beta, 54) == (True, True)
    assert warmup_conditions(beta, 53) == (False, True)      # 53 still fails the first condition
    assert not any(all(warmup_conditions(beta, C)) for C in range(1, 54))


@pytest.mark.parametrize("beta", [0.5, 0.6, 0.75, 0.8, 0.875, 0.95, 0.96875])
def test_warmup_length_is_the_exact_minimum(oracle, beta):
    # betas exactly representable or not: the rational minimum must agree
    b = fr(beta)
    want = next(C for C in range(1, 5000) if all(warmup_conditions(b, C)))
    assert oracle.warmup_length(beta) == want


def test_warmup_length_rejects_bad_beta(oracle):
    for beta in (0.0, 1.0, -0.5, 1.5):
        with pytest.raises(ValueError):
            oracle.warmup_length(beta)
    assert oracle.warmup_length(0.99) > oracle.warmup_length(0.9) > oracle.warmup_length(0.5) >= 1


def test_warmup_iteration_updates_momentum_but_votes_with_the_gradient(oracle):
    rng = np.random.default_rng(21)
    d = 1000
    g = rand_grad(rng, d)
    m = rng.standard_normal(d).astype(np.float32)
    m_a, m_b = m.copy(), m.copy()
    bits_warm = oracle.signum_pack_warmup(g, m_a, 0.9)
    bits_norm = oracle.signum_pack(g, m_b, 0.9)
    assert np.array_equal(m_a, m_b)                                   # momentum accumulates as normal
    assert np.array_equal(bits_warm, oracle.signum_pack(g, None, 0.0))  # the sign is the gradient's
    assert not np.array_equal(bits_warm, bits_norm)
    # a momentum that disagrees with the gradient: Signum follows m, warm-up follows g
    g1 = -np.ones(64, np.float32)
    m1 = np.full(64, 5.0, np.float32)
    assert oracle.signum_pack(g1, m1.copy(), 0.9)[0] == 0
    assert oracle.signum_pack_warmup(g1, m1.copy(), 0.9)[0] == 0xFFFFFFFF
    # without a momentum buffer it is Algorithm 1
    assert np.array_equal(oracle.signum_pack_warmup(g, None, 0.3), oracle.signum_pack(g, None, 0.0))


def test_sum_apply_exact_rational(oracle):
    rng = np.random.default_rng(22)
    d = 400
    x = (rng.standard_normal(d) * 0.05).astype(np.float32)
    sums = rng.integers(-64, 65, d).astype(np.int8)
    for delta in (1e-4, 0.3, 2.0 ** -10):
        x0 = x.copy()
        x1 = x.copy()
        oracle.sum_apply(x1, sums, delta)
        dl = fr(delta)
        for i in range(d):
            t = exact.round_f32(dl * int(sums[i]))                  # the product is rounded on its own
            assert fr(x1[i]) == exact.round_f32(fr(x0[i]) - t)


def test_sum_apply_with_one_worker_is_sign_apply(oracle):
    rng = np.random.default_rng(23)
    d = 777
    g = rand_grad(rng, d)
    bits = oracle.signum_pack(g, None, 0.0)
    xa = rng.standard_normal(d).astype(np.float32)
    xb = xa.copy()
    oracle.sign_apply(xa, bits, 1e-3)
    oracle.sum_apply(xb, oracle.unpack(bits, d), 1e-3)
    assert np.array_equal(xa.view(np.uint32), xb.view(np.uint32))


@pytest.mark.parametrize("M,momentum", [(1, False), (4, True), (7, True), (16, False)])
def test_step_ex_against_its_parts(oracle, M, momentum):
    rng = np.random.default_rng(M)
    d = 2049
    g = [rand_grad(rng, d) for _ in range(M)]
    m0 = [rng.standard_normal(d).astype(np.float32) for _ in range(M)] if momentum else None
    x0 = rng.standard_normal(d).astype(np.float32)
    delta = 1e-2

    def fresh():
        return ([a.copy() for a in m0] if momentum else None), x0.copy()

    # flags = 0 is the plain step
    m, x = fresh()
    voted, packed, sums = oracle.signum_vote_step_ex(g, m, 0.9, delta, x, 0)
    m2, x2 = fresh()
    voted2, packed2 = oracle.signum_vote_step(g, m2, 0.9, delta, x2, want_packed=True)
    assert np.array_equal(voted, voted2) and np.array_equal(x, x2)
    assert all(np.array_equal(a, b) for a, b in zip(packed, packed2))
    assert np.array_equal(sums.astype(np.int32), oracle.vote_sum(packed, d))
    # "(good)": x moves by delta times the sum; the voted bits are the sum's sign
    m3, x3 = fresh()
    voted3, packed3, sums3 = oracle.signum_vote_step_ex(g, m3, 0.9, delta, x3, oracle.STEP_SUM_UPDATE)
    assert np.array_equal(voted3, voted) and np.array_equal(sums3, sums)
    want = x0.copy()
    oracle.sum_apply(want, sums3, delta)
    assert np.array_equal(x3, want)
    assert np.all(np.abs(sums3) <= M) and np.all((sums3.astype(int) - M) % 2 == 0)
    moved = (x3.astype(np.float64) - x0) / delta
    assert np.allclose(moved, -sums3, atol=1e-3)
    # warm-up: votes are on sign(g), momentum as in the plain step
    m4, x4 = fresh()
    voted4, packed4, _ = oracle.signum_vote_step_ex(g, m4, 0.9, delta, x4, oracle.STEP_WARMUP)
    for w in range(M):
        assert np.array_equal(packed4[w], oracle.signum_pack(g[w], None, 0.0))
        if momentum:
            assert np.array_equal(m4[w], m[w])
    assert np.array_equal(voted4, oracle.majority_vote(packed4, d))
    if M == 1:
        # one worker: "(good)" and "(best)" coincide
        assert np.array_equal(x3.view(np.uint32), x.view(np.uint32))
