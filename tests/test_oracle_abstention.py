"""Pins for the oracle's "majority vote with abstention" (Section 6, Discussion,
of arxiv 1802.04434).  The paper gives no thresholds, so the criterion
(|v| < tau abstains; answer 0 unless |S| >= Q) is this build's reading; what is
pinned here is that the oracle computes exactly that reading, by brute force on
small inputs, and that it reduces to Algorithm 3 where it must."""
import itertools

import numpy as np
import pytest

import exact
from test_oracle_pins import fr, rand_grad


def unpack_ternary(oracle, neg, zero, d):
    n = oracle.unpack(neg, d) == -1
    z = oracle.unpack(zero, d) == -1
    assert not np.any(n & z)                 # never both
    return np.where(z, 0, np.where(n, -1, 1))


@pytest.mark.parametrize("d", [1, 31, 33, 257, 1000])
def test_ternary_pack_bruteforce(oracle, d):
    rng = np.random.default_rng(d)
    g = rand_grad(rng, d)
    for tau in (0.0, 0.3, 1.5):
        neg, zero = oracle.signum_pack_ternary(g, None, 0.0, tau)
        want = [0 if abs(float(v)) < float(np.float32(tau)) else (-1 if float(v) < 0 else 1) for v in g]
        assert unpack_ternary(oracle, neg, zero, d).tolist() == want
        assert neg.tolist() == exact.pack([-1 if s == -1 else 1 for s in want])
        assert zero.tolist() == exact.pack([-1 if s == 0 else 1 for s in want])
    # tau = 0: nobody abstains and the negative plane is the ordinary packing
    neg, zero = oracle.signum_pack_ternary(g, None, 0.0, 0.0)
    assert not zero.any() and np.array_equal(neg, oracle.signum_pack(g, None, 0.0))
    # momentum is updated exactly as in Algorithm 2 and the vote is on m
    m = rng.standard_normal(d).astype(np.float32)
    m2 = m.copy()
    neg, zero = oracle.signum_pack_ternary(g, m, 0.9, 0.2)
    oracle.signum_pack(g, m2, 0.9)
    assert np.array_equal(m, m2)
    want = np.where(np.abs(m) < np.float32(0.2), 0, np.where(m < 0, -1, 1))
    assert np.array_equal(unpack_ternary(oracle, neg, zero, d), want)


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5])
def test_quorum_vote_exhaustive(oracle, M):
    # every combination of M ternary votes, one coordinate per combination
    combos = list(itertools.product((-1, 0, 1), repeat=M))
    d = len(combos)
    neg = [np.array(exact.pack([-1 if c[w] == -1 else 1 for c in combos]), np.uint32) for w in range(M)]
    zero = [np.array(exact.pack([-1 if c[w] == 0 else 1 for c in combos]), np.uint32) for w in range(M)]
    for Q in range(1, M + 2):
        vneg, vzero = oracle.quorum_vote(neg, zero, Q, d)
        got = unpack_ternary(oracle, vneg, vzero, d)
        want = [(-1 if sum(c) < 0 else 1) if abs(sum(c)) >= Q else 0 for c in combos]
        assert got.tolist() == want, (M, Q)
    if M % 2 == 1:
        # no abstentions, quorum 1, odd M: Algorithm 3's majority vote
        keep = [i for i, c in enumerate(combos) if 0 not in c]
        vneg, _ = oracle.quorum_vote(neg, zero, 1, d)
        plain = oracle.unpack(oracle.majority_vote(neg, d), d)
        assert np.array_equal(oracle.unpack(vneg, d)[keep], plain[keep])


def test_ternary_apply_moves_or_stays(oracle):
    d = 96
    x = np.linspace(-1, 1, d).astype(np.float32)
    x0 = x.copy()
    neg = np.array([0x0000FFFF, 0, 0xFF, 0], np.uint32)
    zero = np.array([0xFFFF0000, 0, 0xFF00, 0], np.uint32)
    oracle.ternary_apply(x, neg, zero, 0.25)
    ans = unpack_ternary(oracle, neg, zero, d)
    for i in range(d):
        assert fr(x[i]) == (fr(x0[i]) if ans[i] == 0 else exact.apply_step(fr(x0[i]), int(ans[i]), fr(0.25)))


@pytest.mark.parametrize("M", [3, 7, 8])
def test_ternary_step_is_its_parts_and_reduces_to_algorithm_3(oracle, M):
    rng = np.random.default_rng(M)
    d = 3001
    g = [rand_grad(rng, d) for _ in range(M)]
    m0 = [rng.standard_normal(d).astype(np.float32) * np.float32(0.3) for _ in range(M)]
    x0 = rng.standard_normal(d).astype(np.float32)
    m, x = [a.copy() for a in m0], x0.copy()
    vneg, vzero = oracle.signum_vote_step_ternary(g, m, 0.9, 0.15, 2, 1e-2, x)
    m2, x2 = [a.copy() for a in m0], x0.copy()
    parts = [oracle.signum_pack_ternary(g[w], m2[w], 0.9, 0.15) for w in range(M)]
    wneg, wzero = oracle.quorum_vote([p[0] for p in parts], [p[1] for p in parts], 2, d)
    oracle.ternary_apply(x2, wneg, wzero, 1e-2)
    assert np.array_equal(vneg, wneg) and np.array_equal(vzero, wzero) and np.array_equal(x, x2)
    assert all(np.array_equal(a, b) for a, b in zip(m, m2))
    assert 0 < np.count_nonzero(unpack_ternary(oracle, vneg, vzero, d) == 0) < d
    if M % 2 == 1:
        m3, x3 = [a.copy() for a in m0], x0.copy()
        tneg, tzero = oracle.signum_vote_step_ternary(g, m3, 0.9, 0.0, 1, 1e-2, x3)
        m4, x4 = [a.copy() for a in m0], x0.copy()
        voted = oracle.signum_vote_step(g, m4, 0.9, 1e-2, x4)
        assert np.array_equal(tneg, voted) and not tzero.any() and np.array_equal(x3, x4)
