"""Pins for the CPU oracle (no GPU): exact-arithmetic brute force, closed
forms, textbook special cases and invariants, chosen so that a dropped term, a
swapped operand, a wrong bit order, polarity or tie rule each fail something.

References are to arxiv 1802.04434: Algorithm 1 (signSGD), Algorithm 2
(Signum), Algorithm 3 (majority vote), Section 4 (Remark 3, Lemma 1 and the
binomial bound in the proof of Theorem 2(b)), Appendix A (toy quadratic).
"""
import math
import os
import random
from fractions import Fraction

import numpy as np
import pytest

import exact

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")


def paper_constants():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#")[0].split()
            if len(line) == 2:
                out[line[0]] = float(line[1])
    return out


def f32(v):
    return np.float32(v)


def fr(v):
    """exact rational value of an fp32"""
    return Fraction(float(np.float32(v)))


SPECIALS = [0.0, -0.0, 1.0, -1.0, 1e-45, -1e-45, 1.1754942e-38, -1.1754942e-38,
            3.4028235e38, -3.4028235e38, 1.17549435e-38, -1.17549435e-38, 0.5, -0.25]
SIZES = [1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 1000]


def rand_grad(rng, d):
    g = rng.standard_normal(d).astype(np.float32)
    k = min(d, len(SPECIALS))
    idx = rng.permutation(d)[:k]
    g[idx] = np.array(SPECIALS[:k], dtype=np.float32)
    return g


# ---------------------------------------------------------------- pack ----

@pytest.mark.parametrize("d", SIZES)
def test_pack_matches_bruteforce(oracle, d):
    rng = np.random.default_rng(d)
    g = rand_grad(rng, d)
    got = oracle.signum_pack(g, None, 0.0)
    want = exact.pack([exact.sign_of(float(v)) for v in g])
    assert got.tolist() == want
    assert len(got) * 4 == oracle.packed_bytes(d) and len(got) % 4 == 0


def test_pack_sign_convention_on_special_values(oracle):
    # sign(v) = -1 only for v < 0: zeros of both signs are "+", negative
    # subnormals are "-"
    vals = np.array([0.0, -0.0, 1e-45, -1e-45, -1.1754942e-38, 3.4e38, -3.4e38, -1.0],
                    dtype=np.float32)
    got = oracle.signum_pack(vals, None, 0.0)
    assert got[0] == 0b11011000
    assert oracle.unpack(got, 8).tolist() == [1, 1, 1, -1, -1, 1, -1, -1]


def test_pack_bit_order_is_lsb_first_little_words(oracle):
    g = np.ones(70, dtype=np.float32)
    g[0] = -1
    g[33] = -1
    g[69] = -1
    got = oracle.signum_pack(g, None, 0.0)
    assert got.tolist() == [1, 2, 1 << 5, 0]


@pytest.mark.parametrize("d", [1, 33, 257, 4099])
def test_pack_roundtrip_popcount_padding(oracle, d):
    rng = np.random.default_rng(100 + d)
    g = rand_grad(rng, d)
    bits = oracle.signum_pack(g, None, 0.0)
    s = oracle.unpack(bits, d)
    assert np.array_equal(s == -1, g < 0)
    assert sum(bin(int(w)).count("1") for w in bits) == int((g < 0).sum())
    # nothing set at or beyond coordinate d
    big = sum(int(w) << (32 * k) for k, w in enumerate(bits))
    assert big >> d == 0


def test_bf16_is_widened_exactly(oracle):
    # bf16 patterns: sign taken on the widened value; a bf16 subnormal and -0
    pats = np.array([0x3F80, 0xBF80, 0x0000, 0x8000, 0x0001, 0x8001, 0x7F7F, 0xFF7F], dtype=np.uint16)
    got = oracle.signum_pack(pats, None, 0.0)
    assert got[0] == 0b10100010
    # momentum sees bits << 16 as an fp32: beta = 0.5, m0 = 0 -> m = g / 2 exactly
    m = np.zeros(8, dtype=np.float32)
    oracle.signum_pack(pats, m, 0.5)
    wide = (pats.astype(np.uint32) << 16).view(np.float32)
    assert np.array_equal(m[:2], wide[:2] * np.float32(0.5))
    assert m[6] == wide[6] * np.float32(0.5)


# ------------------------------------------------------------ momentum ----

def test_momentum_hand_cases(oracle):
    # exact in binary: tells beta*m + (1-beta)*g from every operand swap
    g = np.array([2.0, 2.0, -8.0], dtype=np.float32)
    m = np.array([4.0, 4.0, 16.0], dtype=np.float32)
    for beta, want in ((0.5, [3.0, 3.0, 4.0]), (0.25, [2.5, 2.5, -2.0]), (0.75, [3.5, 3.5, 10.0])):
        mm = m.copy()
        bits = oracle.signum_pack(g, mm, beta)
        assert mm.tolist() == want
        assert bits[0] == sum(1 << i for i, v in enumerate(want) if v < 0)


def test_momentum_exact_rational_rounding(oracle):
    rnd = random.Random(7)
    rng = np.random.default_rng(7)
    n = 400
    betas = [0.9, 0.99, 0.5, 0.1, 0.999, 1.0 / 3.0]
    told_apart = 0
    for beta in betas:
        b32 = f32(beta)
        scale = np.float32(10.0) ** rng.integers(-3, 3, n).astype(np.float32)
        g = (rng.standard_normal(n).astype(np.float32) * scale).astype(np.float32)
        m = (rng.standard_normal(n).astype(np.float32) * scale).astype(np.float32)
        # near-cancellation cases, where the rounding of each product shows most
        for i in range(0, n, 4):
            m[i] = np.float32(-(1.0 - float(b32)) * float(g[i]) / float(b32)) * np.float32(1 + rnd.randint(-3, 3) * 2.0 ** -22)
        m_new = m.copy()
        bits = oracle.signum_pack(g, m_new, float(b32))
        for i in range(n):
            want = exact.momentum(fr(b32), fr(m[i]), fr(g[i]))
            assert fr(m_new[i]) == want, (beta, i)
            assert ((int(bits[i // 32]) >> (i % 32)) & 1) == (1 if want < 0 else 0)
            if exact.momentum_fused(fr(b32), fr(m[i]), fr(g[i])) != want:
                told_apart += 1
    assert told_apart > 50     # the inputs do distinguish a fused multiply-add


def test_momentum_subnormal_products_are_kept(oracle):
    # (1-beta)*g underflows into the subnormal range and must not be flushed
    beta = f32(0.9)
    g = np.array([2e-38, -2e-38, 1.5e-44, -1.5e-44], dtype=np.float32)
    m = np.zeros(4, dtype=np.float32)
    bits = oracle.signum_pack(g, m, float(beta))
    for i in range(4):
        want = exact.momentum(fr(beta), Fraction(0), fr(g[i]))
        assert fr(m[i]) == want and want != 0
    assert bits[0] == 0b1010


def test_one_minus_beta_is_rounded_once():
    # 1 - 0.9f is exact in fp32 (Sterbenz), and is not the fp32 nearest to 0.1
    omb = exact.round_f32(1 - fr(0.9))
    assert omb == 1 - fr(0.9)
    assert float(omb) == 0.10000002384185791
    assert omb != fr(0.1)


def test_momentum_sign_flips_at_the_closed_form_step(oracle):
    # m_0 = 1, constant g = -1, beta = 0.9: m_k = -1 + 2 * 0.9^k, which is
    # positive through k = 6 and negative from k = 7 (0.9^6 = .531, 0.9^7 = .478)
    m = np.ones(1, dtype=np.float32)
    g = -np.ones(1, dtype=np.float32)
    flips = None
    for k in range(1, 12):
        bits = oracle.signum_pack(g, m, 0.9)
        assert abs(float(m[0]) - (-1 + 2 * 0.9 ** k)) < 1e-5
        if bits[0] == 1 and flips is None:
            flips = k
    assert flips == 7


def test_momentum_closed_form_constant_gradient(oracle):
    # zero start, constant gradient: m_k = (1 - beta^k) g, so sign(m_k) = sign(g)
    rng = np.random.default_rng(3)
    g = rng.standard_normal(257).astype(np.float32)
    m = np.zeros_like(g)
    want_bits = oracle.signum_pack(g, None, 0.0)
    for k in range(1, 30):
        bits = oracle.signum_pack(g, m, 0.9)
        assert np.array_equal(bits, want_bits)
        ref = (1.0 - 0.9 ** k) * g.astype(np.float64)
        assert np.max(np.abs(m - ref)) <= 1e-6 * np.max(np.abs(g))


def test_beta_zero_is_signsgd(oracle):
    rng = np.random.default_rng(4)
    g = rand_grad(rng, 1000)
    m = rng.standard_normal(1000).astype(np.float32)
    b0 = oracle.signum_pack(g, m, 0.0)
    assert np.array_equal(m, g)                       # numerically (-0 == +0)
    assert np.array_equal(b0, oracle.signum_pack(g, None, 0.123))


# ---------------------------------------------------------------- vote ----

def pattern_words(M, w):
    """d = 2^M coordinates, coordinate i carries sign pattern i: worker w is
    negative at i iff bit w of i is set."""
    d = 1 << M
    neg = [(i >> w) & 1 for i in range(d)]
    return np.array(exact.pack([-1 if b else 1 for b in neg]), dtype=np.uint32)


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 6, 7, 8, 9, 16])
def test_vote_exhaustive_over_all_sign_patterns(oracle, M):
    d = 1 << M
    packed = [pattern_words(M, w) for w in range(M)]
    voted = oracle.majority_vote(packed, d)
    sums = oracle.vote_sum(packed, d)
    want_signs, want_sums = [], []
    for i in range(d):
        signs = [-1 if (i >> w) & 1 else 1 for w in range(M)]
        want_sums.append(sum(signs))
        want_signs.append(exact.sign_of(sum(signs)))
    assert sums.tolist() == want_sums
    assert voted.tolist() == exact.pack(want_signs)
    # even M: an exact split is "+"
    if M % 2 == 0:
        s = oracle.unpack(voted, d)
        ties = [i for i in range(d) if bin(i).count("1") * 2 == M]
        assert ties and all(s[i] == 1 for i in ties)


def random_words(rng, d):
    n = (d + 31) // 32
    n += (-n) % 4
    w = rng.integers(0, 1 << 32, n, dtype=np.uint64).astype(np.uint32)
    big_mask = (1 << d) - 1
    return np.array([(big_mask >> (32 * k)) & 0xFFFFFFFF for k in range(n)], dtype=np.uint32) & w


@pytest.mark.parametrize("d", [1, 31, 32, 33, 65, 257, 1000])
def test_vote_special_cases(oracle, d):
    rng = np.random.default_rng(d)
    a, b, c = (random_words(rng, d) for _ in range(3))
    # one voter: the vote is that voter
    assert np.array_equal(oracle.majority_vote([a], d), a)
    # unanimous voters
    assert np.array_equal(oracle.majority_vote([a] * 5, d), a)
    assert np.array_equal(oracle.majority_vote([a] * 4, d), a)
    # three voters: the textbook bitwise majority
    assert np.array_equal(oracle.majority_vote([a, b, c], d), (a & b) | (a & c) | (b & c))
    # two voters: "-" only where both say "-" (a split is "+")
    assert np.array_equal(oracle.majority_vote([a, b], d), a & b)
    # order of the workers does not matter
    ws = [random_words(rng, d) for _ in range(7)]
    v = oracle.majority_vote(ws, d)
    assert np.array_equal(v, oracle.majority_vote(ws[::-1], d))
    assert np.array_equal(v, oracle.majority_vote(ws[3:] + ws[:3], d))
    # odd M: negating every vote negates the outcome
    mask = random_words(np.random.default_rng(0), d) | ~random_words(np.random.default_rng(0), d)
    full = np.array(exact.pack([-1] * d), dtype=np.uint32)
    assert np.array_equal(oracle.majority_vote([w ^ full for w in ws], d), v ^ full)
    del mask
    # monotone: turning one worker's "-" into "+" never creates a "-" outcome
    ws2 = [w.copy() for w in ws]
    ws2[2] &= random_words(rng, d)
    assert not np.any(oracle.majority_vote(ws2, d) & ~v)
    # vote sum: parity of M, bounded by M, consistent with unpack and the vote
    s = oracle.vote_sum(ws, d)
    assert np.all((s - 7) % 2 == 0) and np.all(np.abs(s) <= 7)
    assert np.array_equal(s, sum(oracle.unpack(w, d).astype(np.int32) for w in ws))
    assert np.array_equal(oracle.unpack(v, d) == -1, s < 0)


def test_vote_msb_plane_for_seven_and_fifteen_voters(oracle):
    # with M = 2^k - 1 voters the outcome is the top bit of the count of "-"
    rng = np.random.default_rng(11)
    for M, top in ((7, 4), (15, 8)):
        d = 777
        ws = [random_words(rng, d) for _ in range(M)]
        count = sum((oracle.unpack(w, d) == -1).astype(np.int32) for w in ws)
        v = oracle.unpack(oracle.majority_vote(ws, d), d)
        assert np.array_equal(v == -1, (count & top) != 0)


def normal_cdf(z):
    return 0.5 * math.erfc(-z / math.sqrt(2.0))


def binom_tail_gt_half(M, p):
    """P[Bin(M, p) > M/2]"""
    return sum(math.comb(M, k) * p ** k * (1 - p) ** (M - k) for k in range(M + 1) if 2 * k > M)


def test_remark3_more_workers_make_the_vote_worse(oracle):
    # Section 4, Remark 3: X = 50 w.p. 0.1, -1 w.p. 0.9 has positive mean, yet
    # the vote is "+" only when most workers drew 50: Binomial(M, 0.1) tail.
    c = paper_constants()
    hi, p_hi, lo = c["remark3_value_hi"], c["remark3_prob_hi"], c["remark3_value_lo"]
    assert hi * p_hi + lo * c["remark3_prob_lo"] > 0
    d = 1 << 20
    rng = np.random.default_rng(1802)
    closed = {1: 0.1, 3: 0.028, 7: 0.002728, 15: 3.36e-5}
    last = 1.0
    for M in (1, 3, 7, 15):
        g = [np.where(rng.random(d) < p_hi, hi, lo).astype(np.float32) for _ in range(M)]
        x = np.zeros(d, dtype=np.float32)
        voted = oracle.signum_vote_step(g, None, 0.0, 1.0, x)
        frac_plus = float(np.mean(oracle.unpack(voted, d) == 1))
        p = binom_tail_gt_half(M, p_hi)
        assert abs(p - closed[M]) < 0.01 * closed[M]
        assert abs(frac_plus - p) < 5 * math.sqrt(p * (1 - p) / d) + 1e-9
        assert np.array_equal(x == -1.0, oracle.unpack(voted, d) == 1)   # x - delta*(+1)
        assert frac_plus < last
        last = frac_plus


@pytest.mark.parametrize("S", [0.25, 1.0, 2.0])
def test_gaussian_failure_rates_and_lemma1_bounds(oracle, S):
    # Gaussian noise is unimodal and symmetric, so Lemma 1 bounds the chance
    # that a worker's sign bit is wrong; the true rate is Phi(-S); the vote's
    # failure rate is the binomial tail, bounded by 1/(sqrt(M) S) (proof of
    # Theorem 2(b)).
    d = 1 << 19
    rng = np.random.default_rng(int(S * 100))
    true_sign = np.where(rng.random(d) < 0.5, -1.0, 1.0)
    q = normal_cdf(-S)
    lemma = 2.0 / (9 * S * S) if S > 2 / math.sqrt(3) else 0.5 - S / (2 * math.sqrt(3))
    assert q <= lemma < 0.5
    for M in (1, 7, 15):
        g = [(true_sign * S + rng.standard_normal(d)).astype(np.float32) for _ in range(M)]
        voted, packed = oracle.signum_vote_step(g, None, 0.0, 1e-3, np.zeros(d, np.float32),
                                                want_packed=True)
        wrong_worker = float(np.mean(oracle.unpack(packed[0], d) != true_sign))
        assert abs(wrong_worker - q) < 5 * math.sqrt(q * (1 - q) / d)
        assert wrong_worker <= lemma
        p_fail = binom_tail_gt_half(M, q)          # odd M: wrong iff most are wrong
        wrong_vote = float(np.mean(oracle.unpack(voted, d) != true_sign))
        assert abs(wrong_vote - p_fail) < 5 * math.sqrt(p_fail * (1 - p_fail) / d) + 1e-9
        assert wrong_vote <= 1.0 / (math.sqrt(M) * S)


# --------------------------------------------------------------- apply ----

def test_apply_exact_rational_and_every_coordinate_moves(oracle):
    rng = np.random.default_rng(5)
    d = 300
    x = (rng.standard_normal(d) * 0.05).astype(np.float32)
    x[:4] = [0.0, 1e-4, -1e-4, 1e-45]
    bits = random_words(rng, d)
    delta = f32(1e-4)
    x0 = x.copy()
    oracle.sign_apply(x, bits, float(delta))
    s = oracle.unpack(bits, d)
    for i in range(d):
        assert fr(x[i]) == exact.apply_step(fr(x0[i]), int(s[i]), fr(delta))
    # Theorem 1's proof: every coordinate moves by delta (up to rounding), in
    # the direction opposite to its sign
    moved = x.astype(np.float64) - x0.astype(np.float64)
    assert np.all(np.abs(np.abs(moved) - float(delta)) < 1e-8)
    assert np.array_equal(np.sign(moved), -s)


def test_apply_repeated_steps_walk_linearly(oracle):
    d = 64
    x = np.zeros(d, dtype=np.float32)
    bits = np.array([0x0000FFFF, 0xFFFF0000, 0, 0], dtype=np.uint32)
    for _ in range(100):
        oracle.sign_apply(x, bits, 0.5)        # exact in binary
    s = oracle.unpack(bits, d)
    assert np.array_equal(x, -50.0 * s)


def test_toy_quadratic_noiseless_coordinates_reach_delta_band(oracle):
    # Appendix A, Figure A.1: f(x) = |x|^2 / 2, g(x) = x, Gaussian noise on the
    # first coordinate only, x_0 ~ N(0, I), signSGD with lr 0.01.  A noiseless
    # coordinate walks towards 0 in steps of delta and then stays within delta.
    c = paper_constants()
    d, lr = int(c["toy_d"]), c["toy_lr_signsgd"]
    rng = np.random.default_rng(50)
    x = rng.standard_normal(d).astype(np.float32)
    steps = int(np.max(np.abs(x[1:])) / lr) + 5
    for k in range(steps + 50):
        g = x.copy()
        g[0] += np.float32(c["toy_noise_std"] * rng.standard_normal())
        oracle.signum_vote_step([g], None, 0.0, lr, x)
        if k >= steps:
            assert np.all(np.abs(x[1:]) <= lr * 1.001)
    assert np.all(np.abs(x[1:]) <= lr * 1.001)


# --------------------------------------------------------- whole step ----

@pytest.mark.parametrize("M,d", [(1, 100), (7, 1000), (8, 257), (16, 4133)])
@pytest.mark.parametrize("momentum", [False, True])
def test_step_matches_exact_bruteforce_composition(oracle, M, d, momentum):
    rng = np.random.default_rng(M * 1000 + d)
    beta, delta = f32(0.9), f32(1e-4)
    g = [rand_grad(rng, d) for _ in range(M)]
    m = [rng.standard_normal(d).astype(np.float32) * np.float32(0.1) for _ in range(M)] if momentum else None
    x = (rng.standard_normal(d) * 0.05).astype(np.float32)
    m0 = [a.copy() for a in m] if momentum else None
    x0 = x.copy()
    voted, packed = oracle.signum_vote_step(g, m, float(beta), float(delta), x, want_packed=True)
    n_check = min(d, 300)               # pure python exact arithmetic is slow
    signs = []
    for w in range(M):
        row = []
        for i in range(n_check):
            if momentum:
                v = exact.momentum(fr(beta), fr(m0[w][i]), fr(g[w][i]))
                assert fr(m[w][i]) == v
            else:
                v = fr(g[w][i])
            row.append(exact.sign_of(v))
        signs.append(row)
        assert oracle.unpack(packed[w], d)[:n_check].tolist() == row
    v = exact.vote(signs)
    assert oracle.unpack(voted, d)[:n_check].tolist() == v
    for i in range(n_check):
        assert fr(x[i]) == exact.apply_step(fr(x0[i]), v[i], fr(delta))


@pytest.mark.parametrize("gdt", ["f32", "bf16"])
def test_step_equals_three_calls_and_threaded_split(oracle, gdt):
    rng = np.random.default_rng(9)
    M, d = 5, 70_001
    if gdt == "f32":
        g = [rng.standard_normal(d).astype(np.float32) for _ in range(M)]
    else:
        g = [(rng.standard_normal(d).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16) for _ in range(M)]
    m = [rng.standard_normal(d).astype(np.float32) for _ in range(M)]
    x = rng.standard_normal(d).astype(np.float32)
    # three separate calls
    m3 = [a.copy() for a in m]
    x3 = x.copy()
    p3 = [oracle.signum_pack(g[w], m3[w], 0.9) for w in range(M)]
    v3 = oracle.majority_vote(p3, d)
    oracle.sign_apply(x3, v3, 1e-4)
    for threads in (1, 3, 8):
        mf = [a.copy() for a in m]
        xf = x.copy()
        vf, pf = oracle.signum_vote_step(g, mf, 0.9, 1e-4, xf, want_packed=True, threads=threads)
        assert np.array_equal(vf, v3) and np.array_equal(xf, x3)
        assert all(np.array_equal(a, b) for a, b in zip(mf, m3))
        assert all(np.array_equal(a, b) for a, b in zip(pf, p3))


@pytest.mark.parametrize("d", [1, 31, 4_099, 262_144 + 33, 1_300_007])
@pytest.mark.parametrize("gdt,momentum", [("f32", True), ("bf16", True), ("f32", False)])
def test_threaded_wrapper_equals_the_scalar_routine(oracle, d, gdt, momentum):
    """The large GPU tests use the threaded wrapper with 16 threads as their reference: it must
    return exactly what the scalar routine (the one the pins above hold) returns, whatever the
    thread count and wherever the cuts between threads fall (sizes below, at and far above one
    word per thread; more threads than words)."""
    rng = np.random.default_rng(d)
    M = 4
    if gdt == "f32":
        g = [rng.standard_normal(d).astype(np.float32) for _ in range(M)]
    else:
        g = [(rng.standard_normal(d).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16) for _ in range(M)]
    m0 = [rng.standard_normal(d).astype(np.float32) * np.float32(0.2) for _ in range(M)] if momentum else None
    x0 = rng.standard_normal(d).astype(np.float32)
    m1 = [a.copy() for a in m0] if momentum else None
    x1 = x0.copy()
    v1, p1 = oracle.signum_vote_step(g, m1, 0.9, 1e-3, x1, want_packed=True, threads=1)
    for threads in (2, 16, 64):
        mt = [a.copy() for a in m0] if momentum else None
        xt = x0.copy()
        vt, pt = oracle.signum_vote_step(g, mt, 0.9, 1e-3, xt, want_packed=True, threads=threads)
        assert np.array_equal(vt, v1) and np.array_equal(xt.view(np.uint32), x1.view(np.uint32)), threads
        assert all(np.array_equal(a, b) for a, b in zip(pt, p1)), threads
        if momentum:
            assert all(np.array_equal(a.view(np.uint32), b.view(np.uint32)) for a, b in zip(mt, m1)), threads


def test_empty_input_is_a_no_op(oracle):
    e = np.empty(0, dtype=np.float32)
    assert oracle.packed_words(0) == 0 and oracle.packed_bytes(0) == 0
    assert len(oracle.signum_pack(e, None, 0.0)) == 0
    assert len(oracle.signum_vote_step([e, e], None, 0.0, 0.1, e.copy())) == 0


def test_packed_sizes(oracle):
    for d, words, nbytes in ((1, 1, 16), (32, 1, 16), (33, 2, 16), (128, 4, 16), (129, 5, 32),
                             (272_474, 8515, 34064), (1_500_000_017, 46_875_001, 187_500_016)):
        assert oracle.packed_words(d) == words
        assert oracle.packed_bytes(d) == nbytes
