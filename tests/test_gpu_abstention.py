"""GPU parity for majority vote with abstention (the ternary extension sketched
in Section 6 of arxiv 1802.04434, under this build's reading of it): every
output bit and float against the CPU oracle."""
import numpy as np
import pytest
import torch

import synth
from test_gpu_parity import DEV, RAGGED, assert_same_floats, bits_np, dirty_bits, make_grad, make_momentum

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ss():
    import paper_1802_04434_amd as lib
    lib.load_library()
    return lib


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("momentum", [False, True])
@pytest.mark.parametrize("d", [1, 33, 1000, 4099, 70_001, 1_200_003])
def test_pack_ternary(ss, oracle, d, momentum, dtype):
    rng = np.random.default_rng(d)
    g = make_grad(rng, d, dtype)
    m = make_momentum(rng, d) if momentum else None
    m_dev = torch.from_numpy(m).to(DEV) if momentum else None
    for tau in (0.0, 0.25):
        neg, zero = dirty_bits(ss, d), dirty_bits(ss, d)
        ss.signum_pack_ternary(g.to(DEV), m_dev, 0.9, tau, neg, zero)
        want_neg, want_zero = oracle.signum_pack_ternary(synth.as_numpy(g), m, 0.9, tau)
        assert np.array_equal(bits_np(neg), want_neg) and np.array_equal(bits_np(zero), want_zero)
        if momentum:
            assert_same_floats(m_dev, m, "m")


@pytest.mark.parametrize("M", [1, 2, 3, 7, 8, 16, 33, 64])
def test_quorum_vote_and_apply(ss, oracle, M):
    for d in (1, 97, 4099, 262_144 + 5):
        rng = np.random.default_rng(M * 11 + d)
        n = ss.packed_bytes(d) // 4
        # random planes, including words where both planes are set (zero wins) and garbage padding
        neg = [rng.integers(0, 1 << 32, n, dtype=np.uint64).astype(np.uint32) for _ in range(M)]
        zero = [(rng.integers(0, 1 << 32, n, dtype=np.uint64) & rng.integers(0, 1 << 32, n, dtype=np.uint64))
                .astype(np.uint32) for _ in range(M)]
        to_dev = lambda a: torch.from_numpy(a.view(np.int32)).to(DEV)
        for Q in sorted({1, 2, max(1, M // 2), M + 1}):
            vneg, vzero = dirty_bits(ss, d), dirty_bits(ss, d)
            ss.quorum_vote([to_dev(a) for a in neg], [to_dev(a) for a in zero], Q, vneg, vzero, d)
            want_neg, want_zero = oracle.quorum_vote(neg, zero, Q, d)
            assert np.array_equal(bits_np(vneg), want_neg), (M, d, Q)
            assert np.array_equal(bits_np(vzero), want_zero), (M, d, Q)
        x = (rng.standard_normal(d) * 0.05).astype(np.float32)
        x_dev = torch.from_numpy(x).to(DEV)
        ss.ternary_apply(x_dev, vneg, vzero, 1e-3)
        oracle.ternary_apply(x, want_neg, want_zero, 1e-3)
        assert_same_floats(x_dev, x, "x")


def run_ternary(ss, oracle, M, d, dtype, momentum, tau, Q, seed, steps=2):
    rng = np.random.default_rng(seed)
    m = [make_momentum(rng, d) for _ in range(M)] if momentum else None
    x = (rng.standard_normal(d) * 0.05).astype(np.float32)
    m_dev = [torch.from_numpy(a).to(DEV) for a in m] if momentum else None
    x_dev = torch.from_numpy(x).to(DEV)
    for k in range(steps):
        g = [make_grad(rng, d, dtype, scale=0.5) for _ in range(M)]
        vneg, vzero = dirty_bits(ss, d), dirty_bits(ss, d)
        ss.signum_vote_step_ternary([t.to(DEV) for t in g], m_dev, 0.9, tau, Q, 1e-3, x_dev, vneg, vzero)
        want_neg, want_zero = oracle.signum_vote_step_ternary([synth.as_numpy(t) for t in g], m, 0.9, tau, Q, 1e-3, x)
        assert np.array_equal(bits_np(vneg), want_neg), ("neg", k)
        assert np.array_equal(bits_np(vzero), want_zero), ("zero", k)
        if momentum:
            for w in range(M):
                assert_same_floats(m_dev[w], m[w], "m[%d] step %d" % (w, k))
        assert_same_floats(x_dev, x, "x step %d" % k)


@pytest.mark.parametrize("M,dtype,momentum,tau,Q", [(1, "f32", True, 0.1, 1), (3, "f32", True, 0.2, 2),
                                                    (7, "f32", True, 0.15, 3), (8, "bf16", True, 0.3, 1),
                                                    (16, "f32", False, 0.4, 4), (33, "bf16", False, 0.0, 1)])
def test_fused_ternary_step(ss, oracle, M, dtype, momentum, tau, Q):
    for d in (777, 20_000 + 13):
        run_ternary(ss, oracle, M, d, dtype, momentum, tau, Q, seed=M * 10 + d)


@pytest.mark.parametrize("d", RAGGED)
def test_fused_ternary_step_ragged(ss, oracle, d):
    run_ternary(ss, oracle, 5, d, "f32", True, 0.2, 2, seed=d, steps=1)


def test_fused_ternary_step_streaming_shape_and_reduction_to_algorithm_3(ss, oracle):
    run_ternary(ss, oracle, 7, 2_200_000 + 37, "f32", True, 0.2, 3, seed=1, steps=2)
    # tau = 0, quorum 1, odd M: the plain majority vote step
    d, M = 1_100_003, 7
    gen = torch.Generator(device=DEV)
    gen.manual_seed(3)
    g = [torch.randn(d, device=DEV, generator=gen) for _ in range(M)]
    m0 = [torch.randn(d, device=DEV, generator=gen) * 0.3 for _ in range(M)]
    x0 = torch.randn(d, device=DEV, generator=gen)
    ma, xa, va = [t.clone() for t in m0], x0.clone(), dirty_bits(ss, d)
    ss.signum_vote_step(g, ma, 0.9, 1e-3, xa, va)
    mb, xb, vneg, vzero = [t.clone() for t in m0], x0.clone(), dirty_bits(ss, d), dirty_bits(ss, d)
    ss.signum_vote_step_ternary(g, mb, 0.9, 0.0, 1, 1e-3, xb, vneg, vzero)
    assert torch.equal(va, vneg) and not vzero.any() and torch.equal(xa, xb)
    assert all(torch.equal(p, q) for p, q in zip(ma, mb))
