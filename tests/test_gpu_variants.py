"""GPU parity for the variants of the step: Theorem 3's warm-up iteration and
Section 4's "(good)" update with the vote sum, against the CPU oracle, bit for
bit (arxiv 1802.04434)."""
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
@pytest.mark.parametrize("d", [1, 33, 1000, 4099, 70_001, 2_100_003])
def test_signum_pack_warmup(ss, oracle, d, dtype):
    rng = np.random.default_rng(d)
    g = make_grad(rng, d, dtype)
    m = make_momentum(rng, d)
    m_dev = torch.from_numpy(m).to(DEV)
    packed = dirty_bits(ss, d)
    ss.signum_pack_warmup(g.to(DEV), m_dev, 0.9, packed)
    want = oracle.signum_pack_warmup(synth.as_numpy(g), m, 0.9)
    assert np.array_equal(bits_np(packed), want)
    assert_same_floats(m_dev, m, "m")
    # without momentum it is the plain sign of the gradient
    ss.signum_pack_warmup(g.to(DEV), None, 0.9, packed)
    assert np.array_equal(bits_np(packed), oracle.signum_pack(synth.as_numpy(g), None, 0.0))


@pytest.mark.parametrize("M", [1, 2, 3, 7, 8, 16, 33, 64])
def test_vote_sum_and_sum_apply(ss, oracle, M):
    for d in (1, 15, 16, 17, 97, 4099, 300_000 + 9):
        rng = np.random.default_rng(M * 13 + d)
        n = ss.packed_bytes(d) // 4
        words = [rng.integers(0, 1 << 32, n, dtype=np.uint64).astype(np.uint32) for _ in range(M)]
        dev = [torch.from_numpy(w.view(np.int32)).to(DEV) for w in words]
        sums = torch.full((d,), 99, dtype=torch.int8, device=DEV)
        ss.vote_sum(dev, sums, d)
        want = oracle.vote_sum(words, d)
        got = sums.cpu().numpy()
        assert np.array_equal(got.astype(np.int32), want), (M, d)
        x = (rng.standard_normal(d) * 0.05).astype(np.float32)
        x_dev = torch.from_numpy(x).to(DEV)
        ss.sum_apply(x_dev, sums, 1e-4)
        oracle.sum_apply(x, got, 1e-4)
        assert_same_floats(x_dev, x, "x")


def run_variant(ss, oracle, M, d, dtype, momentum, flags, seed, steps=2, delta=1e-3):
    rng = np.random.default_rng(seed)
    m = [make_momentum(rng, d) for _ in range(M)] if momentum else None
    x = (rng.standard_normal(d) * 0.05).astype(np.float32)
    m_dev = [torch.from_numpy(a).to(DEV) for a in m] if momentum else None
    x_dev = torch.from_numpy(x).to(DEV)
    for k in range(steps):
        g = [make_grad(rng, d, dtype, scale=0.5) for _ in range(M)]
        voted = dirty_bits(ss, d)
        packed = [dirty_bits(ss, d) for _ in range(M)]
        sums = torch.full((d,), 99, dtype=torch.int8, device=DEV)
        ss.signum_vote_step_ex([t.to(DEV) for t in g], m_dev, 0.9, delta, x_dev, voted, packed, sums, flags)
        want_voted, want_packed, want_sums = oracle.signum_vote_step_ex(
            [synth.as_numpy(t) for t in g], m, 0.9, delta, x, flags)
        assert np.array_equal(bits_np(voted), want_voted), ("voted", k)
        for w in range(M):
            assert np.array_equal(bits_np(packed[w]), want_packed[w]), ("packed", k, w)
            if momentum:
                assert_same_floats(m_dev[w], m[w], "m[%d] step %d" % (w, k))
        assert np.array_equal(sums.cpu().numpy(), want_sums), ("sums", k)
        assert_same_floats(x_dev, x, "x step %d" % k)


@pytest.mark.parametrize("flags", [1, 2, 3])
@pytest.mark.parametrize("M,dtype,momentum", [(1, "f32", True), (2, "f32", False), (7, "f32", True),
                                              (8, "bf16", True), (16, "f32", True), (20, "bf16", False)])
def test_step_variants_small_and_ragged(ss, oracle, M, dtype, momentum, flags):
    for d in (777, 20_000 + 13):
        run_variant(ss, oracle, M, d, dtype, momentum, flags, seed=M * 100 + flags * 7 + d)


@pytest.mark.parametrize("flags", [1, 2, 3])
def test_step_variants_streaming_shape(ss, oracle, flags):
    # large enough for the one-worker-at-a-time launch shape, with a ragged tail
    run_variant(ss, oracle, 7, 2_200_000 + 37, "f32", True, flags, seed=flags, steps=2)
    run_variant(ss, oracle, 9, 1_500_000 + 5, "bf16", True, flags, seed=10 + flags, steps=1)


@pytest.mark.parametrize("d", RAGGED)
def test_step_variants_ragged(ss, oracle, d):
    run_variant(ss, oracle, 5, d, "f32", True, 3, seed=d, steps=1)


def test_flags_zero_is_the_plain_step_and_sums_are_optional(ss):
    d, M = 300_001, 7
    gen = torch.Generator(device=DEV)
    gen.manual_seed(7)
    g = [torch.randn(d, device=DEV, generator=gen) for _ in range(M)]
    m0 = [torch.randn(d, device=DEV, generator=gen) * 0.3 for _ in range(M)]
    x0 = torch.randn(d, device=DEV, generator=gen)
    ma, xa, va = [t.clone() for t in m0], x0.clone(), dirty_bits(ss, d)
    ss.signum_vote_step(g, ma, 0.9, 1e-3, xa, va)
    mb, xb, vb = [t.clone() for t in m0], x0.clone(), dirty_bits(ss, d)
    sums = torch.zeros(d, dtype=torch.int8, device=DEV)
    ss.signum_vote_step_ex(g, mb, 0.9, 1e-3, xb, vb, None, sums, 0)
    assert torch.equal(va, vb) and torch.equal(xa, xb)
    assert all(torch.equal(p, q) for p, q in zip(ma, mb))
    # the sums agree with the stand-alone kernel on the per-worker bits
    packed = [dirty_bits(ss, d) for _ in range(M)]
    mc, xc, vc = [t.clone() for t in m0], x0.clone(), dirty_bits(ss, d)
    ss.signum_vote_step(g, mc, 0.9, 1e-3, xc, vc, packed)
    sums2 = torch.zeros(d, dtype=torch.int8, device=DEV)
    ss.vote_sum(packed, sums2, d)
    assert torch.equal(sums, sums2)
    # "(good)" through the fused call equals vote_sum + sum_apply
    md, xd, vd = [t.clone() for t in m0], x0.clone(), dirty_bits(ss, d)
    ss.signum_vote_step_ex(g, md, 0.9, 1e-3, xd, vd, None, None, ss.STEP_SUM_UPDATE)
    xe = x0.clone()
    ss.sum_apply(xe, sums2, 1e-3)
    assert torch.equal(xd.view(torch.int32), xe.view(torch.int32)) and torch.equal(vd, va)


def test_warmup_schedule_of_theorem_3(ss, oracle):
    # the first C(beta) iterations step with sign(g), later ones with sign(m);
    # beta = 0.5 keeps the warm-up short (C = 1) so both regimes are exercised
    beta = 0.5
    C = ss.warmup_length(beta)
    assert C == oracle.warmup_length(beta) == 1 and ss.warmup_length(0.9) == 54
    cfg = synth.C1.scaled(d=40_003, steps=4)
    m_dev = [torch.zeros(cfg.d, device=DEV) for _ in range(cfg.M)]
    x_dev = synth.x0_chunk(cfg, 0, DEV)
    m = [np.zeros(cfg.d, np.float32) for _ in range(cfg.M)]
    x = x_dev.cpu().numpy().copy()
    for k in range(cfg.steps):
        flags = ss.STEP_WARMUP if k < C else 0
        g_dev = [synth.grad_chunk(cfg, k, w, 0, DEV) for w in range(cfg.M)]
        voted = dirty_bits(ss, cfg.d)
        ss.signum_vote_step_ex(g_dev, m_dev, beta, cfg.delta, x_dev, voted, None, None, flags)
        want_voted, _, _ = oracle.signum_vote_step_ex([synth.as_numpy(t) for t in g_dev], m, beta, cfg.delta, x, flags)
        assert np.array_equal(bits_np(voted), want_voted)
        assert_same_floats(x_dev, x, "x")
        for w in range(cfg.M):
            assert_same_floats(m_dev[w], m[w], "m")
