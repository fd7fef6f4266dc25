"""GPU parity at vector sizes where the library changes launch shape.

The kernels that stream one or a few buffers (pack, apply, Welford, copy, the
stand-alone votes) take other tilings - fewer rows per block, a cap on the
blocks per compute unit - once the vector is large (2^27, 2^28 or 2^30
coordinates depending on the entry point).  The arithmetic is the same code;
what changes is which block owns which coordinates and where the ragged end
begins.  Each test runs one entry point just above its threshold, with a
ragged end, and compares every output element with the CPU oracle.
"""
import numpy as np
import pytest
import torch

import synth
from test_gpu_parity import DEV, assert_same_floats, bits_np, dirty_bits

pytestmark = pytest.mark.gpu

D28 = (1 << 28) + 4099      # above the 2^28 threshold; d mod 1024 = 3, d mod 32 = 3
D27 = (1 << 27) + 77
D30 = (1 << 30) + 33


@pytest.fixture(scope="module")
def ss():
    import paper_1802_04434_amd as lib
    lib.load_library()
    return lib


def device_normal(d, seed, scale=1.0, dtype=torch.float32):
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    out = torch.empty(d, device=DEV, dtype=dtype)
    step = 1 << 26
    for a in range(0, d, step):
        n = min(step, d - a)
        out[a:a + n] = (torch.randn(n, device=DEV, generator=gen) * scale).to(dtype)
    # zeros of both signs and subnormals at the start, in the middle and in the ragged end
    if dtype == torch.float32:
        special = torch.tensor([0x00000000, -0x80000000, 0x00000001, -0x7FFFFFFF, 0x007FFFFF, -0x7F800001],
                               dtype=torch.int32, device=DEV)
        for pos in (0, d // 2, d - 6):
            out.view(torch.int32)[pos:pos + 6] = special
    return out


def device_words(n, seed):
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    return torch.randint(-2**31, 2**31 - 1, (n,), dtype=torch.int32, device=DEV, generator=gen)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_pack_large(ss, oracle, dtype):
    d = D28
    g = device_normal(d, 11, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32)
    m_dev = device_normal(d, 12, 0.3)
    m = synth.as_numpy(m_dev).copy()
    packed = dirty_bits(ss, d)
    ss.signum_pack(g, m_dev, 0.9, packed)
    want = oracle.signum_pack(synth.as_numpy(g), m, 0.9)
    assert np.array_equal(bits_np(packed), want)
    assert_same_floats(m_dev, m, "momentum")


@pytest.mark.parametrize("momentum", [False, True])
def test_fused_step_one_worker_large(ss, oracle, momentum):
    d = D27
    g = device_normal(d, 13)
    x_dev = device_normal(d, 14, 0.05)
    x = synth.as_numpy(x_dev).copy()
    m_dev = [device_normal(d, 15, 0.3)] if momentum else None
    m = [synth.as_numpy(m_dev[0]).copy()] if momentum else None
    voted = dirty_bits(ss, d)
    ss.signum_vote_step([g], m_dev, 0.9, 1e-4, x_dev, voted, None)
    want = oracle.signum_vote_step([synth.as_numpy(g)], m, 0.9, 1e-4, x, threads=16)
    assert np.array_equal(bits_np(voted), want[0] if isinstance(want, tuple) else want)
    assert_same_floats(x_dev, x, "x")
    if momentum:
        assert_same_floats(m_dev[0], m[0], "momentum")


def test_pack_ternary_large(ss, oracle):
    d = D28
    g = device_normal(d, 21)
    m_dev = device_normal(d, 22, 0.3)
    m = synth.as_numpy(m_dev).copy()
    neg, zero = dirty_bits(ss, d), dirty_bits(ss, d)
    ss.signum_pack_ternary(g, m_dev, 0.9, 0.05, neg, zero)
    want_neg, want_zero = oracle.signum_pack_ternary(synth.as_numpy(g), m, 0.9, 0.05)
    assert np.array_equal(bits_np(neg), want_neg)
    assert np.array_equal(bits_np(zero), want_zero)
    assert_same_floats(m_dev, m, "momentum")


def test_apply_kernels_large(ss, oracle):
    d = D28
    n = ss.packed_bytes(d) // 4
    b1, b2 = device_words(n, 31), device_words(n, 32)
    h1, h2 = bits_np(b1).copy(), bits_np(b2).copy()
    x_dev = device_normal(d, 33, 0.05)
    x = synth.as_numpy(x_dev).copy()
    ss.sign_apply(x_dev, b1, 1e-4)
    oracle.sign_apply(x, h1, 1e-4)
    assert_same_floats(x_dev, x, "x after sign_apply")
    ss.ternary_apply(x_dev, b1, b2, 3e-4)
    oracle.ternary_apply(x, h1, h2, 3e-4)
    assert_same_floats(x_dev, x, "x after ternary_apply")
    gen = torch.Generator(device=DEV)
    gen.manual_seed(34)
    sums = torch.randint(-64, 65, (d,), dtype=torch.int8, device=DEV, generator=gen)
    ss.sum_apply(x_dev, sums, 1e-5)
    oracle.sum_apply(x, sums.cpu().numpy(), 1e-5)
    assert_same_floats(x_dev, x, "x after sum_apply")


def test_welford_large(ss, oracle):
    d = D27
    mean_dev, m2_dev = torch.zeros(d, device=DEV), torch.zeros(d, device=DEV)
    mean, m2 = np.zeros(d, np.float32), np.zeros(d, np.float32)
    for n in (1, 2, 3):
        g = device_normal(d, 40 + n, 2.0)
        ss.welford_update(g, mean_dev, m2_dev, n)
        oracle.welford_update(synth.as_numpy(g), mean, m2, n)
    assert_same_floats(mean_dev, mean, "mean")
    assert_same_floats(m2_dev, m2, "m2")
    sigma = torch.full((d,), -1.0, device=DEV)
    ss.welford_sigma(m2_dev, 3, sigma)
    assert_same_floats(sigma, oracle.welford_sigma(m2, 3), "sigma")


def test_stream_copy_large_and_small(ss):
    for nbytes in ((1 << 30) + 16 * 4099, (1 << 24) + 16 * 3, 16):
        src = device_words(nbytes // 4, 51)
        dst = torch.full((nbytes // 4 + 4,), -1, dtype=torch.int32, device=DEV)
        ss.stream_copy(dst, src, nbytes)
        assert torch.equal(dst[:nbytes // 4], src)
        assert bool((dst[nbytes // 4:] == -1).all())      # nothing beyond the end


@pytest.mark.parametrize("M", [3, 17])
def test_vote_sum_and_quorum_vote_large(ss, oracle, M):
    d = D27
    n = ss.packed_bytes(d) // 4
    neg = [device_words(n, 60 + w) for w in range(M)]
    zero = [device_words(n, 80 + w) for w in range(M)]
    hneg, hzero = [bits_np(t).copy() for t in neg], [bits_np(t).copy() for t in zero]
    sums = torch.full((d,), 99, dtype=torch.int8, device=DEV)
    ss.vote_sum(neg, sums, d)
    assert np.array_equal(sums.cpu().numpy().astype(np.int32), oracle.vote_sum(hneg, d))
    vn, vz = dirty_bits(ss, d), dirty_bits(ss, d)
    ss.quorum_vote(neg, zero, 2, vn, vz, d)
    want_n, want_z = oracle.quorum_vote(hneg, hzero, 2, d)
    assert np.array_equal(bits_np(vn), want_n)
    assert np.array_equal(bits_np(vz), want_z)


@pytest.mark.parametrize("M", [3, 17])
def test_majority_vote_large(ss, oracle, M):
    d = D30
    n = ss.packed_bytes(d) // 4
    packed = [device_words(n, 90 + w) for w in range(M)]
    voted = dirty_bits(ss, d)
    ss.majority_vote(packed, voted, d)
    want = oracle.majority_vote([bits_np(t).copy() for t in packed], d)
    assert np.array_equal(bits_np(voted), want)
