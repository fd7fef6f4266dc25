"""GPU parity on seeded random argument combinations.

The other GPU tests walk each argument along its own axis (sizes, worker
counts, gradient types, flags, optional outputs).  Here the combinations are
drawn at random from a fixed seed - every d from one coordinate to a few
million, every M up to 64, both gradient types, with and without momentum,
every flag combination, each optional output present or not, odd values of
beta and delta - and every output of every step is compared with the CPU
oracle, bit for bit.  The ternary step gets the same treatment.
"""
import numpy as np
import pytest
import torch

import synth
from test_gpu_parity import DEV, assert_same_floats, bits_np, dirty_bits, make_grad, make_momentum

pytestmark = pytest.mark.gpu

N_CASES = 60


@pytest.fixture(scope="module")
def ss():
    import paper_1802_04434_amd as lib
    lib.load_library()
    return lib


def draw_case(rng):
    # sizes: mostly small and ragged, some around the tile sizes, a few in the streaming range
    kind = rng.integers(0, 10)
    if kind < 5:
        d = int(rng.integers(1, 5000))
    elif kind < 8:
        d = int(rng.choice([1024, 2048, 4096, 8192, 65536]) * rng.integers(1, 8) + rng.integers(-40, 41))
    else:
        d = int((1 << 20) + rng.integers(0, 1 << 21))
    big = d >= (1 << 20)
    M = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 9, 11, 16, 17] if big else
                       [1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 13, 16, 17, 25, 32, 33, 48, 63, 64]))
    return dict(d=max(d, 1), M=M, dtype=str(rng.choice(["f32", "bf16"])), momentum=bool(rng.integers(0, 2)),
                flags=int(rng.integers(0, 4)), want_packed=bool(rng.integers(0, 2)), want_sums=bool(rng.integers(0, 2)),
                beta=float(rng.choice([0.0, 0.5, 0.9, 0.99, 0.123])), delta=float(rng.choice([1e-4, 3e-3, 0.25, 1e-7])),
                steps=int(rng.integers(1, 4)))


@pytest.mark.parametrize("case", range(N_CASES))
def test_random_step(ss, oracle, case):
    rng = np.random.default_rng(9000 + case)
    c = draw_case(rng)
    d, M = c["d"], c["M"]
    m = [make_momentum(rng, d) for _ in range(M)] if c["momentum"] else None
    x = (rng.standard_normal(d) * 0.05).astype(np.float32)
    m_dev = [torch.from_numpy(a).to(DEV) for a in m] if m is not None else None
    x_dev = torch.from_numpy(x).to(DEV)
    for k in range(c["steps"]):
        g = [make_grad(rng, d, c["dtype"], scale=0.5) for _ in range(M)]
        voted = dirty_bits(ss, d)
        packed = [dirty_bits(ss, d) for _ in range(M)] if c["want_packed"] else None
        sums = torch.full((d,), 99, dtype=torch.int8, device=DEV) if c["want_sums"] else None
        ss.signum_vote_step_ex([t.to(DEV) for t in g], m_dev, c["beta"], c["delta"], x_dev, voted, packed, sums, c["flags"])
        want_voted, want_packed, want_sums = oracle.signum_vote_step_ex(
            [synth.as_numpy(t) for t in g], m, c["beta"], c["delta"], x, c["flags"])
        assert np.array_equal(bits_np(voted), want_voted), (c, "voted", k)
        if packed is not None:
            for w in range(M):
                assert np.array_equal(bits_np(packed[w]), want_packed[w]), (c, "packed", k, w)
        if sums is not None:
            assert np.array_equal(sums.cpu().numpy(), want_sums), (c, "sums", k)
        if m is not None:
            for w in range(M):
                assert_same_floats(m_dev[w], m[w], "%s m[%d] step %d" % (c, w, k))
        assert_same_floats(x_dev, x, "%s x step %d" % (c, k))


@pytest.mark.parametrize("case", range(N_CASES // 2))
def test_random_ternary_step(ss, oracle, case):
    rng = np.random.default_rng(7000 + case)
    c = draw_case(rng)
    d, M = c["d"], c["M"]
    tau = float(rng.choice([0.0, 0.05, 0.3, 10.0]))
    quorum = int(rng.integers(1, M + 3))
    m = [make_momentum(rng, d) for _ in range(M)] if c["momentum"] else None
    x = (rng.standard_normal(d) * 0.05).astype(np.float32)
    m_dev = [torch.from_numpy(a).to(DEV) for a in m] if m is not None else None
    x_dev = torch.from_numpy(x).to(DEV)
    for k in range(c["steps"]):
        g = [make_grad(rng, d, c["dtype"], scale=0.5) for _ in range(M)]
        vn, vz = dirty_bits(ss, d), dirty_bits(ss, d)
        ss.signum_vote_step_ternary([t.to(DEV) for t in g], m_dev, c["beta"], tau, quorum, c["delta"], x_dev, vn, vz)
        want_n, want_z = oracle.signum_vote_step_ternary([synth.as_numpy(t) for t in g], m, c["beta"], tau, quorum,
                                                         c["delta"], x)
        assert np.array_equal(bits_np(vn), want_n), (c, tau, quorum, "neg", k)
        assert np.array_equal(bits_np(vz), want_z), (c, tau, quorum, "zero", k)
        if m is not None:
            for w in range(M):
                assert_same_floats(m_dev[w], m[w], "%s m[%d] step %d" % (c, w, k))
        assert_same_floats(x_dev, x, "%s x step %d" % (c, k))
