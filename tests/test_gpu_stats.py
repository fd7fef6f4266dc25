"""GPU parity for the gradient statistics of Section 3 (arxiv 1802.04434):
Welford's update and sigma bit for bit against the CPU oracle; the density of
equation (1) within the tolerance its fp64 sums allow."""
import math

import numpy as np
import pytest
import torch

import synth
from test_gpu_parity import DEV, RAGGED, assert_same_floats

pytestmark = pytest.mark.gpu

# Both sums add exact, non-negative fp64 terms, so every rounding error has the
# same sign bound: relative error <= (number of additions on the longest chain)
# * 2^-53.  A lane adds the 32 elements of a tile, then the tile to its running
# sum: 32 + (tiles per block) + (at most one tail element per 131,072) additions,
# with at most 256 blocks of 16,384 coordinates per tile; then 6 + 7 additions
# combine lanes and waves, and the last block adds 1 + 6 + 7 more.  At
# d = 2^31 that is under 600 roundings of 2^-53 each, < 1e-13; the tolerance
# leaves a factor of ten.  The oracle accumulates in 80-bit long double (its own
# error is 2^-11 of that).
DENSITY_RTOL = 1e-12


@pytest.fixture(scope="module")
def ss():
    import paper_1802_04434_amd as lib
    lib.load_library()
    return lib


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d", [1, 3, 33, 1000, 2048, 4099, 70_001, 1_300_007])
def test_welford_update_and_sigma(ss, oracle, d, dtype):
    rng = np.random.default_rng(d)
    mean = np.zeros(d, np.float32)
    m2 = np.zeros(d, np.float32)
    mean_dev = torch.zeros(d, device=DEV)
    m2_dev = torch.zeros(d, device=DEV)
    for n in range(1, 6):
        # Gaussian samples plus zeros and subnormals of both signs (nothing that
        # overflows: the bit pattern of a NaN is not part of the contract)
        g = (rng.standard_normal(d) * 2.0).astype(np.float32)
        k = min(d, 6)
        g.view(np.uint32)[rng.permutation(d)[:k]] = np.array(
            [0x00000000, 0x80000000, 0x00000001, 0x80000001, 0x007FFFFF, 0x807FFFFF], np.uint32)[:k]
        g = torch.from_numpy(g)
        if dtype == "bf16":
            g = g.to(torch.bfloat16)
        ss.welford_update(g.to(DEV), mean_dev, m2_dev, n)
        oracle.welford_update(synth.as_numpy(g), mean, m2, n)
        assert_same_floats(mean_dev, mean, "mean after %d" % n)
        assert_same_floats(m2_dev, m2, "m2 after %d" % n)
    sigma_dev = torch.full((d,), -1.0, device=DEV)
    ss.welford_sigma(m2_dev, 5, sigma_dev)
    assert_same_floats(sigma_dev, oracle.welford_sigma(m2, 5), "sigma")


@pytest.fixture(scope="module")
def ws(ss):
    # one workspace for the whole module: every call must leave it ready for the next
    return ss.new_density_workspace(DEV)


@pytest.mark.parametrize("d", [0] + RAGGED + [9_000_011])
def test_density(ss, oracle, ws, d):
    rng = np.random.default_rng(d + 1)
    v = (rng.standard_normal(d) * 10.0 ** rng.integers(-3, 3, d)).astype(np.float32)
    out = torch.full((3,), -1.0, dtype=torch.float64, device=DEV)
    ss.density(torch.from_numpy(v).to(DEV) if d else torch.zeros(4, device=DEV), out, ws, d=d)
    got = out.cpu().numpy()
    want = oracle.density(v)
    assert got[0] == pytest.approx(want[0], rel=DENSITY_RTOL)
    assert got[1] == pytest.approx(want[1], rel=DENSITY_RTOL)
    assert got[2] == pytest.approx(want[2], rel=3 * DENSITY_RTOL)


def test_density_is_the_same_bits_on_every_run(ss, ws):
    # the order of every addition depends on d alone: repeated runs, runs after a
    # call of another size on the same workspace, and a fresh workspace all agree
    gen = torch.Generator(device=DEV)
    gen.manual_seed(11)
    for d in (1, 4099, 1_300_007, 25_557_032):
        v = torch.randn(d, device=DEV, generator=gen) * 3.0
        outs = []
        for rep in range(6):
            out = torch.full((3,), -1.0, dtype=torch.float64, device=DEV)
            if rep == 3:      # another size in between
                ss.density(v, out, ws, d=max(1, d // 3))
            work = ss.new_density_workspace(DEV) if rep == 5 else ws
            ss.density(v, out, work)
            outs.append(out.cpu().numpy().view(np.uint64).copy())
        for o in outs[1:]:
            assert np.array_equal(o, outs[0]), d
        assert int(ws[0]) == 0                                   # the ticket is back at zero


def test_density_special_vectors(ss, ws):
    out = torch.empty(3, dtype=torch.float64, device=DEV)
    d = 5_000_001
    ss.density(torch.full((d,), -2.5, device=DEV), out, ws)
    assert out.cpu().tolist() == [2.5 * d, 6.25 * d, 1.0]                       # fully dense
    hot = torch.zeros(d, device=DEV)
    hot[d - 1] = 3.0
    ss.density(hot, out, ws)
    assert out.cpu().tolist() == [3.0, 9.0, 9.0 / (d * 9.0)]                   # one-hot: 1/d
    ss.density(torch.zeros(d, device=DEV), out, ws)
    assert out.cpu().tolist() == [0.0, 0.0, 0.0]


def test_gradient_and_noise_density_of_a_synthetic_run(ss, oracle, ws):
    # what Figure 1 measures, on the C3 recipe: Welford over K stochastic
    # gradients of one worker, then phi(mean) and phi(sigma).  The mean of
    # Gaussian gradients around a Gaussian mu is Gaussian: phi -> 2/pi; sigma
    # is a scaled chi with K-1 degrees of freedom: phi -> E[chi]^2 / E[chi^2].
    cfg = synth.C3.scaled(d=3_000_017)
    K = 16
    mean = torch.zeros(cfg.d, device=DEV)
    m2 = torch.zeros(cfg.d, device=DEV)
    mean_h = np.zeros(cfg.d, np.float32)
    m2_h = np.zeros(cfg.d, np.float32)
    for k in range(K):
        g = synth.grad_chunk(cfg, k, 0, 0, DEV)
        ss.welford_update(g, mean, m2, k + 1)
        oracle.welford_update(synth.as_numpy(g), mean_h, m2_h, k + 1)
    assert_same_floats(mean, mean_h, "mean")
    assert_same_floats(m2, m2_h, "m2")
    sigma = torch.empty_like(m2)
    ss.welford_sigma(m2, K, sigma)
    out = torch.empty(3, dtype=torch.float64, device=DEV)
    ss.density(mean, out, ws)
    phi_g = float(out[2])
    assert phi_g == pytest.approx(oracle.density(mean_h)[2], rel=3 * DENSITY_RTOL)
    ss.density(sigma, out, ws)
    phi_s = float(out[2])
    assert phi_s == pytest.approx(oracle.density(oracle.welford_sigma(m2_h, K))[2], rel=3 * DENSITY_RTOL)
    nu = K - 1
    chi_ratio = 2.0 * math.exp(2 * (math.lgamma((nu + 1) / 2) - math.lgamma(nu / 2))) / nu
    assert phi_g == pytest.approx(2 / math.pi, abs=3e-3)
    assert phi_s == pytest.approx(chi_ratio, abs=3e-3)
    assert phi_s > phi_g            # noise denser than the gradient for this recipe
