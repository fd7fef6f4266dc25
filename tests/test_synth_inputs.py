"""The seeded input recipes (host side, small sizes): determinism, chunk
addressing, and that each workload has the structure it is meant to exercise."""
import numpy as np
import torch

import synth


def test_blocks_are_deterministic_and_distinct():
    cfg = synth.C3.scaled(d=synth.CHUNK + 1000)
    a = synth.grad_chunk(cfg, 2, 3, 1)
    b = synth.grad_chunk(cfg, 2, 3, 1)
    assert torch.equal(a, b) and a.numel() == 1000
    for other in (synth.grad_chunk(cfg, 2, 4, 1), synth.grad_chunk(cfg, 3, 3, 1),
                  synth.grad_chunk(cfg, 2, 3, 0)[:1000]):
        assert not torch.equal(a, other)
    seeds = {synth.block_seed(c, r, s, w, k) for c in range(1, 6) for r in synth._ROLES
             for s in range(3) for w in range(3) for k in range(3)}
    assert len(seeds) == 5 * len(synth._ROLES) * 27


def test_config_table_matches_the_benchmark_definition():
    got = {k: (c.d, c.M, c.grad_dtype, c.beta, c.delta, c.steps) for k, c in synth.CONFIGS.items()}
    assert got == {
        "C1": (272_474, 7, "f32", 0.9, 1e-4, 10),
        "C2": (25_557_032, 1, "f32", None, 1e-4, 20),
        "C3": (25_557_032, 7, "f32", 0.9, 1e-4, 20),
        "C4": (138_357_544, 16, "f32", 0.9, 1e-4, 10),
        "C5": (1_500_000_017, 8, "bf16", 0.9, 1e-5, 5),
    }
    assert synth.C5.d % 32 == 17 and synth.C1.d % 4 == 2


def test_c2_zeros_and_planted_values():
    cfg = synth.C2.scaled(d=200_000)
    g = synth.grad_chunk(cfg, 0, 0, 0)
    frac = float((g == 0).float().mean())
    assert 0.04 < frac < 0.06
    bits = g.view(torch.int32).numpy().view(np.uint32)
    for idx, pat in synth.PLANTED_C2:
        assert bits[idx] == pat


def test_c4_forced_ties_split_the_workers_evenly(oracle):
    cfg = synth.C4.scaled(d=50_003, steps=4)
    is_tie, pattern = synth.tie_chunk(cfg, 0)
    assert 0.08 < float(is_tie.float().mean()) < 0.12
    pop = sum(((pattern >> w) & 1) for w in range(cfg.M))
    assert torch.all(pop == cfg.M // 2)
    tie = is_tie.numpy()
    m = [np.zeros(cfg.d, np.float32) for _ in range(cfg.M)]
    x = synth.as_numpy(synth.x0_chunk(cfg, 0))
    for k in range(cfg.steps):
        g = [synth.as_numpy(synth.grad_chunk(cfg, k, w, 0)) for w in range(cfg.M)]
        voted, packed = oracle.signum_vote_step(g, m, cfg.beta, cfg.delta, x, want_packed=True)
        s = oracle.vote_sum(packed, cfg.d)
        assert np.all(s[tie] == 0)                                  # exact 8 : 8 on the voted quantity
        assert np.all(oracle.unpack(voted, cfg.d)[tie] == 1)        # a tie votes "+"
        assert np.mean(s == 0) > 0.12                               # natural ties on top


def test_c5_is_bf16_with_laplace_mean():
    cfg = synth.C5.scaled(d=100_001)
    g = synth.grad_chunk(cfg, 0, 0, 0)
    assert g.dtype == torch.bfloat16
    assert synth.as_numpy(g).dtype == np.uint16
    mu = synth.mu_chunk(cfg, 0)
    # Laplace(0, b): mean |mu| = b
    assert abs(float(mu.abs().mean()) - 0.05) < 0.002
    assert torch.isfinite(mu).all()
