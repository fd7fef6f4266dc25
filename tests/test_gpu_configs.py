"""GPU parity on the five benchmark workloads at their FULL sizes, in the launch
configuration bench.py times (fused ss_signum_vote_step).

Two kinds of check per step:
  * against the CPU oracle, bit for bit, on EVERY coordinate of all five
    workloads: voted bits, every worker's packed bits (on the steps that ask
    for them), every momentum buffer and x, after every step.  Coordinates do
    not interact, so the oracle follows the vector chunk by chunk; its state
    (all momentum buffers and x) lives in host memory, the chunks travel
    through pinned staging buffers.
  * again on every coordinate, properties that hold at any size, evaluated
    with plain torch operations on the device: each worker's bit is [m_w < 0],
    the voted bit is [2 * (number of "-" workers) > M], and x moved by exactly
    -delta or +delta according to its voted bit (rounded once); padding bits
    are zero.
"""
import numpy as np
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"
SLAB = 8     # chunks checked together on the device


@pytest.fixture(scope="module")
def ss():
    import paper_1802_04434_amd as lib
    lib.load_library()
    return lib


def unpack_device(bits_i32, n):
    """first n bits of a device int32 word tensor as a bool tensor"""
    shifts = torch.arange(32, device=bits_i32.device, dtype=torch.int32)
    return ((bits_i32.unsqueeze(1) >> shifts) & 1).bool().reshape(-1)[:n]


def fill_gradients(cfg, step, g, mus, ties):
    for c in range(cfg.n_chunks):
        lo, hi = cfg.chunk_range(c)
        mu = mus[c] if mus is not None else synth.mu_chunk(cfg, c, DEV)
        tie = ties[c] if ties is not None else None
        for w in range(cfg.M):
            g[w][lo:hi] = synth.grad_chunk(cfg, step, w, c, DEV, mu=mu, tie=tie)


class Staging:
    """pinned host buffers one chunk long, reused for every device -> host copy"""

    def __init__(self, M, gdtype, has_m):
        n, nw = synth.CHUNK, synth.CHUNK // 32 + 4
        pin = lambda *shape, dtype: torch.empty(*shape, dtype=dtype, pin_memory=True)
        self.g = [pin(n, dtype=gdtype) for _ in range(M)]
        self.m = [pin(n, dtype=torch.float32) for _ in range(M)] if has_m else None
        self.x = pin(n, dtype=torch.float32)
        self.voted = pin(nw, dtype=torch.int32)
        self.packed = [pin(nw, dtype=torch.int32) for _ in range(M)]

    @staticmethod
    def fetch(stage, dev):
        out = stage[:dev.numel()]
        out.copy_(dev, non_blocking=True)
        return out


def host_view(t):
    """numpy view of a (pinned) host tensor in the oracle's conventions"""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.int32:
        return t.numpy().view(np.uint32)
    return t.numpy()


def run_config(ss, oracle, cfg, oracle_chunks, threads=16, three_calls=False):
    d, M = cfg.d, cfg.M
    has_m = cfg.beta is not None
    beta = cfg.beta if has_m else 0.0
    gdtype = torch.float32 if cfg.grad_dtype == "f32" else torch.bfloat16
    n_words = ss.packed_bytes(d) // 4
    g = [torch.empty(d, device=DEV, dtype=gdtype) for _ in range(M)]
    m = [torch.zeros(d, device=DEV) for _ in range(M)] if has_m else None
    x = torch.empty(d, device=DEV)
    for c in range(cfg.n_chunks):
        lo, hi = cfg.chunk_range(c)
        x[lo:hi] = synth.x0_chunk(cfg, c, DEV)
    x_before = torch.empty_like(x)
    # mean gradients and tie sets are fixed over steps: keep them when they fit comfortably
    keep = d <= 200_000_000
    mus = [synth.mu_chunk(cfg, c, DEV) for c in range(cfg.n_chunks)] if keep else None
    ties = [synth.tie_chunk(cfg, c, DEV) for c in range(cfg.n_chunks)] if (keep and cfg.tie_frac > 0) else None
    voted = ss.new_bits(d, DEV)
    packed = [ss.new_bits(d, DEV) for _ in range(M)]

    # oracle state per followed chunk
    host = {}
    for c in oracle_chunks:
        lo, hi = cfg.chunk_range(c)
        host[c] = {"m": [np.zeros(hi - lo, np.float32) for _ in range(M)] if has_m else None,
                   "x": x[lo:hi].cpu().numpy().copy()}
    stage = Staging(M, gdtype, has_m)

    delta_t = torch.tensor(cfg.delta, dtype=torch.float32, device=DEV)
    forced_ties_seen = 0
    for k in range(cfg.steps):
        fill_gradients(cfg, k, g, mus, ties)
        x_before.copy_(x)
        voted.fill_(-1)
        with_packed = (k % 2 == 1) or k == 0
        if with_packed:
            for p in packed:
                p.fill_(-1)
        print("step", k, cfg.name, "packed_out" if with_packed else "voted only", flush=True)
        if three_calls:
            # the same step as M + 2 library calls: pack per worker, vote, apply
            with_packed = True
            for w in range(M):
                ss.signum_pack(g[w], m[w] if has_m else None, beta, packed[w])
            ss.majority_vote(packed, voted, d)
            ss.sign_apply(x, voted, cfg.delta)
        else:
            ss.signum_vote_step(g, m, beta, cfg.delta, x, voted, packed if with_packed else None)
        torch.cuda.synchronize()

        # ---- every coordinate: internal consistency on the device
        for c0 in range(0, cfg.n_chunks, SLAB):
            lo = c0 * synth.CHUNK
            hi = min(d, (c0 + SLAB) * synth.CHUNK)
            n = hi - lo
            wlo, whi = lo // 32, (hi + 31) // 32
            count = torch.zeros(n, dtype=torch.int32, device=DEV)
            for w in range(M):
                neg = (m[w][lo:hi] if has_m else g[w][lo:hi].float()) < 0
                count += neg
                if with_packed:
                    assert torch.equal(unpack_device(packed[w][wlo:whi], n), neg), ("packed", k, w, c0)
            vbits = unpack_device(voted[wlo:whi], n)
            assert torch.equal(vbits, 2 * count > M), ("vote", k, c0)
            want_x = torch.where(vbits, x_before[lo:hi] + delta_t, x_before[lo:hi] - delta_t)
            assert torch.equal(x[lo:hi].view(torch.int32), want_x.view(torch.int32)), ("x", k, c0)
            if ties is not None:
                for c in range(c0, min(c0 + SLAB, cfg.n_chunks)):
                    clo, chi = cfg.chunk_range(c)
                    is_tie = ties[c][0]
                    assert torch.all(count[clo - lo:chi - lo][is_tie] * 2 == M), ("forced tie split", k, c)
                    assert not torch.any(vbits[clo - lo:chi - lo][is_tie]), ("tie votes +", k, c)
                    forced_ties_seen += int(is_tie.sum())
        # padding: bits at and beyond d, and pad words, are zero
        last = voted[d // 32:].cpu().numpy().view(np.uint32)
        big = sum(int(v) << (32 * i) for i, v in enumerate(last))
        assert big >> (d % 32) == 0
        assert n_words * 4 == ss.packed_bytes(d)

        # ---- followed chunks: bit-exact against the oracle
        for c in oracle_chunks:
            lo, hi = cfg.chunk_range(c)
            st = host[c]
            gh = [host_view(stage.fetch(stage.g[w], g[w][lo:hi])) for w in range(M)]
            torch.cuda.synchronize()
            want_voted, want_packed = oracle.signum_vote_step(gh, st["m"], beta, cfg.delta, st["x"],
                                                              want_packed=True, threads=threads)
            nw = len(want_voted)
            wlo = lo // 32
            got_voted = host_view(stage.fetch(stage.voted, voted[wlo: wlo + nw]))
            got_x = host_view(stage.fetch(stage.x, x[lo:hi]))
            got_m = [host_view(stage.fetch(stage.m[w], m[w][lo:hi])) for w in range(M)] if has_m else None
            got_packed = [host_view(stage.fetch(stage.packed[w], packed[w][wlo: wlo + nw])) for w in range(M)] \
                if with_packed else None
            torch.cuda.synchronize()
            assert np.array_equal(got_voted, want_voted), ("oracle voted", k, c)
            if with_packed:
                for w in range(M):
                    assert np.array_equal(got_packed[w], want_packed[w]), ("oracle packed", k, c, w)
            if has_m:
                for w in range(M):
                    assert np.array_equal(got_m[w].view(np.uint32), st["m"][w].view(np.uint32)), ("oracle m", k, c, w)
            assert np.array_equal(got_x.view(np.uint32), st["x"].view(np.uint32)), ("oracle x", k, c)
    if ties is not None:
        assert forced_ties_seen > 0.08 * d * cfg.steps
    del g, m, x, x_before, packed, voted
    torch.cuda.empty_cache()


def sampled_chunks(cfg, extra=3):
    rng = np.random.default_rng(cfg.config_id)
    n = cfg.n_chunks
    picks = {0, n - 1} | {int(v) for v in rng.integers(1, max(2, n - 1), extra)}
    return sorted(c for c in picks if c < n)


def test_c1_tiny_signum_vote_every_coordinate(ss, oracle):
    run_config(ss, oracle, synth.C1, list(range(synth.C1.n_chunks)))


def test_c2_signsgd_single_worker_every_coordinate(ss, oracle):
    # Algorithm 1: no momentum buffer, 5 % exact zeros plus planted -0.0 / subnormals
    run_config(ss, oracle, synth.C2, list(range(synth.C2.n_chunks)))


def test_c3_signum_vote_headline_every_coordinate(ss, oracle):
    run_config(ss, oracle, synth.C3, list(range(synth.C3.n_chunks)))


def test_c3_three_call_path_every_coordinate(ss, oracle):
    # the benchmark's "3-kernel path" at the headline size: M x ss_signum_pack,
    # ss_majority_vote, ss_sign_apply, every output of every call against the oracle
    run_config(ss, oracle, synth.C3.scaled(d=synth.C3.d, steps=6), list(range(synth.C3.n_chunks)), three_calls=True)


def test_c4_even_m_ties_every_coordinate(ss, oracle):
    run_config(ss, oracle, synth.C4, list(range(synth.C4.n_chunks)))


def test_c5_bf16_large_every_coordinate(ss, oracle):
    assert synth.C5.d % 32 == 17 and synth.C5.d % 4 == 1
    run_config(ss, oracle, synth.C5, list(range(synth.C5.n_chunks)))


def test_c3_variants_full_size(ss, oracle):
    """The variants of the step at the headline size: warm-up + "(good)" update with
    the int8 sums, vote with abstention, and Welford + density; sampled chunks
    against the oracle, every coordinate against properties evaluated with torch."""
    cfg = synth.C3.scaled(d=synth.C3.d, steps=3)
    d, M = cfg.d, cfg.M
    chunks = sampled_chunks(cfg, extra=1)
    g = [torch.empty(d, device=DEV) for _ in range(M)]
    mus = [synth.mu_chunk(cfg, c, DEV) for c in range(cfg.n_chunks)]
    x0 = torch.cat([synth.x0_chunk(cfg, c, DEV) for c in range(cfg.n_chunks)])
    delta_t = torch.tensor(cfg.delta, dtype=torch.float32, device=DEV)

    # ---- warm-up + sum update
    m = [torch.zeros(d, device=DEV) for _ in range(M)]
    x = x0.clone()
    voted = ss.new_bits(d, DEV)
    sums = torch.empty(d, dtype=torch.int8, device=DEV)
    host = {c: {"m": [np.zeros(cfg.chunk_range(c)[1] - cfg.chunk_range(c)[0], np.float32) for _ in range(M)],
                "x": x[cfg.chunk_range(c)[0]:cfg.chunk_range(c)[1]].cpu().numpy().copy()} for c in chunks}
    flags = ss.STEP_WARMUP | ss.STEP_SUM_UPDATE
    for k in range(cfg.steps):
        fill_gradients(cfg, k, g, mus, None)
        x_before = x.clone()
        voted.fill_(-1)
        sums.fill_(99)
        ss.signum_vote_step_ex(g, m, cfg.beta, cfg.delta, x, voted, None, sums, flags)
        torch.cuda.synchronize()
        count = torch.zeros(d, dtype=torch.int32, device=DEV)
        for w in range(M):
            count += g[w] < 0                                  # warm-up: the vote is on sign(g)
        assert torch.equal(sums.to(torch.int32), M - 2 * count)
        assert torch.equal(unpack_device(voted[: (d + 31) // 32], d), 2 * count > M)
        want_x = x_before - delta_t * sums.float()
        assert torch.equal(x.view(torch.int32), want_x.view(torch.int32))
        for c in chunks:
            lo, hi = cfg.chunk_range(c)
            st = host[c]
            wv, _, ws = oracle.signum_vote_step_ex([synth.as_numpy(g[w][lo:hi]) for w in range(M)], st["m"],
                                                   cfg.beta, cfg.delta, st["x"], flags)
            assert np.array_equal(voted[lo // 32: lo // 32 + len(wv)].cpu().numpy().view(np.uint32), wv)
            assert np.array_equal(sums[lo:hi].cpu().numpy(), ws)
            assert np.array_equal(x[lo:hi].cpu().numpy().view(np.uint32), st["x"].view(np.uint32))
            for w in range(M):
                assert np.array_equal(m[w][lo:hi].cpu().numpy().view(np.uint32), st["m"][w].view(np.uint32))

    # ---- vote with abstention (tau = 0.05, quorum 3), continuing from that state
    tau, Q = 0.05, 3
    vneg, vzero = ss.new_bits(d, DEV), ss.new_bits(d, DEV)
    for k in range(2):
        fill_gradients(cfg, 10 + k, g, mus, None)
        x_before = x.clone()
        ss.signum_vote_step_ternary(g, m, cfg.beta, tau, Q, cfg.delta, x, vneg, vzero)
        torch.cuda.synchronize()
        S = torch.zeros(d, dtype=torch.int32, device=DEV)
        tau_t = torch.tensor(tau, dtype=torch.float32, device=DEV)
        for w in range(M):
            votes = torch.where(m[w].abs() < tau_t, 0, torch.where(m[w] < 0, -1, 1))
            S += votes.to(torch.int32)
        neg_bits = unpack_device(vneg[: (d + 31) // 32], d)
        zero_bits = unpack_device(vzero[: (d + 31) // 32], d)
        assert torch.equal(neg_bits, S <= -Q) and torch.equal(zero_bits, S.abs() < Q)
        want_x = torch.where(zero_bits, x_before, torch.where(neg_bits, x_before + delta_t, x_before - delta_t))
        assert torch.equal(x.view(torch.int32), want_x.view(torch.int32))
        for c in chunks:
            lo, hi = cfg.chunk_range(c)
            st = host[c]
            wn, wz = oracle.signum_vote_step_ternary([synth.as_numpy(g[w][lo:hi]) for w in range(M)], st["m"],
                                                     cfg.beta, tau, Q, cfg.delta, st["x"])
            assert np.array_equal(vneg[lo // 32: lo // 32 + len(wn)].cpu().numpy().view(np.uint32), wn)
            assert np.array_equal(vzero[lo // 32: lo // 32 + len(wz)].cpu().numpy().view(np.uint32), wz)
            assert np.array_equal(x[lo:hi].cpu().numpy().view(np.uint32), st["x"].view(np.uint32))

    # ---- Welford over the workers' gradients of one step, then the two densities
    mean, m2 = torch.zeros(d, device=DEV), torch.zeros(d, device=DEV)
    hw = {c: (np.zeros(cfg.chunk_range(c)[1] - cfg.chunk_range(c)[0], np.float32),
              np.zeros(cfg.chunk_range(c)[1] - cfg.chunk_range(c)[0], np.float32)) for c in chunks}
    for w in range(M):
        ss.welford_update(g[w], mean, m2, w + 1)
        for c in chunks:
            lo, hi = cfg.chunk_range(c)
            oracle.welford_update(synth.as_numpy(g[w][lo:hi]), hw[c][0], hw[c][1], w + 1)
    sigma = torch.empty(d, device=DEV)
    ss.welford_sigma(m2, M, sigma)
    for c in chunks:
        lo, hi = cfg.chunk_range(c)
        assert np.array_equal(mean[lo:hi].cpu().numpy().view(np.uint32), hw[c][0].view(np.uint32))
        assert np.array_equal(m2[lo:hi].cpu().numpy().view(np.uint32), hw[c][1].view(np.uint32))
        assert np.array_equal(sigma[lo:hi].cpu().numpy().view(np.uint32),
                              oracle.welford_sigma(hw[c][1], M).view(np.uint32))
    out = torch.empty(3, dtype=torch.float64, device=DEV)
    ws = ss.new_density_workspace(DEV)
    for vec in (mean, sigma):
        ss.density(vec, out, ws)
        want = oracle.density(vec.cpu().numpy())
        got = out.cpu().numpy()
        assert got[0] == pytest.approx(want[0], rel=1e-12) and got[1] == pytest.approx(want[1], rel=1e-12)
        assert got[2] == pytest.approx(want[2], rel=3e-12)


def test_more_than_2_to_32_coordinates(ss, oracle):
    """Maximum-size case: d just above 2^32, so that any 32-bit index in a kernel
    or in the launch arithmetic would wrap.  One worker, bf16 gradient, no
    momentum (26 GB of state).  Every coordinate is checked with torch, the
    first and last stretches against the oracle."""
    d = (1 << 32) + 4096 + 5
    n = 1 << 20                                    # stretch compared with the oracle at both ends
    gen = torch.Generator(device=DEV)
    gen.manual_seed(42)
    g = torch.empty(d, device=DEV, dtype=torch.bfloat16)
    x = torch.empty(d, device=DEV)
    step = 1 << 28
    for lo in range(0, d, step):
        hi = min(d, lo + step)
        g[lo:hi] = torch.randn(hi - lo, device=DEV, generator=gen).to(torch.bfloat16)
        x[lo:hi] = torch.randn(hi - lo, device=DEV, generator=gen) * 0.05
    ends = [(0, n), (d - n - 5, d)]                 # the second one starts on a word boundary
    assert all(lo % 32 == 0 for lo, _ in ends)
    host_x = [x[lo:hi].cpu().numpy().copy() for lo, hi in ends]
    voted = ss.new_bits(d, DEV)
    voted.fill_(-1)
    delta = 1e-3
    delta_t = torch.tensor(delta, dtype=torch.float32, device=DEV)
    x_before = x.clone()
    ss.signum_vote_step([g], None, 0.0, delta, x, voted)
    torch.cuda.synchronize()
    for lo in range(0, d, step):
        hi = min(d, lo + step)
        bits = unpack_device(voted[lo // 32:(hi + 31) // 32], hi - lo)
        assert torch.equal(bits, g[lo:hi].float() < 0), lo
        want = torch.where(bits, x_before[lo:hi] + delta_t, x_before[lo:hi] - delta_t)
        assert torch.equal(x[lo:hi].view(torch.int32), want.view(torch.int32)), lo
    tail_words = voted[d // 32:].cpu().numpy().view(np.uint32)
    assert sum(int(v) << (32 * i) for i, v in enumerate(tail_words)) >> (d % 32) == 0
    for (lo, hi), hx in zip(ends, host_x):
        want_voted = oracle.signum_vote_step([synth.as_numpy(g[lo:hi])], None, 0.0, delta, hx, threads=16)
        got = voted[lo // 32: lo // 32 + len(want_voted)].cpu().numpy().view(np.uint32)
        assert np.array_equal(got, want_voted)
        assert np.array_equal(x[lo:hi].cpu().numpy().view(np.uint32), hx.view(np.uint32))
    # the stand-alone kernels at the same size: pack, vote (one voter), apply
    packed = ss.new_bits(d, DEV)
    ss.signum_pack(g, None, 0.0, packed)
    assert torch.equal(packed, voted)
    voted2 = ss.new_bits(d, DEV)
    ss.majority_vote([packed], voted2, d)
    assert torch.equal(voted2, voted)
    ss.sign_apply(x_before, voted2, delta)
    assert torch.equal(x_before.view(torch.int32), x.view(torch.int32))
    del g, x, x_before, voted, voted2, packed
    torch.cuda.empty_cache()
