"""GPU parity: the HIP library (through its C ABI) against the CPU oracle,
element by element, on the same seeded inputs.  Bit-exact on every output:
packed sign bits, voted bits, all M momentum buffers, parameters.

Sizes here are the ones the oracle finishes in seconds; they span several
1024-coordinate tiles plus a ragged tail.  Full-size configurations are in
test_gpu_configs.py.
"""
import numpy as np
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu

DEV = "cuda"
RAGGED = [1, 2, 31, 32, 33, 127, 128, 129, 255, 1000, 1023, 1024, 1025, 4096, 4099, 8192 + 31,
          70_001, 300_007]
SPECIAL_BITS = [0x00000000, 0x80000000, 0x00000001, 0x80000001, 0x007FFFFF, 0x807FFFFF, 0x00800000,
                0x80800000, 0x7F7FFFFF, 0xFF7FFFFF, 0x3F800000, 0xBF800000, 0x33800000, 0xB3800000]


@pytest.fixture(scope="module")
def ss():
    import paper_1802_04434_amd as lib
    lib.load_library()
    assert torch.cuda.is_available()
    return lib


def bits_np(t):
    return t.cpu().numpy().view(np.uint32)


def dirty_bits(ss, d):
    """output buffer pre-filled with ones, so that unwritten padding shows"""
    b = ss.new_bits(d, DEV)
    b.fill_(-1)
    return b


def make_grad(rng, d, dtype, scale=1.0):
    g = (rng.standard_normal(d) * scale).astype(np.float32)
    k = min(d, len(SPECIAL_BITS))
    idx = rng.permutation(d)[:k]
    special = np.array(SPECIAL_BITS[:k], dtype=np.uint32)
    if dtype == "bf16":
        special &= np.uint32(0xFFFF0000)     # keep them finite after rounding to bf16
    g.view(np.uint32)[idx] = special
    t = torch.from_numpy(g)
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t


def make_momentum(rng, d):
    m = (rng.standard_normal(d) * 0.3).astype(np.float32)
    k = min(d, len(SPECIAL_BITS))
    idx = rng.permutation(d)[:k]
    m.view(np.uint32)[idx] = np.array(SPECIAL_BITS[:k], dtype=np.uint32)
    # near-cancelling momentum on a stretch of coordinates: sign decided by rounding
    return m


def assert_same_floats(dev_t, host_a, what):
    # bit patterns, not values: also the sign of a zero must agree
    gb, hb = dev_t.cpu().numpy().view(np.uint32), host_a.view(np.uint32)
    same = gb == hb
    assert same.all(), "%s differs at %s" % (what, np.flatnonzero(~same)[:5])


# ------------------------------------------------------------ pack ------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("momentum", [False, True])
@pytest.mark.parametrize("d", RAGGED)
def test_signum_pack(ss, oracle, d, momentum, dtype):
    rng = np.random.default_rng(d * 4 + momentum * 2 + (dtype == "bf16"))
    g = make_grad(rng, d, dtype)
    m = make_momentum(rng, d) if momentum else None
    if momentum and d > 64:
        gf = g.float().numpy()
        m[32:64] = -(np.float32(1) - np.float32(0.9)) * gf[32:64] / np.float32(0.9)
    g_dev = g.to(DEV)
    m_dev = torch.from_numpy(m).to(DEV) if momentum else None
    packed = dirty_bits(ss, d)
    ss.signum_pack(g_dev, m_dev, 0.9, packed)
    want = oracle.signum_pack(synth.as_numpy(g), m, 0.9)
    assert np.array_equal(bits_np(packed), want)
    if momentum:
        assert_same_floats(m_dev, m, "m")


# ------------------------------------------------------------ vote ------

@pytest.mark.parametrize("M", list(range(1, 18)) + [31, 32, 33, 63, 64])
def test_majority_vote(ss, oracle, M):
    for d in (1, 97, 4099, 262_144 + 5):
        rng = np.random.default_rng(M * 7 + d)
        n = ss.packed_bytes(d) // 4
        # bias the words so that some coordinates sit right at the threshold
        words = [rng.integers(0, 1 << 32, n, dtype=np.uint64).astype(np.uint32) for _ in range(M)]
        dev = [torch.from_numpy(w.view(np.int32)).to(DEV) for w in words]   # padding bits are garbage on purpose
        voted = dirty_bits(ss, d)
        ss.majority_vote(dev, voted, d)
        want = oracle.majority_vote(words, d)
        assert np.array_equal(bits_np(voted), want), (M, d)


def test_majority_vote_exhaustive_patterns(ss, oracle):
    # coordinate i carries sign pattern i over the M workers: all 2^M cases
    for M in (1, 2, 3, 4, 5, 6, 7, 8, 9, 16):
        d = 1 << M
        i = np.arange(d, dtype=np.uint64)
        words = []
        for w in range(M):
            neg = ((i >> np.uint64(w)) & np.uint64(1)).astype(np.uint8)
            b = np.packbits(neg, bitorder="little")
            b = np.concatenate([b, np.zeros((-len(b)) % 16, np.uint8)])
            words.append(b.view(np.uint32).copy())
        dev = [torch.from_numpy(w.view(np.int32)).to(DEV) for w in words]
        voted = dirty_bits(ss, d)
        ss.majority_vote(dev, voted, d)
        assert np.array_equal(bits_np(voted), oracle.majority_vote(words, d)), M
        got = oracle.unpack(bits_np(voted), d)
        pop = np.array([bin(int(k)).count("1") for k in range(d)])
        assert np.array_equal(got == -1, 2 * pop > M)


def test_majority_vote_over_coordinate_shards(ss, oracle):
    # How the vote splits over several devices (Algorithm 3 with the server's work divided by
    # coordinate): shard j holds words [j W/M, (j+1) W/M) of all M workers' vectors and votes
    # on them alone.  The vote is pointwise, so the shards' results side by side are the vote
    # over the whole vector.  Shard boundaries are multiples of 128 coordinates (16 bytes).
    M, d = 8, 3_194_629            # one device's share of the headline workload with 8 workers, ragged end
    rng = np.random.default_rng(818)
    n = ss.packed_bytes(d) // 4
    words = [rng.integers(0, 1 << 32, n, dtype=np.uint64).astype(np.uint32) for _ in range(M)]
    dev = [torch.from_numpy(w.view(np.int32)).to(DEV) for w in words]
    whole = dirty_bits(ss, d)
    ss.majority_vote(dev, whole, d)
    want = oracle.majority_vote(words, d)
    assert np.array_equal(bits_np(whole), want)
    sharded = dirty_bits(ss, d)
    per = (d // M) // 128 * 128
    for j in range(M):
        lo = j * per
        dj = per if j < M - 1 else d - lo
        ss.majority_vote([t[lo // 32:] for t in dev], sharded[lo // 32:], dj)
    assert np.array_equal(bits_np(sharded), want)


# ----------------------------------------------------------- apply ------

@pytest.mark.parametrize("d", RAGGED)
def test_sign_apply(ss, oracle, d):
    rng = np.random.default_rng(d)
    x = (rng.standard_normal(d) * 0.05).astype(np.float32)
    x[: min(d, 3)] = np.array([0.0, 1e-4, -1e-4], dtype=np.float32)[: min(d, 3)]
    n = ss.packed_bytes(d) // 4
    bits = rng.integers(0, 1 << 32, n, dtype=np.uint64).astype(np.uint32)
    x_dev = torch.from_numpy(x).to(DEV)
    ss.sign_apply(x_dev, torch.from_numpy(bits.view(np.int32)).to(DEV), 1e-4)
    oracle.sign_apply(x, bits, 1e-4)
    assert_same_floats(x_dev, x, "x")


# ------------------------------------------------------ whole step ------

def run_both(ss, oracle, M, d, dtype, momentum, want_packed, seed, steps=2, beta=0.9, delta=1e-4):
    rng = np.random.default_rng(seed)
    m = [make_momentum(rng, d) for _ in range(M)] if momentum else None
    x = (rng.standard_normal(d) * 0.05).astype(np.float32)
    m_dev = [torch.from_numpy(a).to(DEV) for a in m] if momentum else None
    x_dev = torch.from_numpy(x).to(DEV)
    for k in range(steps):
        g = [make_grad(rng, d, dtype, scale=0.5) for _ in range(M)]
        g_dev = [t.to(DEV) for t in g]
        voted = dirty_bits(ss, d)
        packed = [dirty_bits(ss, d) for _ in range(M)] if want_packed else None
        ss.signum_vote_step(g_dev, m_dev, beta, delta, x_dev, voted, packed)
        out = oracle.signum_vote_step([synth.as_numpy(t) for t in g], m, beta, delta, x, want_packed=True)
        want_voted, want_bits = out
        assert np.array_equal(bits_np(voted), want_voted), ("voted", k)
        if want_packed:
            for w in range(M):
                assert np.array_equal(bits_np(packed[w]), want_bits[w]), ("packed", k, w)
        if momentum:
            for w in range(M):
                assert_same_floats(m_dev[w], m[w], "m[%d] step %d" % (w, k))
        assert_same_floats(x_dev, x, "x step %d" % k)


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 6, 7, 8, 9, 15, 16, 17, 33, 64])
@pytest.mark.parametrize("momentum", [False, True])
def test_fused_step_f32(ss, oracle, M, momentum):
    for d in (777, 20_000 + 13):
        run_both(ss, oracle, M, d, "f32", momentum, want_packed=True, seed=M * 31 + d)


@pytest.mark.parametrize("M", [1, 3, 8, 16, 20])
@pytest.mark.parametrize("momentum", [False, True])
def test_fused_step_bf16(ss, oracle, M, momentum):
    for d in (333, 12_289 + 17):
        run_both(ss, oracle, M, d, "bf16", momentum, want_packed=True, seed=M * 17 + d)


@pytest.mark.parametrize("d", RAGGED)
def test_fused_step_ragged_sizes(ss, oracle, d):
    run_both(ss, oracle, 7, d, "f32", True, want_packed=(d % 2 == 1), seed=d)
    run_both(ss, oracle, 8, d, "bf16", True, want_packed=(d % 2 == 0), seed=d + 1)


def test_fused_equals_three_call_path(ss):
    M, d = 7, 1_000_003
    gen = torch.Generator(device=DEV)
    gen.manual_seed(5)
    g = [torch.randn(d, device=DEV, generator=gen) for _ in range(M)]
    m0 = [torch.randn(d, device=DEV, generator=gen) * 0.2 for _ in range(M)]
    x0 = torch.randn(d, device=DEV, generator=gen) * 0.05
    # fused
    mf = [t.clone() for t in m0]
    xf = x0.clone()
    vf = dirty_bits(ss, d)
    pf = [dirty_bits(ss, d) for _ in range(M)]
    ss.signum_vote_step(g, mf, 0.9, 1e-4, xf, vf, pf)
    # three calls
    m3 = [t.clone() for t in m0]
    x3 = x0.clone()
    p3 = [dirty_bits(ss, d) for _ in range(M)]
    for w in range(M):
        ss.signum_pack(g[w], m3[w], 0.9, p3[w])
    v3 = dirty_bits(ss, d)
    ss.majority_vote(p3, v3, d)
    ss.sign_apply(x3, v3, 1e-4)
    torch.cuda.synchronize()
    assert torch.equal(vf, v3) and torch.equal(xf.view(torch.int32), x3.view(torch.int32))
    for w in range(M):
        assert torch.equal(pf[w], p3[w])
        assert torch.equal(mf[w].view(torch.int32), m3[w].view(torch.int32))
    # without per-worker bits the other outputs are the same
    mq = [t.clone() for t in m0]
    xq = x0.clone()
    vq = dirty_bits(ss, d)
    ss.signum_vote_step(g, mq, 0.9, 1e-4, xq, vq, None)
    assert torch.equal(vq, vf) and torch.equal(xq.view(torch.int32), xf.view(torch.int32))


@pytest.mark.parametrize("M,dtype", [(7, "f32"), (16, "f32"), (8, "bf16")])
def test_fused_equals_three_call_path_streaming_shape(ss, M, dtype):
    # d >= 2^20, M >= 2: the fused call takes the streaming launch shape that the
    # benchmark times; its outputs must be those of M packs + vote + apply, both with
    # and without per-worker bits (ragged d, so the scalar tail takes part)
    d = 3 * (1 << 20) + 2048 + 77
    gen = torch.Generator(device=DEV)
    gen.manual_seed(100 + M)
    gdt = torch.float32 if dtype == "f32" else torch.bfloat16
    g = [torch.randn(d, device=DEV, generator=gen).to(gdt) for _ in range(M)]
    m0 = [torch.randn(d, device=DEV, generator=gen) * 0.2 for _ in range(M)]
    x0 = torch.randn(d, device=DEV, generator=gen) * 0.05
    m3 = [t.clone() for t in m0]
    x3 = x0.clone()
    p3 = [dirty_bits(ss, d) for _ in range(M)]
    for w in range(M):
        ss.signum_pack(g[w], m3[w], 0.9, p3[w])
    v3 = dirty_bits(ss, d)
    ss.majority_vote(p3, v3, d)
    ss.sign_apply(x3, v3, 1e-4)
    for with_packed in (True, False):
        mf = [t.clone() for t in m0]
        xf = x0.clone()
        vf = dirty_bits(ss, d)
        pf = [dirty_bits(ss, d) for _ in range(M)] if with_packed else None
        ss.signum_vote_step(g, mf, 0.9, 1e-4, xf, vf, pf)
        torch.cuda.synchronize()
        assert torch.equal(vf, v3) and torch.equal(xf.view(torch.int32), x3.view(torch.int32))
        for w in range(M):
            assert torch.equal(mf[w].view(torch.int32), m3[w].view(torch.int32)), w
            if with_packed:
                assert torch.equal(pf[w], p3[w]), w


def test_nan_and_inf_follow_the_sign_rule(ss, oracle):
    # "bit = (v < 0)" applied literally: NaN is "+", -Inf is "-", +Inf is "+".  Packed and voted
    # bits and x are compared with the oracle exactly; momentum exactly wherever it is not a NaN
    # (a NaN's payload is not part of the contract), and NaN where the oracle's is NaN.
    M, d = 5, 8192 + 333
    rng = np.random.default_rng(77)
    nan, inf = np.float32("nan"), np.float32("inf")
    g = [(rng.standard_normal(d)).astype(np.float32) for _ in range(M)]
    m = [(rng.standard_normal(d) * 0.3).astype(np.float32) for _ in range(M)]
    x = (rng.standard_normal(d) * 0.05).astype(np.float32)
    for w in range(M):
        idx = rng.permutation(d)[:600]
        g[w][idx[:100]] = nan
        g[w][idx[100:200]] = inf
        g[w][idx[200:300]] = -inf
        m[w][idx[300:400]] = nan
        m[w][idx[400:500]] = inf
        m[w][idx[500:600]] = -inf
    m[0][:64] = inf
    g[0][:64] = -inf            # inf - inf = NaN inside the update
    for momentum in (True, False):
        g_dev = [torch.from_numpy(a).to(DEV) for a in g]
        m_dev = [torch.from_numpy(a.copy()).to(DEV) for a in m] if momentum else None
        m_host = [a.copy() for a in m] if momentum else None
        x_dev, x_host = torch.from_numpy(x.copy()).to(DEV), x.copy()
        voted = dirty_bits(ss, d)
        packed = [dirty_bits(ss, d) for _ in range(M)]
        ss.signum_vote_step(g_dev, m_dev, 0.9, 1e-3, x_dev, voted, packed)
        want_voted, want_packed = oracle.signum_vote_step(g, m_host, 0.9, 1e-3, x_host, want_packed=True)
        assert np.array_equal(bits_np(voted), want_voted)
        for w in range(M):
            assert np.array_equal(bits_np(packed[w]), want_packed[w]), w
        assert_same_floats(x_dev, x_host, "x")
        if momentum:
            for w in range(M):
                got = m_dev[w].cpu().numpy()
                isn = np.isnan(m_host[w])
                assert np.array_equal(np.isnan(got), isn), w
                assert isn.sum() >= 200
                assert np.array_equal(got.view(np.uint32)[~isn], m_host[w].view(np.uint32)[~isn]), w
        # the stand-alone pack on the same inputs
        for w in range(M):
            p = dirty_bits(ss, d)
            mm = torch.from_numpy(m[w].copy()).to(DEV) if momentum else None
            ss.signum_pack(g_dev[w], mm, 0.9, p)
            assert np.array_equal(bits_np(p), want_packed[w]), w


def test_inputs_that_are_only_read_may_coincide(ss, oracle):
    # one gradient handed in for several workers, one packed buffer handed in for several
    # voters: allowed (nothing is written there) and equal to separate copies
    d = 70_001
    gen = torch.Generator(device=DEV)
    gen.manual_seed(9)
    g = torch.randn(d, device=DEV, generator=gen)
    x0 = torch.randn(d, device=DEV, generator=gen) * 0.05
    xa, xb = x0.clone(), x0.clone()
    va, vb = dirty_bits(ss, d), dirty_bits(ss, d)
    ss.signum_vote_step([g, g, g], None, 0.0, 1e-3, xa, va)
    ss.signum_vote_step([g, g.clone(), g.clone()], None, 0.0, 1e-3, xb, vb)
    assert torch.equal(va, vb) and torch.equal(xa.view(torch.int32), xb.view(torch.int32))
    p = dirty_bits(ss, d)
    ss.signum_pack(g, None, 0.0, p)
    assert torch.equal(p, va)                       # three identical voters: the vote is their sign
    v2 = dirty_bits(ss, d)
    ss.majority_vote([p, p, p, p], v2, d)
    assert torch.equal(v2, p)
    # a bf16 gradient is half as long: a buffer that starts right behind it is clear of it
    gb = torch.randn(2 * d + 64, device=DEV, generator=gen).to(torch.bfloat16)
    packed = dirty_bits(ss, d)
    ss.signum_pack(gb, None, 0.0, packed, d=d)
    assert np.array_equal(bits_np(packed), oracle.signum_pack(synth.as_numpy(gb[:d]), None, 0.0))
    # ... and a written buffer that does touch an input is refused
    with pytest.raises(ss.SignSGDError):
        ss.signum_vote_step([g, g], [g, torch.zeros(d, device=DEV)], 0.9, 1e-3, xa, va)


def test_subnormals_are_not_flushed(ss, oracle):
    # products that underflow into the subnormal range, and subnormal inputs:
    # the device must keep them (a flush would turn "-" votes into "+")
    d = 2048 + 7
    rng = np.random.default_rng(1)
    g = (rng.standard_normal(d) * 1e-38).astype(np.float32)
    g[::3] = (rng.standard_normal(len(g[::3])) * 1e-44).astype(np.float32)
    m = (rng.standard_normal(d) * 1e-39).astype(np.float32)
    g_dev, m_dev = torch.from_numpy(g).to(DEV), torch.from_numpy(m).to(DEV)
    packed = dirty_bits(ss, d)
    ss.signum_pack(g_dev, m_dev, 0.9, packed)
    want = oracle.signum_pack(g, m, 0.9)
    assert np.array_equal(bits_np(packed), want)
    assert_same_floats(m_dev, m, "m")
    assert np.count_nonzero(m) > d // 2 and np.abs(m).max() < 1.2e-38


def test_beta_zero_equals_no_momentum(ss):
    d = 50_001
    gen = torch.Generator(device=DEV)
    gen.manual_seed(2)
    g = [torch.randn(d, device=DEV, generator=gen) for _ in range(3)]
    g[0][:100] = 0.0
    g[1][:50] = -0.0
    x0 = torch.randn(d, device=DEV, generator=gen)
    xa, xb = x0.clone(), x0.clone()
    va, vb = dirty_bits(ss, d), dirty_bits(ss, d)
    m = [torch.randn(d, device=DEV, generator=gen) for _ in range(3)]
    ss.signum_vote_step(g, m, 0.0, 1e-3, xa, va)
    ss.signum_vote_step(g, None, 0.77, 1e-3, xb, vb)
    assert torch.equal(va, vb) and torch.equal(xa, xb)
    for w in range(3):
        assert torch.equal(m[w], g[w])        # numerically: -0 == +0


def test_runs_on_the_callers_stream_and_checks_arguments(ss, oracle):
    d = 100_000
    s = torch.cuda.Stream()
    g = torch.randn(d, device=DEV)
    packed = dirty_bits(ss, d)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        ss.signum_pack(g, None, 0.0, packed)
    s.synchronize()
    assert np.array_equal(bits_np(packed), oracle.signum_pack(g.cpu().numpy(), None, 0.0))
    with pytest.raises(ss.SignSGDError) as e:
        ss.signum_pack(g[1:], None, 0.0, packed, d=d - 1)      # misaligned view
    assert e.value.status == -3
    with pytest.raises(TypeError):
        ss.signum_pack(g.cpu(), None, 0.0, packed)
    with pytest.raises(ss.SignSGDError) as e:
        ss.majority_vote([packed] * 65, packed, d)
    assert e.value.status == -2
    # d == 0 launches nothing
    ss.signum_vote_step([g], None, 0.0, 0.1, g, packed, d=0)


def test_checkpoint_resume_is_bit_identical(ss):
    # the library keeps no state: 4 steps == 2 steps, copy state out and back, 2 steps
    cfg = synth.C1.scaled(d=100_003, steps=4)
    def run(split):
        m = [torch.zeros(cfg.d, device=DEV) for _ in range(cfg.M)]
        x = synth.x0_chunk(cfg, 0, DEV)
        voted = dirty_bits(ss, cfg.d)
        for k in range(cfg.steps):
            if split and k == 2:
                saved = [t.cpu() for t in m], x.cpu()
                m = [t.to(DEV) for t in saved[0]]
                x = saved[1].to(DEV)
            g = [synth.grad_chunk(cfg, k, w, 0, DEV) for w in range(cfg.M)]
            ss.signum_vote_step(g, m, cfg.beta, cfg.delta, x, voted)
        return m, x, voted
    a, b = run(False), run(True)
    assert torch.equal(a[1], b[1]) and torch.equal(a[2], b[2])
    assert all(torch.equal(p, q) for p, q in zip(a[0], b[0]))


@pytest.mark.parametrize("M,dtype,momentum", [(2, "f32", True), (3, "bf16", True), (4, "f32", False),
                                              (9, "f32", True), (11, "bf16", False)])
def test_fused_step_large_d_streaming_shape(ss, oracle, M, dtype, momentum):
    # large enough for the one-worker-at-a-time launch shape with capped
    # occupancy; ragged so that the scalar tail runs as well
    d = 9_000_000 + 1234 + 19
    cfg = synth.Config("large", 40 + M, d, M, dtype, 0.9 if momentum else None, 1e-4, 2, "normal", 0.1, 0.5)
    m = [np.zeros(d, np.float32) for _ in range(M)] if momentum else None
    m_dev = [torch.zeros(d, device=DEV) for _ in range(M)] if momentum else None
    x_dev = torch.cat([synth.x0_chunk(cfg, c, DEV) for c in range(cfg.n_chunks)])
    x = x_dev.cpu().numpy().copy()
    for k in range(cfg.steps):
        g_dev = [torch.cat([synth.grad_chunk(cfg, k, w, c, DEV) for c in range(cfg.n_chunks)]) for w in range(M)]
        voted = dirty_bits(ss, d)
        packed = [dirty_bits(ss, d) for _ in range(M)] if k == 1 else None
        ss.signum_vote_step(g_dev, m_dev, 0.9, 1e-4, x_dev, voted, packed)
        want_voted, want_bits = oracle.signum_vote_step([synth.as_numpy(t) for t in g_dev], m, 0.9, 1e-4, x,
                                                        want_packed=True, threads=16)
        assert np.array_equal(bits_np(voted), want_voted), ("voted", k)
        if packed is not None:
            for w in range(M):
                assert np.array_equal(bits_np(packed[w]), want_bits[w]), ("packed", k, w)
        if momentum:
            for w in range(M):
                assert_same_floats(m_dev[w], m[w], "m[%d] step %d" % (w, k))
        assert_same_floats(x_dev, x, "x step %d" % k)


@pytest.mark.parametrize("M,dtype,momentum", [(13, "bf16", True), (6, "bf16", True), (33, "f32", True),
                                              (64, "f32", False), (17, "bf16", False)])
def test_fused_step_streaming_shape_any_worker_count(ss, oracle, M, dtype, momentum):
    # worker counts without a kernel of their own (the run-time-M kernel), in every streaming
    # shape: stages of two workers plus a remainder (bf16 + momentum, odd M), one worker per stage
    # (fp32 + momentum), several gradient loads per lane (no momentum); ragged d, two steps,
    # per-worker bits on the second
    d = (1 << 20) + 4096 + 333
    rng = np.random.default_rng(1000 + M)
    m = [make_momentum(rng, d) for _ in range(M)] if momentum else None
    x = (rng.standard_normal(d) * 0.05).astype(np.float32)
    m_dev = [torch.from_numpy(a).to(DEV) for a in m] if momentum else None
    x_dev = torch.from_numpy(x).to(DEV)
    for k in range(2):
        g = [make_grad(rng, d, dtype, scale=0.5) for _ in range(M)]
        g_dev = [t.to(DEV) for t in g]
        voted = dirty_bits(ss, d)
        packed = [dirty_bits(ss, d) for _ in range(M)] if k == 1 else None
        ss.signum_vote_step(g_dev, m_dev, 0.9, 1e-4, x_dev, voted, packed)
        want_voted, want_bits = oracle.signum_vote_step([synth.as_numpy(t) for t in g], m, 0.9, 1e-4, x,
                                                        want_packed=True, threads=16)
        assert np.array_equal(bits_np(voted), want_voted), ("voted", k)
        if packed is not None:
            for w in range(M):
                assert np.array_equal(bits_np(packed[w]), want_bits[w]), ("packed", k, w)
        if momentum:
            for w in range(M):
                assert_same_floats(m_dev[w], m[w], "m[%d] step %d" % (w, k))
        assert_same_floats(x_dev, x, "x step %d" % k)


@pytest.mark.parametrize("M,dtype,flags", [(10, "f32", 0), (12, "f32", 1), (4, "bf16", 0), (5, "bf16", 1)])
def test_fused_step_with_packed_out_at_many_workers(ss, oracle, M, dtype, flags):
    # d >= 2^24 with per-worker bits requested: the call may hand the signs
    # from launch to launch through packed_out; results must not change
    d = (1 << 24) + 1000 + 21
    rng = np.random.default_rng(M)
    g = [make_grad(rng, d, dtype, scale=0.5) for _ in range(M)]
    m = [make_momentum(rng, d) for _ in range(M)]
    x = (rng.standard_normal(d) * 0.05).astype(np.float32)
    g_dev = [t.to(DEV) for t in g]
    m_dev = [torch.from_numpy(a).to(DEV) for a in m]
    x_dev = torch.from_numpy(x).to(DEV)
    voted = dirty_bits(ss, d)
    packed = [dirty_bits(ss, d) for _ in range(M)]
    ss.signum_vote_step_ex(g_dev, m_dev, 0.9, 1e-4, x_dev, voted, packed, None, flags)
    # the same call without packed_out (always the one-pass kernel)
    m2 = [torch.from_numpy(a).to(DEV) for a in m]
    x2 = torch.from_numpy(x).to(DEV)
    voted2 = dirty_bits(ss, d)
    ss.signum_vote_step_ex(g_dev, m2, 0.9, 1e-4, x2, voted2, None, None, flags)
    assert torch.equal(voted, voted2) and torch.equal(x_dev.view(torch.int32), x2.view(torch.int32))
    assert all(torch.equal(a.view(torch.int32), b.view(torch.int32)) for a, b in zip(m_dev, m2))
    gh = [synth.as_numpy(t) for t in g]
    if flags == 0:
        want_voted, want_packed = oracle.signum_vote_step(gh, m, 0.9, 1e-4, x, want_packed=True, threads=16)
    else:       # warm-up, from its parts (the threaded oracle entry point has no flags)
        want_packed = [oracle.signum_pack_warmup(gh[w], m[w], 0.9) for w in range(M)]
        want_voted = oracle.majority_vote(want_packed, d)
        oracle.sign_apply(x, want_voted, 1e-4)
    assert np.array_equal(bits_np(voted), want_voted)
    for w in range(M):
        assert np.array_equal(bits_np(packed[w]), want_packed[w]), w
        assert_same_floats(m_dev[w], m[w], "m[%d]" % w)
    assert_same_floats(x_dev, x, "x")
