"""Host-only checks of the C-ABI HIP library: it loads, exports every symbol the
header declares, and rejects bad arguments before anything is launched.  No
kernel runs here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "signsgd.h")


@pytest.fixture(scope="module")
def lib():
    import paper_1802_04434_amd as ss
    return ss.load_library()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ss_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"ss_signum_pack", "ss_majority_vote", "ss_sign_apply", "ss_signum_vote_step",
            "ss_packed_words", "ss_packed_bytes", "ss_last_hip_error"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_packed_sizes(lib):
    for d, words, nbytes in ((0, 0, 0), (1, 1, 16), (32, 1, 16), (33, 2, 16), (128, 4, 16), (129, 5, 32),
                             (25_557_032, 798_658, 3_194_640), (1_500_000_017, 46_875_001, 187_500_016)):
        assert lib.ss_packed_words(d) == words
        assert lib.ss_packed_bytes(d) == nbytes


def test_argument_errors_come_back_as_status_codes(lib):
    OK, NULL, BAD_M, ALIGN, DTYPE = 0, -1, -2, -3, -4
    a = ctypes.c_void_p(0x1000)        # never dereferenced: validation fails first
    odd = ctypes.c_void_p(0x1004)
    one = (ctypes.c_void_p * 1)(0x1000)
    one_odd = (ctypes.c_void_p * 1)(0x1008)
    one_null = (ctypes.c_void_p * 1)(None)
    # d == 0: nothing to do, even with null pointers
    assert lib.ss_signum_pack(None, 0, None, 0.9, None, 0, None) == OK
    assert lib.ss_majority_vote(None, 1, None, 0, None) == OK
    assert lib.ss_sign_apply(None, None, 0.1, 0, None) == OK
    assert lib.ss_signum_vote_step(None, 0, None, 1, 0.9, 0.1, None, None, None, 0, None) == OK
    # dtype
    assert lib.ss_signum_pack(a, 2, None, 0.9, a, 8, None) == DTYPE
    assert lib.ss_signum_vote_step(one, -1, None, 1, 0.9, 0.1, a, a, None, 8, None) == DTYPE
    # worker count
    for M in (0, -3, 65):
        assert lib.ss_majority_vote(one, M, a, 8, None) == BAD_M
        assert lib.ss_signum_vote_step(one, 0, None, M, 0.9, 0.1, a, a, None, 8, None) == BAD_M
    # null pointers
    assert lib.ss_signum_pack(None, 0, None, 0.9, a, 8, None) == NULL
    assert lib.ss_signum_pack(a, 0, None, 0.9, None, 8, None) == NULL
    assert lib.ss_majority_vote(None, 1, a, 8, None) == NULL
    assert lib.ss_majority_vote(one_null, 1, a, 8, None) == NULL
    assert lib.ss_majority_vote(one, 1, None, 8, None) == NULL
    assert lib.ss_sign_apply(None, a, 0.1, 8, None) == NULL
    assert lib.ss_sign_apply(a, None, 0.1, 8, None) == NULL
    assert lib.ss_signum_vote_step(None, 0, None, 1, 0.9, 0.1, a, a, None, 8, None) == NULL
    assert lib.ss_signum_vote_step(one_null, 0, None, 1, 0.9, 0.1, a, a, None, 8, None) == NULL
    assert lib.ss_signum_vote_step(one, 0, one_null, 1, 0.9, 0.1, a, a, None, 8, None) == NULL
    assert lib.ss_signum_vote_step(one, 0, None, 1, 0.9, 0.1, None, a, None, 8, None) == NULL
    assert lib.ss_signum_vote_step(one, 0, None, 1, 0.9, 0.1, a, None, None, 8, None) == NULL
    assert lib.ss_signum_vote_step(one, 0, None, 1, 0.9, 0.1, a, a, one_null, 8, None) == NULL
    # alignment
    assert lib.ss_signum_pack(odd, 0, None, 0.9, a, 8, None) == ALIGN
    assert lib.ss_signum_pack(a, 0, odd, 0.9, a, 8, None) == ALIGN
    assert lib.ss_signum_pack(a, 0, None, 0.9, odd, 8, None) == ALIGN
    assert lib.ss_majority_vote(one_odd, 1, a, 8, None) == ALIGN
    assert lib.ss_majority_vote(one, 1, odd, 8, None) == ALIGN
    assert lib.ss_sign_apply(odd, a, 0.1, 8, None) == ALIGN
    assert lib.ss_sign_apply(a, odd, 0.1, 8, None) == ALIGN
    assert lib.ss_signum_vote_step(one_odd, 0, None, 1, 0.9, 0.1, a, a, None, 8, None) == ALIGN
    assert lib.ss_signum_vote_step(one, 0, one_odd, 1, 0.9, 0.1, a, a, None, 8, None) == ALIGN
    assert lib.ss_signum_vote_step(one, 0, None, 1, 0.9, 0.1, odd, a, None, 8, None) == ALIGN
    assert lib.ss_signum_vote_step(one, 0, None, 1, 0.9, 0.1, a, odd, None, 8, None) == ALIGN
    assert lib.ss_signum_vote_step(one, 0, None, 1, 0.9, 0.1, a, a, one_odd, 8, None) == ALIGN
    assert lib.ss_stream_copy(a, a, 24, None) == -5
    assert lib.ss_last_hip_error() == 0


def test_product_package_does_not_reach_the_oracle():
    pkg = os.path.join(ROOT, "paper_1802_04434_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower().replace("no fallback", ""), f
                assert "sso_" not in text, f


def test_warmup_length_matches_the_paper_and_the_oracle(lib, oracle):
    lib.ss_warmup_length.restype = ctypes.c_long
    lib.ss_warmup_length.argtypes = [ctypes.c_float]
    assert lib.ss_warmup_length(0.9) == 54                  # Theorem 3: "for beta = 0.9 we have C = 54"
    for beta in (0.1, 0.5, 0.75, 0.8, 0.9, 0.95, 0.99, 0.999):
        assert lib.ss_warmup_length(beta) == oracle.warmup_length(beta)
    for beta in (0.0, 1.0, -1.0, 2.0, float("nan")):
        assert lib.ss_warmup_length(beta) == -5
    # the search is bounded: a beta so close to 1 that C would exceed the documented
    # maximum comes back as SS_ERR_RANGE (distinct from an invalid beta) after a bounded time
    import time
    t0 = time.perf_counter()
    assert lib.ss_warmup_length(1.0 - 2.0 ** -24) == -7
    assert lib.ss_warmup_length(0.9999999) == -7
    assert time.perf_counter() - t0 < 2.0
    assert lib.ss_warmup_length(0.9999) == oracle.warmup_length(0.9999) > 100_000


def test_a_written_buffer_may_not_overlap_any_other(lib):
    """No kernel is launched: the overlap check comes after the NULL / alignment
    checks and before the launch, and the pointers here are not device memory."""
    ARG = -5
    vp = ctypes.c_void_p
    d = 1024                                   # 4096 bytes of fp32, 128 bytes of packed bits
    g, m, x, bits, out = 0x100000, 0x200000, 0x300000, 0x400000, 0x500000
    one = lambda p: (vp * 1)(p)
    two = lambda p, q: (vp * 2)(p, q)
    f = ctypes.c_float
    # ss_signum_pack: m inside g, packed inside m, exact alias, last byte only
    assert lib.ss_signum_pack(vp(g), 0, vp(g + 16), f(0.9), vp(bits), d, None) == ARG
    assert lib.ss_signum_pack(vp(g), 0, vp(m), f(0.9), vp(m + 4080), d, None) == ARG
    assert lib.ss_signum_pack(vp(g), 0, vp(g), f(0.9), vp(bits), d, None) == ARG
    assert lib.ss_signum_pack(vp(g), 0, None, f(0.9), vp(g + 4080), d, None) == ARG
    # bf16 gradients are half as long: the same offset is now clear of g ...
    # (validation passes, so do not run this one - it would launch; checked on the GPU instead)
    # ss_majority_vote: voted aliases an input; two inputs may coincide (read only) - that
    # case passes validation and would launch, so it is exercised in the GPU tests
    assert lib.ss_majority_vote(two(bits, bits + 0x1000), 2, vp(bits + 0x1000), d, None) == ARG
    assert lib.ss_majority_vote(two(bits, bits + 0x1000), 2, vp(bits + 112), d, None) == ARG
    # ss_sign_apply
    assert lib.ss_sign_apply(vp(x), vp(x + 2048), f(0.1), d, None) == ARG
    # the fused step: every written buffer against everything else
    step = lib.ss_signum_vote_step
    ok_g, ok_m = two(g, g + 0x10000), two(m, m + 0x10000)
    assert step(ok_g, 0, two(m, m + 2048), 2, f(0.9), f(0.1), vp(x), vp(bits), None, d, None) == ARG      # m0 / m1
    assert step(ok_g, 0, two(m, g + 0x10000), 2, f(0.9), f(0.1), vp(x), vp(bits), None, d, None) == ARG  # m1 == g1
    assert step(ok_g, 0, ok_m, 2, f(0.9), f(0.1), vp(m + 0x10000 + 4000), vp(bits), None, d, None) == ARG  # x / m1
    assert step(ok_g, 0, ok_m, 2, f(0.9), f(0.1), vp(x), vp(x + 4080), None, d, None) == ARG              # voted / x
    assert step(ok_g, 0, ok_m, 2, f(0.9), f(0.1), vp(x), vp(bits), two(out, bits), d, None) == ARG        # packed_out1 == voted
    assert step(ok_g, 0, None, 2, f(0.9), f(0.1), vp(g + 0x10000), vp(bits), None, d, None) == ARG        # x == g1
    ex = lib.ss_signum_vote_step_ex
    assert ex(ok_g, 0, ok_m, 2, f(0.9), f(0.1), vp(x), vp(bits), None, vp(x + 4000), d, 2, None) == ARG    # sums / x
    # the "(good)" pair, Welford, the ternary calls and the copy
    assert lib.ss_vote_sum(two(bits, bits + 0x1000), 2, vp(bits + 0x1000 + 64), d, None) == ARG
    assert lib.ss_sum_apply(vp(x), vp(x + 1024), f(0.1), d, None) == ARG
    u64 = ctypes.c_uint64
    assert lib.ss_welford_update(vp(g), 0, vp(m), vp(m + 16), u64(1), d, None) == ARG
    assert lib.ss_welford_update(vp(g), 0, vp(g), vp(m), u64(1), d, None) == ARG
    assert lib.ss_welford_sigma(vp(m), u64(2), vp(m), d, None) == ARG
    assert lib.ss_signum_pack_ternary(vp(g), 0, None, f(0.9), f(0.1), vp(bits), vp(bits + 64), d, None) == ARG
    assert lib.ss_quorum_vote(one(bits), one(bits + 0x1000), 1, 1, vp(out), vp(out + 16), d, None) == ARG
    assert lib.ss_quorum_vote(one(bits), one(bits + 0x1000), 1, 1, vp(out), vp(bits + 0x1000), d, None) == ARG
    assert lib.ss_ternary_apply(vp(x), vp(bits), vp(x + 4000), f(0.1), d, None) == ARG
    tstep = lib.ss_signum_vote_step_ternary
    assert tstep(ok_g, 0, ok_m, 2, f(0.9), f(0.1), 1, f(0.1), vp(x), vp(bits), vp(bits + 96), d, None) == ARG
    assert tstep(ok_g, 0, two(m, m), 2, f(0.9), f(0.1), 1, f(0.1), vp(x), vp(bits), vp(out), d, None) == ARG
    assert lib.ss_stream_copy(vp(x), vp(x + 1024), 4096, None) == ARG
    assert lib.ss_last_hip_error() == 0


def test_variant_entry_points_validate_arguments(lib):
    a = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    one = (ctypes.c_void_p * 1)(0x1000)
    step_ex = lib.ss_signum_vote_step_ex
    assert step_ex(one, 0, None, 1, 0.9, 0.1, a, a, None, None, 8, 4, None) == -5      # unknown flag
    assert step_ex(one, 0, None, 1, 0.9, 0.1, a, a, None, odd, 8, 2, None) == -3
    assert step_ex(one, 0, None, 0, 0.9, 0.1, a, a, None, None, 8, 0, None) == -2
    assert step_ex(None, 0, None, 1, 0.9, 0.1, a, a, None, None, 0, 3, None) == 0
    assert lib.ss_vote_sum(one, 1, None, 8, None) == -1
    assert lib.ss_vote_sum(one, 1, odd, 8, None) == -3
    assert lib.ss_vote_sum(one, 65, a, 8, None) == -2
    assert lib.ss_vote_sum(None, 1, None, 0, None) == 0
    assert lib.ss_sum_apply(None, a, 0.1, 8, None) == -1
    assert lib.ss_sum_apply(a, odd, 0.1, 8, None) == -3
    assert lib.ss_signum_pack_warmup(a, 5, None, 0.9, a, 8, None) == -4
    assert lib.ss_signum_pack_warmup(None, 0, None, 0.9, a, 8, None) == -1


def test_statistics_entry_points_validate_arguments(lib):
    a = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1008)
    u64 = ctypes.c_uint64
    assert lib.ss_welford_update(a, 0, a, a, u64(0), 8, None) == -5            # n counts from 1
    assert lib.ss_welford_update(a, 0, a, a, u64((1 << 24) + 1), 8, None) == -5  # n must be exact in fp32
    assert lib.ss_welford_update(a, 3, a, a, u64(1), 8, None) == -4
    assert lib.ss_welford_update(None, 0, a, a, u64(1), 8, None) == -1
    assert lib.ss_welford_update(a, 0, odd, a, u64(1), 8, None) == -3
    assert lib.ss_welford_update(None, 0, None, None, u64(1), 0, None) == 0
    assert lib.ss_welford_sigma(a, u64(0), a, 8, None) == -5
    assert lib.ss_welford_sigma(None, u64(2), a, 8, None) == -1
    assert lib.ss_welford_sigma(a, u64(2), odd, 8, None) == -3
    b, c = ctypes.c_void_p(0x2000), ctypes.c_void_p(0x9000)
    lib.ss_density_workspace_bytes.restype = ctypes.c_size_t
    wsb = lib.ss_density_workspace_bytes()
    assert wsb % 16 == 0 and 1024 <= wsb <= 16 * 1024
    assert lib.ss_density(a, 8, None, c, None) == -1
    assert lib.ss_density(None, 8, b, c, None) == -1
    assert lib.ss_density(a, 8, b, None, None) == -1
    assert lib.ss_density(a, 8, odd, c, None) == -3
    assert lib.ss_density(a, 8, b, odd, None) == -3
    assert lib.ss_density(a, 8, c, c, None) == -5                       # out inside the workspace


def test_abstention_entry_points_validate_arguments(lib):
    a = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1008)
    one = (ctypes.c_void_p * 1)(0x1000)
    f = ctypes.c_float
    assert lib.ss_signum_pack_ternary(a, 0, None, f(0.9), f(-0.1), a, a, 8, None) == -5      # tau < 0
    assert lib.ss_signum_pack_ternary(a, 0, None, f(0.9), f(float("nan")), a, a, 8, None) == -5
    assert lib.ss_signum_pack_ternary(a, 0, None, f(0.9), f(0.1), None, a, 8, None) == -1
    assert lib.ss_signum_pack_ternary(a, 0, None, f(0.9), f(0.1), a, odd, 8, None) == -3
    assert lib.ss_signum_pack_ternary(None, 0, None, f(0.9), f(0.1), None, None, 0, None) == 0
    assert lib.ss_quorum_vote(one, one, 1, 0, a, a, 8, None) == -5                           # quorum >= 1
    assert lib.ss_quorum_vote(one, one, 65, 1, a, a, 8, None) == -2
    assert lib.ss_quorum_vote(one, None, 1, 1, a, a, 8, None) == -1
    assert lib.ss_quorum_vote(one, one, 1, 1, a, odd, 8, None) == -3
    assert lib.ss_ternary_apply(a, None, a, f(0.1), 8, None) == -1
    assert lib.ss_ternary_apply(odd, a, a, f(0.1), 8, None) == -3
    step = lib.ss_signum_vote_step_ternary
    assert step(one, 0, None, 1, f(0.9), f(0.1), 0, f(0.1), a, a, a, 8, None) == -5
    assert step(one, 0, None, 0, f(0.9), f(0.1), 1, f(0.1), a, a, a, 8, None) == -2
    assert step(one, 0, None, 1, f(0.9), f(0.1), 1, f(0.1), a, None, a, 8, None) == -1
    assert step(one, 0, None, 1, f(0.9), f(0.1), 1, f(0.1), a, a, odd, 8, None) == -3
    assert step(one, 9, None, 1, f(0.9), f(0.1), 1, f(0.1), a, a, a, 8, None) == -4
