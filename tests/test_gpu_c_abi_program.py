"""The boundary on its own: a plain C++ host program (csrc/abi_check.cpp, built
next to the library) calls ss_signum_vote_step with hipMalloc'd buffers - no
Python, no torch in that process - and its outputs must equal the CPU
oracle's, bit for bit."""
import os
import struct
import subprocess

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROGRAM = os.path.join(ROOT, "paper_1802_04434_amd", "abi_check")


@pytest.mark.parametrize("M,d,bf16", [(3, 70_001, False), (7, 1_300_021, False), (8, 250_007, True)])
def test_c_program_matches_the_oracle(oracle, tmp_path, M, d, bf16):
    if not os.path.exists(PROGRAM):
        # normally built beforehand with the library; a one-second host-only g++ build otherwise
        from paper_1802_04434_amd import build as lib_build
        lib_build.build_abi_check()
    rng = np.random.default_rng(M + d)
    if bf16:
        g = [(rng.standard_normal(d).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16) for _ in range(M)]
    else:
        g = [rng.standard_normal(d).astype(np.float32) for _ in range(M)]
    m = [(rng.standard_normal(d) * 0.3).astype(np.float32) for _ in range(M)]
    x = (rng.standard_normal(d) * 0.05).astype(np.float32)
    beta, delta = np.float32(0.9), np.float32(1e-3)
    inp, outp = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(inp, "wb") as f:
        f.write(struct.pack("<QiiFf".replace("F", "f"), d, M, int(bf16), float(beta), float(delta)))
        for a in g + m + [x]:
            f.write(a.tobytes())
    res = subprocess.run([PROGRAM, str(inp), str(outp)], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stderr
    want_voted, want_packed = oracle.signum_vote_step(g, m, float(beta), float(delta), x, want_packed=True)
    raw = np.fromfile(outp, dtype=np.uint8)
    pbytes = oracle.packed_bytes(d)
    pos = 0

    def take(n):
        nonlocal pos
        part = raw[pos:pos + n]
        pos += n
        return part

    assert np.array_equal(take(pbytes).view(np.uint32), want_voted)
    for w in range(M):
        assert np.array_equal(take(pbytes).view(np.uint32), want_packed[w]), w
    for w in range(M):
        assert np.array_equal(take(4 * d).view(np.uint32), m[w].view(np.uint32)), w
    assert np.array_equal(take(4 * d).view(np.uint32), x.view(np.uint32))
    assert pos == len(raw)
