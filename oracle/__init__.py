"""ctypes binding to the CPU oracle (oracle/signsgd_oracle.c).

Test infrastructure only: tests, the smoke check and the benchmark's CPU
baseline may import this; the product package must not.  All arrays are
numpy, host memory.  Functions mutate m / x in place like the C routines and
return the packed / voted words.
"""
import ctypes
import os

import numpy as np

from . import build as _build

F32 = 0
BF16 = 1

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        vp, sz, i32, f32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_float
        L.sso_packed_words.restype = sz
        L.sso_packed_words.argtypes = [sz]
        L.sso_packed_bytes.restype = sz
        L.sso_packed_bytes.argtypes = [sz]
        L.sso_signum_pack.argtypes = [vp, i32, vp, f32, vp, sz]
        L.sso_unpack.argtypes = [vp, sz, vp]
        L.sso_vote_sum.argtypes = [vp, i32, sz, vp]
        L.sso_majority_vote.argtypes = [vp, i32, vp, sz]
        L.sso_sign_apply.argtypes = [vp, vp, f32, sz]
        L.sso_signum_vote_step.argtypes = [vp, i32, vp, i32, f32, f32, vp, vp, vp, sz]
        L.sso_signum_vote_step_mt.argtypes = [vp, i32, vp, i32, f32, f32, vp, vp, vp, sz, i32]
        L.sso_warmup_length.restype = ctypes.c_long
        L.sso_warmup_length.argtypes = [f32]
        L.sso_signum_pack_warmup.argtypes = [vp, i32, vp, f32, vp, sz]
        L.sso_sum_apply.argtypes = [vp, vp, f32, sz]
        L.sso_signum_vote_step_ex.argtypes = [vp, i32, vp, i32, f32, f32, vp, vp, vp, vp, sz, ctypes.c_uint]
        L.sso_density.argtypes = [vp, sz, vp]
        L.sso_welford_update.argtypes = [vp, i32, vp, vp, ctypes.c_uint64, sz]
        L.sso_welford_sigma.argtypes = [vp, ctypes.c_uint64, vp, sz]
        L.sso_signum_pack_ternary.argtypes = [vp, i32, vp, f32, f32, vp, vp, sz]
        L.sso_quorum_vote.argtypes = [vp, vp, i32, i32, vp, vp, sz]
        L.sso_ternary_apply.argtypes = [vp, vp, vp, f32, sz]
        L.sso_signum_vote_step_ternary.argtypes = [vp, i32, vp, i32, f32, f32, i32, f32, vp, vp, vp, sz]
        _lib = L
    return _lib


def packed_words(d):
    return lib().sso_packed_words(d)


def packed_bytes(d):
    return lib().sso_packed_bytes(d)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError("%s failed with status %d" % (what, rc))


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def _ptr_array(arrs):
    return (ctypes.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])


def _grad_dtype(g):
    if g.dtype == np.float32:
        return F32
    if g.dtype == np.uint16:          # bf16 bit patterns
        return BF16
    raise TypeError("gradient must be float32 or uint16 (bf16 bits), got %s" % g.dtype)


def _need(a, dtype, n, name):
    if a.dtype != dtype or not a.flags.c_contiguous or a.ndim != 1 or a.shape[0] < n:
        raise TypeError("%s must be a contiguous 1-d %s array with >= %d elements" % (name, dtype, n))


def new_bits(d):
    return np.empty(packed_bytes(d) // 4, dtype=np.uint32)


def signum_pack(g, m, beta, d=None):
    d = len(g) if d is None else d
    gdt = _grad_dtype(g)
    _need(g, g.dtype, d, "g")
    if m is not None:
        _need(m, np.float32, d, "m")
    packed = new_bits(d)
    _check(lib().sso_signum_pack(_ptr(g), gdt, _ptr(m) if m is not None else None,
                                 float(np.float32(beta)), _ptr(packed), d), "sso_signum_pack")
    return packed


def unpack(bits, d):
    _need(bits, np.uint32, packed_words(d), "bits")
    out = np.empty(d, dtype=np.int8)
    _check(lib().sso_unpack(_ptr(bits), d, _ptr(out)), "sso_unpack")
    return out


def vote_sum(packed, d):
    for p in packed:
        _need(p, np.uint32, packed_words(d), "packed")
    out = np.empty(d, dtype=np.int32)
    _check(lib().sso_vote_sum(_ptr_array(packed), len(packed), d, _ptr(out)), "sso_vote_sum")
    return out


def majority_vote(packed, d):
    for p in packed:
        _need(p, np.uint32, packed_words(d), "packed")
    voted = new_bits(d)
    _check(lib().sso_majority_vote(_ptr_array(packed), len(packed), _ptr(voted), d),
           "sso_majority_vote")
    return voted


def sign_apply(x, bits, delta, d=None):
    d = len(x) if d is None else d
    _need(x, np.float32, d, "x")
    _need(bits, np.uint32, packed_words(d), "bits")
    _check(lib().sso_sign_apply(_ptr(x), _ptr(bits), float(np.float32(delta)), d), "sso_sign_apply")


def signum_vote_step(g, m, beta, delta, x, d=None, want_packed=False, threads=1):
    """g: list of M gradient arrays; m: list of M momentum arrays or None."""
    M = len(g)
    d = len(x) if d is None else d
    gdt = _grad_dtype(g[0])
    for a in g:
        _need(a, g[0].dtype, d, "g")
    if m is not None:
        for a in m:
            _need(a, np.float32, d, "m")
    _need(x, np.float32, d, "x")
    voted = new_bits(d)
    packed = [new_bits(d) for _ in range(M)] if want_packed else None
    args = [_ptr_array(g), gdt, _ptr_array(m) if m is not None else None, M,
            float(np.float32(beta)), float(np.float32(delta)), _ptr(x), _ptr(voted),
            _ptr_array(packed) if packed is not None else None, d]
    if threads == 1:
        _check(lib().sso_signum_vote_step(*args), "sso_signum_vote_step")
    else:
        _check(lib().sso_signum_vote_step_mt(*args, int(threads)), "sso_signum_vote_step_mt")
    return (voted, packed) if want_packed else voted


STEP_WARMUP = 1
STEP_SUM_UPDATE = 2


def warmup_length(beta):
    """Theorem 3's C(beta); raises for beta outside (0, 1)"""
    c = lib().sso_warmup_length(float(np.float32(beta)))
    if c < 0:
        raise ValueError("beta must lie in (0, 1)")
    return c


def signum_pack_warmup(g, m, beta, d=None):
    d = len(g) if d is None else d
    gdt = _grad_dtype(g)
    _need(g, g.dtype, d, "g")
    if m is not None:
        _need(m, np.float32, d, "m")
    packed = new_bits(d)
    _check(lib().sso_signum_pack_warmup(_ptr(g), gdt, _ptr(m) if m is not None else None,
                                        float(np.float32(beta)), _ptr(packed), d), "sso_signum_pack_warmup")
    return packed


def sum_apply(x, sums, delta, d=None):
    d = len(x) if d is None else d
    _need(x, np.float32, d, "x")
    _need(sums, np.int8, d, "sums")
    _check(lib().sso_sum_apply(_ptr(x), _ptr(sums), float(np.float32(delta)), d), "sso_sum_apply")


def signum_vote_step_ex(g, m, beta, delta, x, flags, d=None):
    """returns (voted, packed list, sums int8)"""
    M = len(g)
    d = len(x) if d is None else d
    gdt = _grad_dtype(g[0])
    for a in g:
        _need(a, g[0].dtype, d, "g")
    if m is not None:
        for a in m:
            _need(a, np.float32, d, "m")
    _need(x, np.float32, d, "x")
    voted = new_bits(d)
    packed = [new_bits(d) for _ in range(M)]
    sums = np.empty(d, dtype=np.int8)
    _check(lib().sso_signum_vote_step_ex(_ptr_array(g), gdt, _ptr_array(m) if m is not None else None, M,
                                         float(np.float32(beta)), float(np.float32(delta)), _ptr(x), _ptr(voted),
                                         _ptr_array(packed), _ptr(sums), d, int(flags)),
           "sso_signum_vote_step_ex")
    return voted, packed, sums


def density(v):
    """(|v|_1, |v|_2^2, phi(v)) of equation (1)"""
    _need(v, np.float32, len(v), "v")
    out = np.zeros(3, dtype=np.float64)
    _check(lib().sso_density(_ptr(v) if len(v) else None, len(v), _ptr(out)), "sso_density")
    return tuple(float(t) for t in out)


def welford_update(g, mean, m2, n):
    d = len(mean)
    gdt = _grad_dtype(g)
    _need(g, g.dtype, d, "g")
    _need(mean, np.float32, d, "mean")
    _need(m2, np.float32, d, "m2")
    _check(lib().sso_welford_update(_ptr(g), gdt, _ptr(mean), _ptr(m2), int(n), d), "sso_welford_update")


def welford_sigma(m2, n):
    sigma = np.empty_like(m2)
    _check(lib().sso_welford_sigma(_ptr(m2), int(n), _ptr(sigma), len(m2)), "sso_welford_sigma")
    return sigma


def signum_pack_ternary(g, m, beta, tau, d=None):
    """returns (neg bits, zero bits)"""
    d = len(g) if d is None else d
    gdt = _grad_dtype(g)
    _need(g, g.dtype, d, "g")
    if m is not None:
        _need(m, np.float32, d, "m")
    neg, zero = new_bits(d), new_bits(d)
    _check(lib().sso_signum_pack_ternary(_ptr(g), gdt, _ptr(m) if m is not None else None,
                                         float(np.float32(beta)), float(np.float32(tau)), _ptr(neg), _ptr(zero), d),
           "sso_signum_pack_ternary")
    return neg, zero


def quorum_vote(neg, zero, quorum, d):
    vneg, vzero = new_bits(d), new_bits(d)
    _check(lib().sso_quorum_vote(_ptr_array(neg), _ptr_array(zero), len(neg), int(quorum), _ptr(vneg), _ptr(vzero), d),
           "sso_quorum_vote")
    return vneg, vzero


def ternary_apply(x, neg, zero, delta, d=None):
    d = len(x) if d is None else d
    _check(lib().sso_ternary_apply(_ptr(x), _ptr(neg), _ptr(zero), float(np.float32(delta)), d), "sso_ternary_apply")


def signum_vote_step_ternary(g, m, beta, tau, quorum, delta, x, d=None):
    M = len(g)
    d = len(x) if d is None else d
    gdt = _grad_dtype(g[0])
    vneg, vzero = new_bits(d), new_bits(d)
    _check(lib().sso_signum_vote_step_ternary(_ptr_array(g), gdt, _ptr_array(m) if m is not None else None, M,
                                              float(np.float32(beta)), float(np.float32(tau)), int(quorum),
                                              float(np.float32(delta)), _ptr(x), _ptr(vneg), _ptr(vzero), d),
           "sso_signum_vote_step_ternary")
    return vneg, vzero
