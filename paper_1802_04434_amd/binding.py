"""ctypes marshalling for libsignsgd.so.  Function names and argument order
follow include/signsgd.h (ss_ prefix dropped)."""
import ctypes
import os

import torch

F32 = 0
BF16 = 1
MAX_WORKERS = 64

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsignsgd.so")
_lib = None

_STATUS = {0: "SS_OK", -1: "SS_ERR_NULL", -2: "SS_ERR_BAD_M", -3: "SS_ERR_ALIGN",
           -4: "SS_ERR_DTYPE", -5: "SS_ERR_ARG", -6: "SS_ERR_HIP", -7: "SS_ERR_RANGE"}


class SignSGDError(RuntimeError):
    def __init__(self, call, status):
        self.status = status
        detail = ""
        if status == -6 and _lib is not None:
            detail = " (hipError_t %d)" % _lib.ss_last_hip_error()
        super().__init__("%s returned %s%s" % (call, _STATUS.get(status, status), detail))


def library_path():
    return _LIB_PATH


def load_library():
    """Load the built HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                "%s is missing: build it with `python -m paper_1802_04434_amd.build` "
                "(there is no fallback path)" % _LIB_PATH)
        L = ctypes.CDLL(_LIB_PATH)
        vp, sz, i32, f32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_float
        L.ss_packed_words.restype = sz
        L.ss_packed_words.argtypes = [sz]
        L.ss_packed_bytes.restype = sz
        L.ss_packed_bytes.argtypes = [sz]
        L.ss_last_hip_error.restype = i32
        L.ss_last_hip_error.argtypes = []
        L.ss_signum_pack.argtypes = [vp, i32, vp, f32, vp, sz, vp]
        L.ss_majority_vote.argtypes = [vp, i32, vp, sz, vp]
        L.ss_sign_apply.argtypes = [vp, vp, f32, sz, vp]
        L.ss_signum_vote_step.argtypes = [vp, i32, vp, i32, f32, f32, vp, vp, vp, sz, vp]
        L.ss_stream_copy.argtypes = [vp, vp, sz, vp]
        L.ss_warmup_length.restype = ctypes.c_long
        L.ss_warmup_length.argtypes = [f32]
        L.ss_signum_pack_warmup.argtypes = [vp, i32, vp, f32, vp, sz, vp]
        L.ss_vote_sum.argtypes = [vp, i32, vp, sz, vp]
        L.ss_sum_apply.argtypes = [vp, vp, f32, sz, vp]
        L.ss_signum_vote_step_ex.argtypes = [vp, i32, vp, i32, f32, f32, vp, vp, vp, vp, sz, ctypes.c_uint, vp]
        L.ss_welford_update.argtypes = [vp, i32, vp, vp, ctypes.c_uint64, sz, vp]
        L.ss_welford_sigma.argtypes = [vp, ctypes.c_uint64, vp, sz, vp]
        L.ss_density.argtypes = [vp, sz, vp, vp, vp]
        L.ss_density_workspace_bytes.restype = sz
        L.ss_density_workspace_bytes.argtypes = []
        L.ss_density_static.argtypes = [vp, sz, vp, vp]
        L.ss_density_static.restype = i32
        L.ss_signum_pack_ternary.argtypes = [vp, i32, vp, f32, f32, vp, vp, sz, vp]
        L.ss_quorum_vote.argtypes = [vp, vp, i32, i32, vp, vp, sz, vp]
        L.ss_ternary_apply.argtypes = [vp, vp, vp, f32, sz, vp]
        L.ss_signum_vote_step_ternary.argtypes = [vp, i32, vp, i32, f32, f32, i32, f32, vp, vp, vp, sz, vp]
        for name in ("ss_signum_pack_ternary", "ss_quorum_vote", "ss_ternary_apply",
                     "ss_signum_vote_step_ternary"):
            getattr(L, name).restype = i32
        for name in ("ss_welford_update", "ss_welford_sigma", "ss_density"):
            getattr(L, name).restype = i32
        for name in ("ss_signum_pack", "ss_majority_vote", "ss_sign_apply", "ss_signum_vote_step",
                     "ss_stream_copy", "ss_signum_pack_warmup", "ss_vote_sum", "ss_sum_apply",
                     "ss_signum_vote_step_ex"):
            getattr(L, name).restype = i32
        _lib = L
    return _lib


def packed_words(d):
    return load_library().ss_packed_words(d)


def packed_bytes(d):
    return load_library().ss_packed_bytes(d)


def last_hip_error():
    return load_library().ss_last_hip_error()


def new_bits(d, device="cuda"):
    """uninitialised packed / voted buffer for d coordinates (int32 storage)"""
    return torch.empty(packed_bytes(d) // 4, dtype=torch.int32, device=device)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev(t, dtype, n, name):
    if not t.is_cuda:
        raise TypeError("%s must live in device memory" % name)
    if t.dtype not in (dtype if isinstance(dtype, tuple) else (dtype,)):
        raise TypeError("%s has dtype %s" % (name, t.dtype))
    if not t.is_contiguous() or t.numel() < n:
        raise TypeError("%s must be contiguous with at least %d elements" % (name, n))
    return t.data_ptr()


def _grad_dtype(g):
    if g.dtype == torch.float32:
        return F32
    if g.dtype == torch.bfloat16:
        return BF16
    raise TypeError("gradient dtype must be float32 or bfloat16, got %s" % g.dtype)


def _ptr_array(ptrs):
    return (ctypes.c_void_p * len(ptrs))(*ptrs)


def _check(call, status):
    if status != 0:
        raise SignSGDError(call, status)


_BITS = (torch.int32, torch.uint32) if hasattr(torch, "uint32") else (torch.int32,)


def _signum_pack(name, g, m, beta, packed, d, stream):
    L = load_library()
    d = g.numel() if d is None else d
    gp = _dev(g, (torch.float32, torch.bfloat16), d, "g")
    mp = _dev(m, torch.float32, d, "m") if m is not None else None
    pp = _dev(packed, _BITS, L.ss_packed_bytes(d) // 4, "packed")
    _check(name, getattr(L, name)(gp, _grad_dtype(g), mp, beta, pp, d, _stream(stream)))
    return packed


def signum_pack(g, m, beta, packed, d=None, stream=None):
    """ss_signum_pack: m <- beta m + (1-beta) g; packed <- bits of sign(m)
    (m None: bits of sign(g))."""
    return _signum_pack("ss_signum_pack", g, m, beta, packed, d, stream)


def signum_pack_warmup(g, m, beta, packed, d=None, stream=None):
    """ss_signum_pack_warmup: m updated as above, packed <- bits of sign(g)"""
    return _signum_pack("ss_signum_pack_warmup", g, m, beta, packed, d, stream)


def warmup_length(beta):
    """ss_warmup_length: Theorem 3's C(beta)"""
    c = load_library().ss_warmup_length(beta)
    if c < 0:
        raise SignSGDError("ss_warmup_length", c)
    return c


def vote_sum(packed, sums, d, stream=None):
    """ss_vote_sum: sums <- per-coordinate sum of the workers' signs (int8)"""
    L = load_library()
    n = L.ss_packed_bytes(d) // 4
    ptrs = [_dev(p, _BITS, n, "packed[%d]" % i) for i, p in enumerate(packed)]
    sp = _dev(sums, torch.int8, d, "sums")
    _check("ss_vote_sum", L.ss_vote_sum(_ptr_array(ptrs), len(ptrs), sp, d, _stream(stream)))
    return sums


def sum_apply(x, sums, delta, d=None, stream=None):
    """ss_sum_apply: x <- x - delta * sums"""
    L = load_library()
    d = x.numel() if d is None else d
    xp = _dev(x, torch.float32, d, "x")
    sp = _dev(sums, torch.int8, d, "sums")
    _check("ss_sum_apply", L.ss_sum_apply(xp, sp, delta, d, _stream(stream)))
    return x


def majority_vote(packed, voted, d, stream=None):
    """ss_majority_vote: voted <- bits of sign(sum_w sign_w)"""
    L = load_library()
    n = L.ss_packed_bytes(d) // 4
    ptrs = [_dev(p, _BITS, n, "packed[%d]" % i) for i, p in enumerate(packed)]
    vp = _dev(voted, _BITS, n, "voted")
    _check("ss_majority_vote", L.ss_majority_vote(_ptr_array(ptrs), len(ptrs), vp, d, _stream(stream)))
    return voted


def sign_apply(x, bits, delta, d=None, stream=None):
    """ss_sign_apply: x <- x - delta * (+-1 from bits)"""
    L = load_library()
    d = x.numel() if d is None else d
    xp = _dev(x, torch.float32, d, "x")
    bp = _dev(bits, _BITS, L.ss_packed_words(d), "bits")
    _check("ss_sign_apply", L.ss_sign_apply(xp, bp, delta, d, _stream(stream)))
    return x


STEP_DEFAULT = 0
STEP_WARMUP = 1
STEP_SUM_UPDATE = 2


def signum_vote_step(g, m, beta, delta, x, voted, packed_out=None, d=None, stream=None):
    """ss_signum_vote_step: the whole step for M = len(g) workers in one pass.
    g: list of gradients; m: list of momentum buffers or None."""
    return signum_vote_step_ex(g, m, beta, delta, x, voted, packed_out, None, None, d, stream)


def signum_vote_step_ex(g, m, beta, delta, x, voted, packed_out=None, sums_out=None, flags=None, d=None,
                        stream=None):
    """ss_signum_vote_step_ex (flags None: the plain ss_signum_vote_step entry point)"""
    L = load_library()
    M = len(g)
    d = x.numel() if d is None else d
    n = L.ss_packed_bytes(d) // 4
    gdt = _grad_dtype(g[0])
    gp = [_dev(t, g[0].dtype, d, "g[%d]" % i) for i, t in enumerate(g)]
    mp = [_dev(t, torch.float32, d, "m[%d]" % i) for i, t in enumerate(m)] if m is not None else None
    pp = [_dev(t, _BITS, n, "packed_out[%d]" % i) for i, t in enumerate(packed_out)] \
        if packed_out is not None else None
    if (mp is not None and len(mp) != M) or (pp is not None and len(pp) != M):
        raise ValueError("g, m and packed_out must have one entry per worker")
    xp = _dev(x, torch.float32, d, "x")
    vp = _dev(voted, _BITS, n, "voted")
    g_arr = _ptr_array(gp)
    m_arr = _ptr_array(mp) if mp is not None else None
    p_arr = _ptr_array(pp) if pp is not None else None
    if flags is None and sums_out is None:
        _check("ss_signum_vote_step", L.ss_signum_vote_step(
            g_arr, gdt, m_arr, M, beta, delta, xp, vp, p_arr, d, _stream(stream)))
    else:
        sp = _dev(sums_out, torch.int8, d, "sums_out") if sums_out is not None else None
        _check("ss_signum_vote_step_ex", L.ss_signum_vote_step_ex(
            g_arr, gdt, m_arr, M, beta, delta, xp, vp, p_arr, sp, d, int(flags or 0), _stream(stream)))
    return voted


def stream_copy(dst, src, nbytes, stream=None):
    """ss_stream_copy: measurement aid, dst <- src"""
    L = load_library()
    _check("ss_stream_copy", L.ss_stream_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream(stream)))


def welford_update(g, mean, m2, n, d=None, stream=None):
    """ss_welford_update: fold the n-th gradient (n counts from 1) into mean / m2"""
    L = load_library()
    d = mean.numel() if d is None else d
    gp = _dev(g, (torch.float32, torch.bfloat16), d, "g")
    _check("ss_welford_update", L.ss_welford_update(gp, _grad_dtype(g), _dev(mean, torch.float32, d, "mean"),
                                                    _dev(m2, torch.float32, d, "m2"), n, d, _stream(stream)))


def welford_sigma(m2, n, sigma, d=None, stream=None):
    """ss_welford_sigma: sigma <- sqrt(m2 / n)"""
    L = load_library()
    d = m2.numel() if d is None else d
    _check("ss_welford_sigma", L.ss_welford_sigma(_dev(m2, torch.float32, d, "m2"), n,
                                                  _dev(sigma, torch.float32, d, "sigma"), d, _stream(stream)))
    return sigma


def new_density_workspace(device="cuda"):
    """zero-filled workspace for ss_density (ss_density_workspace_bytes() bytes)"""
    return torch.zeros(load_library().ss_density_workspace_bytes() // 8, dtype=torch.int64, device=device)


def density(v, out, workspace, d=None, stream=None):
    """ss_density: out (3 float64 on the device) <- |v|_1, |v|_2^2, phi(v)"""
    L = load_library()
    d = v.numel() if d is None else d
    vp = _dev(v, torch.float32, d, "v") if d else None
    wp = _dev(workspace, torch.int64, L.ss_density_workspace_bytes() // 8, "workspace")
    _check("ss_density", L.ss_density(vp, d, _dev(out, torch.float64, 3, "out"), wp, _stream(stream)))
    return out


def density_static(v, out, d=None, stream=None):
    """ss_density_static: ss_density on the library's own fixed scratch array (allocates nothing)"""
    L = load_library()
    d = v.numel() if d is None else d
    vp = _dev(v, torch.float32, d, "v") if d else None
    _check("ss_density_static", L.ss_density_static(vp, d, _dev(out, torch.float64, 3, "out"), _stream(stream)))
    return out


def signum_pack_ternary(g, m, beta, tau, neg, zero, d=None, stream=None):
    """ss_signum_pack_ternary: momentum update, then this worker's ternary vote"""
    L = load_library()
    d = g.numel() if d is None else d
    n = L.ss_packed_bytes(d) // 4
    _check("ss_signum_pack_ternary", L.ss_signum_pack_ternary(
        _dev(g, (torch.float32, torch.bfloat16), d, "g"), _grad_dtype(g),
        _dev(m, torch.float32, d, "m") if m is not None else None, beta, tau,
        _dev(neg, _BITS, n, "neg"), _dev(zero, _BITS, n, "zero"), d, _stream(stream)))


def quorum_vote(neg, zero, quorum, voted_neg, voted_zero, d, stream=None):
    """ss_quorum_vote: the server's ternary answer from the workers' planes"""
    L = load_library()
    n = L.ss_packed_bytes(d) // 4
    np_ = [_dev(t, _BITS, n, "neg[%d]" % i) for i, t in enumerate(neg)]
    zp = [_dev(t, _BITS, n, "zero[%d]" % i) for i, t in enumerate(zero)]
    if len(np_) != len(zp):
        raise ValueError("one neg and one zero plane per worker")
    _check("ss_quorum_vote", L.ss_quorum_vote(_ptr_array(np_), _ptr_array(zp), len(np_), quorum,
                                              _dev(voted_neg, _BITS, n, "voted_neg"),
                                              _dev(voted_zero, _BITS, n, "voted_zero"), d, _stream(stream)))


def ternary_apply(x, neg, zero, delta, d=None, stream=None):
    """ss_ternary_apply: x <- x - delta * answer"""
    L = load_library()
    d = x.numel() if d is None else d
    n = L.ss_packed_words(d)
    _check("ss_ternary_apply", L.ss_ternary_apply(_dev(x, torch.float32, d, "x"), _dev(neg, _BITS, n, "neg"),
                                                  _dev(zero, _BITS, n, "zero"), delta, d, _stream(stream)))


def signum_vote_step_ternary(g, m, beta, tau, quorum, delta, x, voted_neg, voted_zero, d=None, stream=None):
    """ss_signum_vote_step_ternary: the whole step with abstention in one pass"""
    L = load_library()
    M = len(g)
    d = x.numel() if d is None else d
    n = L.ss_packed_bytes(d) // 4
    gp = [_dev(t, g[0].dtype, d, "g[%d]" % i) for i, t in enumerate(g)]
    mp = [_dev(t, torch.float32, d, "m[%d]" % i) for i, t in enumerate(m)] if m is not None else None
    if mp is not None and len(mp) != M:
        raise ValueError("one momentum buffer per worker")
    _check("ss_signum_vote_step_ternary", L.ss_signum_vote_step_ternary(
        _ptr_array(gp), _grad_dtype(g[0]), _ptr_array(mp) if mp is not None else None, M, beta, tau, quorum, delta,
        _dev(x, torch.float32, d, "x"), _dev(voted_neg, _BITS, n, "voted_neg"),
        _dev(voted_zero, _BITS, n, "voted_zero"), d, _stream(stream)))
