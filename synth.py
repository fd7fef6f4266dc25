"""Seeded synthetic inputs for the signSGD / Signum majority-vote step.

Serves BOTH the CPU oracle's tests and the HIP path's tests and benchmark, and
therefore holds none of the method's arithmetic: only random draws and the
recipes that turn them into gradients, initial parameters and initial
momentum.  Whoever compares two implementations generates a block ONCE here
and hands the same bytes to both.

Every block is addressed by (config, role, step, worker, chunk): a chunk is
CHUNK consecutive coordinates, and its values depend only on that key and on
the device type that draws them (torch's generators are counter based; the
host and the GPU draw different streams, which is why a block is generated on
one device and copied, never generated twice).  Any chunk can be produced in
any order, so a d = 1.5e9 configuration can be checked on sampled chunks.

The gradients stand in for mini-batch gradients of the networks the paper
trains (Section 2, "Experimental benchmarks"): dense, with unimodal, symmetric,
roughly Gaussian noise around a fixed mean (Figures 1 and 2).
"""
from dataclasses import dataclass, replace
from itertools import combinations

import torch

S0 = 180204434
CHUNK = 1 << 22

_ROLES = {"mu": 1, "x0": 2, "noise": 3, "zero_mask": 4, "tie_mask": 5, "tie_pattern": 6}
_MASK64 = (1 << 64) - 1


def _mix(h):
    """splitmix64 finaliser on a python int"""
    h = (h + 0x9E3779B97F4A7C15) & _MASK64
    h = ((h ^ (h >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    h = ((h ^ (h >> 27)) * 0x94D049BB133111EB) & _MASK64
    return h ^ (h >> 31)


def block_seed(config_id, role, step, worker, chunk):
    h = S0
    for part in (config_id, _ROLES[role], step + 1, worker + 1, chunk + 1):
        h = _mix(h ^ part)
    return h & ((1 << 63) - 1)


@dataclass(frozen=True)
class Config:
    """One workload.  beta is None for Algorithm 1 / 3 without momentum."""
    name: str
    config_id: int
    d: int
    M: int
    grad_dtype: str          # "f32" | "bf16"
    beta: float              # None: no momentum buffers
    delta: float
    steps: int
    mu_kind: str             # "normal" | "laplace" | "none"
    mu_scale: float
    noise_scale: float
    x0_scale: float = 0.05
    zero_frac: float = 0.0   # fraction of gradient entries forced to +0.0
    tie_frac: float = 0.0    # fraction of coordinates forced to an exact M/2 : M/2 split

    def scaled(self, d, steps=None):
        return replace(self, d=d, steps=self.steps if steps is None else steps)

    @property
    def n_chunks(self):
        return (self.d + CHUNK - 1) // CHUNK

    def chunk_range(self, c):
        lo = c * CHUNK
        return lo, min(self.d, lo + CHUNK)


# The five workloads, in the order the benchmark definition lists them.
C1 = Config("C1_tiny_signum_vote", 1, 272_474, 7, "f32", 0.9, 1e-4, 10, "normal", 0.01, 0.1)
C2 = Config("C2_signsgd_single", 2, 25_557_032, 1, "f32", None, 1e-4, 20, "none", 0.0, 1.0,
            zero_frac=0.05)
C3 = Config("C3_signum_vote", 3, 25_557_032, 7, "f32", 0.9, 1e-4, 20, "normal", 0.1, 0.5)
C4 = Config("C4_even_tie", 4, 138_357_544, 16, "f32", 0.9, 1e-4, 10, "normal", 0.1, 1.0,
            tie_frac=0.10)
C5 = Config("C5_bf16_large", 5, 1_500_000_017, 8, "bf16", 0.9, 1e-5, 5, "laplace", 0.05, 1.0)
CONFIGS = {c.name.split("_")[0]: c for c in (C1, C2, C3, C4, C5)}

# Config 2 plants a few special values at fixed coordinates (when d allows):
# negative zero and subnormals of both signs.  (index, fp32 bit pattern)
PLANTED_C2 = ((3, 0x80000000), (35, 0x00000001), (67, 0x80000001),
              (100, 0x007FFFFF), (131, 0x807FFFFF), (164, 0x80000000))


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _randn(cfg, role, step, worker, chunk, n, device):
    return torch.randn(n, generator=_gen(block_seed(cfg.config_id, role, step, worker, chunk), device),
                       device=device, dtype=torch.float32)


def _rand(cfg, role, step, worker, chunk, n, device):
    return torch.rand(n, generator=_gen(block_seed(cfg.config_id, role, step, worker, chunk), device),
                      device=device, dtype=torch.float32)


def mu_chunk(cfg, c, device="cpu"):
    """Mean gradient of chunk c, fixed over steps and workers."""
    lo, hi = cfg.chunk_range(c)
    n = hi - lo
    if cfg.mu_kind == "none":
        return torch.zeros(n, device=device, dtype=torch.float32)
    if cfg.mu_kind == "normal":
        return _randn(cfg, "mu", 0, 0, c, n, device) * cfg.mu_scale
    if cfg.mu_kind == "laplace":
        u = _rand(cfg, "mu", 0, 0, c, n, device) - 0.5
        mag = -torch.log1p(-2.0 * u.abs().clamp(max=0.49999997))
        return cfg.mu_scale * torch.sign(u) * mag
    raise ValueError(cfg.mu_kind)


def x0_chunk(cfg, c, device="cpu"):
    lo, hi = cfg.chunk_range(c)
    return _randn(cfg, "x0", 0, 0, c, hi - lo, device) * cfg.x0_scale


_TIE_TABLES = {}


def _tie_table(M, device):
    """All M-bit patterns with exactly M/2 ones."""
    key = (M, str(device))
    if key not in _TIE_TABLES:
        pats = [sum(1 << b for b in comb) for comb in combinations(range(M), M // 2)]
        _TIE_TABLES[key] = torch.tensor(pats, dtype=torch.int64, device=device)
    return _TIE_TABLES[key]


def tie_chunk(cfg, c, device="cpu"):
    """(is_tie, pattern): coordinates forced to an exact split, and for each
    the M-bit set of workers whose gradient is positive there (fixed over
    steps, so that each worker's momentum keeps the sign of its gradient)."""
    lo, hi = cfg.chunk_range(c)
    n = hi - lo
    is_tie = _rand(cfg, "tie_mask", 0, 0, c, n, device) < cfg.tie_frac
    table = _tie_table(cfg.M, device)
    idx = torch.randint(0, table.numel(), (n,), device=device,
                        generator=_gen(block_seed(cfg.config_id, "tie_pattern", 0, 0, c), device))
    return is_tie, table[idx]


def grad_chunk(cfg, step, worker, c, device="cpu", mu=None, tie=None):
    """Worker `worker`'s stochastic gradient for chunk c at step `step`:
    torch.float32, or torch.bfloat16 (rounded once, here) for bf16 configs.
    mu / tie may be passed in when the caller already holds this chunk's."""
    lo, hi = cfg.chunk_range(c)
    n = hi - lo
    z = _randn(cfg, "noise", step, worker, c, n, device)
    if mu is None:
        mu = mu_chunk(cfg, c, device)
    g = mu + cfg.noise_scale * z
    if cfg.zero_frac > 0.0:
        zero = _rand(cfg, "zero_mask", step, worker, c, n, device) < cfg.zero_frac
        g = torch.where(zero, torch.zeros_like(g), g)
        if c == 0:
            gi = g.view(torch.int32)
            for idx, bits in PLANTED_C2:
                if idx < n:
                    gi[idx] = bits - (1 << 32) if bits >= (1 << 31) else bits
    if cfg.tie_frac > 0.0:
        is_tie, pattern = tie_chunk(cfg, c, device) if tie is None else tie
        positive = ((pattern >> worker) & 1).bool()
        mag = z.abs().clamp(min=2.0 ** -20)
        g = torch.where(is_tie, torch.where(positive, mag, -mag), g)
    if cfg.grad_dtype == "bf16":
        g = g.to(torch.bfloat16)
    return g


def as_numpy(t):
    """Host numpy view for the oracle: float32 stays float32, bf16 becomes its
    uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    return t.numpy()
