"""Exact-arithmetic brute force used to pin the CPU oracle.

Everything here works on python ints and fractions.Fraction: no hardware
floating point takes part in a result, so the rounding order the oracle claims
(each product rounded, then the sum rounded, round-to-nearest-even, subnormals
kept) is checked against the definition of IEEE-754 binary32 rounding itself.
Pure python loops: small inputs only.
"""
import struct
from fractions import Fraction


def f32_bits(x):
    """bit pattern of a numpy.float32 / python float that is exactly an fp32"""
    return struct.unpack("<I", struct.pack("<f", float(x)))[0]


def bits_f32(b):
    return struct.unpack("<f", struct.pack("<I", b & 0xFFFFFFFF))[0]


def round_f32(q):
    """Round the rational q to the nearest binary32 value, ties to even.
    Returns a Fraction (the value of that binary32).  No overflow handling:
    callers stay far from FLT_MAX."""
    q = Fraction(q)
    if q == 0:
        return Fraction(0)
    sign = -1 if q < 0 else 1
    a = abs(q)
    # exponent e with 2^e <= a < 2^(e+1)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    e = max(e, -126)                      # subnormals share the exponent -126
    ulp = Fraction(2) ** (e - 23)
    n = a / ulp
    lo = n.numerator // n.denominator
    rem = n - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    return sign * lo * ulp


def sign_of(v):
    """the paper's sign with the oracle's reading of zero: -1 if v < 0 else +1"""
    return -1 if v < 0 else 1


def momentum(beta, m, g):
    """Algorithm 2's momentum line with three fp32 roundings.  beta, m, g are
    Fractions holding exact fp32 values.  Returns the new m as a Fraction."""
    omb = round_f32(1 - beta)
    return round_f32(round_f32(beta * m) + round_f32(omb * g))


def momentum_fused(beta, m, g):
    """what a fused multiply-add would give instead (to find inputs that tell
    the two apart)"""
    omb = round_f32(1 - beta)
    return round_f32(beta * m + round_f32(omb * g))


def pack(signs):
    """signs: list of +-1.  Words as the oracle's header lays them out:
    coordinate i -> bit i%32 (LSB first) of word i//32, bit set for -1, zero
    padding to a multiple of 4 words."""
    big = 0
    for i, s in enumerate(signs):
        if s == -1:
            big |= 1 << i
    nwords = (len(signs) + 31) // 32
    nwords += (-nwords) % 4
    return [(big >> (32 * k)) & 0xFFFFFFFF for k in range(nwords)]


def vote(sign_lists):
    """Algorithm 3: sign of the per-coordinate sum of the workers' signs"""
    d = len(sign_lists[0])
    return [sign_of(sum(w[i] for w in sign_lists)) for i in range(d)]


def apply_step(x, s, delta):
    """x - delta*s rounded once to fp32 (x, delta Fractions, s = +-1)"""
    return round_f32(x - delta * s)
