"""The single-rounding bf16 quotient used by the merge kernels, as arithmetic.

The HIP helper `round_div_pack_bf16` (csrc/ckv_device.h) produces bf16(S / n) with ONE rounding from
fp32 operations only: q = S * (1/n), the hardware converter where q is clear of every bf16
midpoint, and otherwise the sign of (q - M) * n + (S - q * n), two fused multiply-adds whose
operands are exact.  This test restates those steps with exactly rounded fp32 operations built on
rational arithmetic and checks them against the correctly rounded quotient, with the reciprocal
forced one ulp off in either direction (the kernel's reciprocal is good to an ulp; powers of two
are exact).  It checks the ALGORITHM; that the kernel follows it bit for bit is what the GPU test
`test_bf16_centroids_are_bit_identical_to_the_oracle` checks.
"""
import math
import random
import struct
from fractions import Fraction


def f32_bits(x):
    return struct.unpack("<I", struct.pack("<f", x))[0]


def bits_f32(u):
    return struct.unpack("<f", struct.pack("<I", u & 0xFFFFFFFF))[0]


def _round_to(x: Fraction, mant_bits: int) -> Fraction:
    """Round-to-nearest-even of a positive rational to a binary float with `mant_bits` fraction bits."""
    e = math.floor(math.log2(float(x)))
    while Fraction(2) ** e > x:
        e -= 1
    while Fraction(2) ** (e + 1) <= x:
        e += 1
    scaled = x / Fraction(2) ** (e - mant_bits)
    k = scaled.numerator // scaled.denominator
    rem = scaled - k
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (k & 1)):
        k += 1
    return Fraction(k) * Fraction(2) ** (e - mant_bits)


def rn_f32(x: Fraction) -> float:
    if x == 0:
        return 0.0
    return float(_round_to(abs(x), 23)) * (-1 if x < 0 else 1)


def rn_bf16_bits(x: Fraction) -> int:
    if x == 0:
        return 0
    return (f32_bits(float(_round_to(abs(x), 7))) >> 16) | (0x8000 if x < 0 else 0)


def fma32(a, b, c):
    return rn_f32(Fraction(a) * Fraction(b) + Fraction(c))


def kernel_rounding(S: float, n: int, ulp_off: int) -> int:
    """Upper 16 bits of the bf16 the kernel's steps produce for S / n."""
    fn = float(n)
    pow2 = (n & (n - 1)) == 0
    rcp = bits_f32(f32_bits(rn_f32(Fraction(1, n))) + (0 if pow2 else ulp_off))
    q = rn_f32(Fraction(S) * Fraction(rcp))
    u = f32_bits(q)
    near_midpoint = (((u & 0xFFFF) - 0x7FFD) & 0xFFFF) <= 6
    if pow2 or not near_midpoint:
        return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) & 0xFFFF          # the converter: nearest even
    H = u & 0xFFFF0000
    M = bits_f32(H | 0x8000)
    r = fma32(-q, fn, S)
    if r == 0.0:                                                          # q * n == S: q is the quotient
        return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) & 0xFFFF
    d = fma32(rn_f32(Fraction(q) - Fraction(M)), fn, r)
    if d == 0.0:
        up = (H >> 16) & 1
    else:
        up = 1 if ((d > 0) == ((u >> 31) == 0)) else 0
    return ((H >> 16) + up) & 0xFFFF


def test_single_rounding_of_the_quotient_is_exact_for_any_reciprocal_within_an_ulp():
    rng = random.Random(1)

    def bf16_val():
        return rng.choice([-1, 1]) * rng.randint(128, 255) * 2.0 ** (rng.randint(-8, 6) - 7)

    tested = in_window = 0
    for trial in range(12000):
        k = rng.choice([2, 3, 3, 5, 6, 7, 9, 10, 12, 17, 100, 513, 1025, 4099, 70001, 1048575])
        terms = rng.randint(2, 6)
        ws = [rng.randint(1, max(1, k // terms)) for _ in range(terms)]
        n = sum(ws)
        acc = 0.0
        for w in ws:                                   # a weighted fp32 sum of bf16 values, as the kernel forms it
            acc = fma32(float(w), bf16_val(), acc)
        if trial % 3 == 0:                             # adversarial: put the quotient next to a bf16 midpoint
            target = bits_f32((f32_bits(bf16_val()) & 0xFFFF0000) | 0x8000)
            jitter = Fraction(rng.randint(-3, 3)) * Fraction(2) ** (math.frexp(target * n)[1] - 24) if trial % 6 == 0 else 0
            acc = rn_f32(Fraction(target) * n + jitter)
        if acc == 0.0:
            continue
        ref = rn_bf16_bits(Fraction(acc) / n)
        tested += 1
        u = f32_bits(rn_f32(Fraction(acc) * Fraction(rn_f32(Fraction(1, n)))))
        in_window += (((u & 0xFFFF) - 0x7FFD) & 0xFFFF) <= 6
        for off in (-1, 0, 1):
            assert kernel_rounding(acc, n, off) == ref, (acc, n, off)
    assert tested > 10000 and in_window > 2000
