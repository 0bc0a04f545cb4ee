"""Exact-rational re-evaluation of the block step, for tiny inputs.  TEST INFRASTRUCTURE.

Every fp32 operation of the step is carried out on python Fractions (infinitely precise) and then
rounded to the nearest fp32 value, ties to even, with gradual underflow -- i.e. IEEE-754 binary32
arithmetic built from its definition rather than from a floating-point unit.  It follows the same
reading of the update as lohan_oracle.c (Sec. IV-C "CPU Compute" step; Table II tensors; Adam per
Sec. II; the numerical conventions are restated in the code below) but shares no code with it, so that
agreement between the two pins the C file's conversions, rounding and compiler flags.

Only finite values are supported (an overflow to infinity raises); pure-python loops, so keep
n in the hundreds.
"""
import math
import struct
from fractions import Fraction

_F32_MIN_EXP = -126      # exponent of the smallest normal
_F32_MANT = 23
_F32_MAX = Fraction((2 ** 24 - 1) * 2 ** (127 - 23))


def _floor_log2(x: Fraction) -> int:
    """floor(log2(x)) for x > 0, exactly."""
    e = x.numerator.bit_length() - x.denominator.bit_length()
    if Fraction(2) ** e > x:
        e -= 1
    elif Fraction(2) ** (e + 1) <= x:
        e += 1
    return e


def _round_int_ties_even(k: Fraction) -> int:
    fl = math.floor(k)
    rem = k - fl
    if rem > Fraction(1, 2):
        return fl + 1
    if rem < Fraction(1, 2):
        return fl
    return fl if fl % 2 == 0 else fl + 1


def rn32(x: Fraction) -> Fraction:
    """Nearest binary32 value to the exact rational x (ties to even, subnormals kept)."""
    if x == 0:
        return Fraction(0)
    sign = -1 if x < 0 else 1
    a = abs(x)
    e = max(_floor_log2(a), _F32_MIN_EXP)
    quantum = Fraction(2) ** (e - _F32_MANT)
    r = _round_int_ties_even(a / quantum) * quantum
    if r > _F32_MAX:
        raise OverflowError("result overflows binary32")
    return sign * r


def sqrt32(x: Fraction) -> Fraction:
    """Correctly rounded binary32 square root of an exact rational x >= 0."""
    if x < 0:
        raise ValueError("sqrt of a negative value")
    if x == 0:
        return Fraction(0)
    e = max(_floor_log2(x) // 2, _F32_MIN_EXP)     # sqrt(x) in [2^e, 2^(e+1)) when not subnormal
    quantum = Fraction(2) ** (e - _F32_MANT)
    k = math.isqrt(math.floor(x / (quantum * quantum)))   # floor(sqrt(x)/quantum)
    mid = (Fraction(k) + Fraction(1, 2)) * quantum
    if mid * mid < x:
        k += 1
    elif mid * mid == x and k % 2 == 1:
        k += 1
    return k * quantum


def f32_bits_to_frac(b: int) -> Fraction:
    sign = -1 if (b >> 31) & 1 else 1
    expo = (b >> 23) & 0xFF
    frac = b & 0x7FFFFF
    if expo == 0xFF:
        raise OverflowError("non-finite binary32 input")
    if expo == 0:
        return sign * Fraction(frac) * Fraction(2) ** (-149)
    return sign * Fraction(frac | 0x800000) * Fraction(2) ** (expo - 150)


def frac_to_f32_bits(x: Fraction) -> int:
    """Bit pattern of a rational that is exactly a binary32 value (sign of zero: +0)."""
    return struct.unpack("<I", struct.pack("<f", float(x)))[0]


def float_to_frac(x) -> Fraction:
    """fp32 rounding of a python/numpy float, as a Fraction."""
    return f32_bits_to_frac(struct.unpack("<I", struct.pack("<f", float(x)))[0])


def half_bits_to_frac(h: int) -> Fraction:
    sign = -1 if (h >> 15) & 1 else 1
    expo = (h >> 10) & 0x1F
    frac = h & 0x3FF
    if expo == 0x1F:
        raise OverflowError("non-finite binary16 input")
    if expo == 0:
        return sign * Fraction(frac, 2 ** 24)
    return sign * Fraction(frac | 0x400) * Fraction(2) ** (expo - 25)


def bf16_bits_rne(x: Fraction) -> int:
    """bfloat16 bit pattern nearest to a binary32 value x (ties to even): 8 significant bits,
    same exponent range as binary32."""
    if x == 0:
        return 0
    sign = 0x8000 if x < 0 else 0
    a = abs(x)
    e = max(_floor_log2(a), _F32_MIN_EXP)
    quantum = Fraction(2) ** (e - 7)
    k = _round_int_ties_even(a / quantum)
    r = k * quantum
    bits32 = frac_to_f32_bits(r)       # r is a bf16 value, hence exactly a binary32 value
    return sign | (bits32 >> 16)


def half_bits_rne(x: Fraction) -> int:
    """binary16 bit pattern nearest to x (ties to even): 11 significant bits, smallest normal
    2^-14, quantum 2^-24 below it, 65520 and above round to infinity."""
    if x == 0:
        return 0
    sign = 0x8000 if x < 0 else 0
    a = abs(x)
    e = max(_floor_log2(a), -14)
    quantum = Fraction(2) ** (e - 10)
    r = _round_int_ties_even(a / quantum) * quantum
    if r >= 65536:
        return sign | 0x7C00
    if r == 0:
        return sign
    er = _floor_log2(r)
    if er < -14:
        return sign | int(r / Fraction(2) ** -24)
    return sign | ((er + 15) << 10) | (int(r / Fraction(2) ** (er - 10)) - 1024)


def scalars(lr, beta1, beta2, wd, step, loss_scale):
    """Per-call scalars as Fractions (each an exact binary32 value)."""
    lr, beta1, beta2, wd, S = map(float_to_frac, (lr, beta1, beta2, wd, loss_scale))
    one = Fraction(1)
    return {
        "inv": rn32(one / S),
        "omb1": rn32(one - beta1),
        "omb2": rn32(one - beta2),
        # the float64 value of 1 - beta^t is within 2^-51 of the exact one; rounding the exact
        # one to binary32 gives the same result unless it sits that close to a rounding
        # boundary, which the tests that use this evaluator check for.
        "bc1": rn32(one - beta1 ** step),
        "bc2": rn32(one - beta2 ** step),
        "lr": lr, "beta1": beta1, "beta2": beta2, "wd": wd,
    }


def adam_block_step_exact(p_bits, m_bits, v_bits, g16_bits, *, lr, beta1, beta2, eps,
                          weight_decay, step, loss_scale, l2_mode=False, half_out=False):
    """Lists of binary32 bit patterns in, (p', m', v', bf16) lists of bit patterns out."""
    s = scalars(lr, beta1, beta2, weight_decay, step, loss_scale)
    eps = float_to_frac(eps)
    sbc2 = sqrt32(s["bc2"])
    ss = rn32(s["lr"] / s["bc1"])
    decay = rn32(Fraction(1) - rn32(s["lr"] * s["wd"]))
    out_p, out_m, out_v, out_h = [], [], [], []
    for pb, mb, vb, gb in zip(p_bits, m_bits, v_bits, g16_bits):
        p, m, v = f32_bits_to_frac(pb), f32_bits_to_frac(mb), f32_bits_to_frac(vb)
        g = rn32(half_bits_to_frac(gb) * s["inv"])
        if l2_mode:
            g = rn32(g + rn32(s["wd"] * p))
        m_new = rn32(rn32(s["beta1"] * m) + rn32(s["omb1"] * g))
        v_new = rn32(rn32(s["beta2"] * v) + rn32(s["omb2"] * rn32(g * g)))
        den = rn32(rn32(sqrt32(v_new) / sbc2) + eps)
        u = rn32(m_new / den)
        pp = p if l2_mode else rn32(p * decay)
        p_new = rn32(pp - rn32(ss * u))
        out_p.append(frac_to_f32_bits(p_new))
        out_m.append(frac_to_f32_bits(m_new))
        out_v.append(frac_to_f32_bits(v_new))
        out_h.append(half_bits_rne(p_new) if half_out else bf16_bits_rne(p_new))
    return out_p, out_m, out_v, out_h
