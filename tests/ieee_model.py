"""Exact-arithmetic model of IEEE-754 binary formats, written from the
standard's definition of roundTiesToEven with Python integers and Fractions.

Used only by the tests that pin the CPU oracle: it shares nothing with the
oracle's C++ (no float arithmetic happens here at all) and nothing with the
HIP library.
"""
from fractions import Fraction

# (precision p incl. hidden bit, emin, emax, total width[, bias, ieee_like])
# bias defaults to emax (true for every IEEE interchange format); ieee_like
# False marks OCP E4M3: no infinity, the top exponent holds ordinary numbers and
# only S.1111.111 is NaN.
BINARY32 = (24, -126, 127, 32)
BFLOAT16 = (8, -126, 127, 16)
BINARY16 = (11, -14, 15, 16)
E5M2 = (3, -14, 15, 8)
E4M3 = (4, -6, 8, 8, 7, False)


def _bias(fmt):
    return fmt[4] if len(fmt) > 4 else fmt[2]


def _ieee_like(fmt):
    return fmt[5] if len(fmt) > 5 else True


def decode(bits: int, fmt):
    """bits -> ('nan'|'inf'|'num', sign, Fraction magnitude)."""
    p, emin, emax, width = fmt[:4]
    ebits = width - p
    sign = bits >> (width - 1)
    e = (bits >> (p - 1)) & ((1 << ebits) - 1)
    f = bits & ((1 << (p - 1)) - 1)
    if _ieee_like(fmt):
        if e == (1 << ebits) - 1:
            return ("nan" if f else "inf", sign, None)
    elif e == (1 << ebits) - 1 and f == (1 << (p - 1)) - 1:
        return ("nan", sign, None)
    if e == 0:
        return ("num", sign, Fraction(f, 1) * Fraction(2) ** (emin - (p - 1)))
    return ("num", sign, Fraction((1 << (p - 1)) | f, 1) * Fraction(2) ** (e - _bias(fmt) - (p - 1)))


def value(bits: int, fmt) -> Fraction:
    kind, sign, mag = decode(bits, fmt)
    assert kind == "num"
    return -mag if sign else mag


def encode_rne(q: Fraction, fmt, zero_sign: int = 0) -> int:
    """Nearest representable value to the exact rational q, ties to even;
    overflow goes to infinity. An exact zero takes zero_sign."""
    p, emin, emax, width = fmt[:4]
    ebits = width - p
    if q == 0:
        return zero_sign << (width - 1)
    sign = 1 if q < 0 else 0
    a = -q if sign else q
    # floor(log2(a))
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    e_q = max(e, emin)
    quantum = Fraction(2) ** (e_q - (p - 1))
    m = a / quantum
    lo = m.numerator // m.denominator
    rem = m - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (lo & 1)):
        lo += 1
    # lo may have reached 2**p (carry): renormalise
    if lo == (1 << p):
        lo >>= 1
        e_q += 1
    if lo >= (1 << (p - 1)):
        # normal number
        if _ieee_like(fmt):
            if e_q > emax:
                return (sign << (width - 1)) | (((1 << ebits) - 1) << (p - 1))   # infinity
        else:
            nan = (1 << (width - 1)) - 1                                       # S.1111.111
            if e_q > emax or (e_q == emax and (lo & ((1 << (p - 1)) - 1)) == (1 << (p - 1)) - 1):
                return (sign << (width - 1)) | nan                              # beyond the largest number
        biased = e_q + _bias(fmt)
        return (sign << (width - 1)) | (biased << (p - 1)) | (lo & ((1 << (p - 1)) - 1))
    # subnormal (or zero after rounding)
    assert e_q == emin
    return (sign << (width - 1)) | lo


def add_rne(x_bits: int, y_bits: int, fmt=BINARY32) -> int:
    """fl(x + y) on bit patterns, finite operands."""
    kx, sx, mx = decode(x_bits, fmt)
    ky, sy, my = decode(y_bits, fmt)
    assert kx == "num" and ky == "num"
    if mx == 0 and my == 0:
        # (+0)+(+0)=+0, (-0)+(-0)=-0, mixed = +0 under roundTiesToEven
        return encode_rne(Fraction(0), fmt, zero_sign=1 if (sx and sy) else 0)
    q = (-mx if sx else mx) + (-my if sy else my)
    return encode_rne(q, fmt, zero_sign=0)


def mul_rne(x_bits: int, y_bits: int, fmt=BINARY32) -> int:
    kx, sx, mx = decode(x_bits, fmt)
    ky, sy, my = decode(y_bits, fmt)
    assert kx == "num" and ky == "num"
    sign = sx ^ sy
    q = mx * my
    if q == 0:
        return encode_rne(Fraction(0), fmt, zero_sign=sign)
    out = encode_rne(-q if sign else q, fmt)
    if out & ~(1 << (fmt[3] - 1)) == 0:
        # underflow to zero keeps the product's sign
        return sign << (fmt[3] - 1)
    return out


def narrow_f32_to_bf16(x_bits: int) -> int:
    kind, s, m = decode(x_bits, BINARY32)
    if kind == "inf":
        return (s << 15) | 0x7F80
    assert kind == "num"
    if m == 0:
        return s << 15
    out = encode_rne(-m if s else m, BFLOAT16)
    if out & 0x7FFF == 0:
        return s << 15
    return out


def narrow_f32_to_f16(x_bits: int) -> int:
    kind, s, m = decode(x_bits, BINARY32)
    if kind == "inf":
        return (s << 15) | 0x7C00
    assert kind == "num"
    if m == 0:
        return s << 15
    out = encode_rne(-m if s else m, BINARY16)
    if out & 0x7FFF == 0:
        return s << 15
    return out


def widen_f16_to_f32(h_bits: int) -> int:
    kind, s, m = decode(h_bits, BINARY16)
    if kind == "inf":
        return (s << 31) | 0x7F800000
    assert kind == "num"
    if m == 0:
        return s << 31
    return encode_rne(-m if s else m, BINARY32)


def widen_fp8_to_f32(b_bits: int, fmt) -> int:
    kind, s, m = decode(b_bits, fmt)
    if kind == "inf":
        return (s << 31) | 0x7F800000
    assert kind == "num"
    if m == 0:
        return s << 31
    return encode_rne(-m if s else m, BINARY32)


def narrow_f32_to_fp8(x_bits: int, fmt) -> int:
    """binary32 -> E5M2 / E4M3: RNE; overflow (and, for E4M3, infinity) gives
    infinity where the format has one, NaN where it has none."""
    kind, s, m = decode(x_bits, BINARY32)
    if kind == "inf":
        return (s << 7) | (0x7C if _ieee_like(fmt) else 0x7F)
    assert kind == "num"
    if m == 0:
        return s << 7
    out = encode_rne(-m if s else m, fmt)
    if out & 0x7F == 0:
        return s << 7
    return out
