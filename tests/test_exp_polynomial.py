"""The softmax exponential of the INT8 attention kernels (csrc/attention.hip, exp_nonpos) is a binary64 polynomial
whose result is rounded to binary32; the rounding is the correct one only if the polynomial is accurate far beyond a
binary32 ulp.  This test reads the constants out of the kernel source and replays the function on the CPU with every
fused multiply-add evaluated exactly (rational arithmetic, one rounding), against a 60-digit exponential."""
import math
import os
import random
import re
import struct
from decimal import Decimal, getcontext
from fractions import Fraction

SRC = os.path.join(os.path.dirname(__file__), "..", "paper_2209_09130_amd", "csrc", "attention.hip")


def fma(a, b, c):
    return float(Fraction(a) * Fraction(b) + Fraction(c))          # Fraction -> float rounds to nearest even


def constants():
    text = open(SRC).read()
    body = text[text.index("double exp_nonpos(double x)"):]
    body = body[:body.index("return __builtin_ldexp")]
    num = r"-?(?:0x[0-9a-fA-F.]+p[-+]?\d+|\d+\.\d+(?:e[-+]?\d+)?)"
    lits = [float.fromhex(t) if "0x" in t else float(t) for t in re.findall(num, body)]
    # in source order: log2 e, the shift (twice: added, then taken off), the two parts of -ln 2, the coefficients
    log2e, shift, shift_again, ln2_hi, ln2_lo = lits[:5]
    assert shift_again == shift
    poly = lits[5:]
    return log2e, shift, ln2_hi, ln2_lo, poly


def exp_nonpos(x, log2e, shift, ln2_hi, ln2_lo, poly):
    shifted = fma(x, log2e, shift)
    k = shifted - shift
    r = fma(k, ln2_hi, x)
    r = fma(k, ln2_lo, r)
    p = poly[0]
    for c in poly[1:]:
        p = fma(p, r, c)
    return math.ldexp(p, int(k)), r


def test_exponential_polynomial_is_accurate_far_beyond_a_binary32_ulp():
    getcontext().prec = 60
    log2e, shift, ln2_hi, ln2_lo, poly = constants()
    assert shift == 1.5 * 2.0 ** 52 and abs(log2e - 1 / math.log(2)) < 1e-15
    assert abs(-(ln2_hi + ln2_lo) - math.log(2)) < 1e-16 and poly[-1] == 1.0 and poly[-2] == 1.0
    f32 = lambda v: struct.unpack("f", struct.pack("f", v))[0]
    rnd = random.Random(11)
    xs = [f32(-rnd.random() * 100) for _ in range(4000)] + [f32(-rnd.random() * 0.7) for _ in range(1500)] + [0.0]
    xs += [f32(-(k + 0.5) * math.log(2)) for k in range(0, 140, 3)]           # the ends of the reduced range
    xs += [-745.0, -700.25, -87.5]
    worst, r_max = 0.0, 0.0
    for x in xs:
        y, r = exp_nonpos(x, log2e, shift, ln2_hi, ln2_lo, poly)
        exact = Fraction(str(Decimal(x).exp()))
        if exact > Fraction(1, 2 ** 1000):                                   # normal results
            worst = max(worst, float(abs(Fraction(y) - exact) / exact))
        r_max = max(r_max, abs(r))
    assert r_max <= 0.34665, r_max                                            # the interval the polynomial was fitted on
    assert worst < 2.0 ** -48, math.log2(worst)
    assert exp_nonpos(0.0, log2e, shift, ln2_hi, ln2_lo, poly)[0] == 1.0
    # far below the range of binary32 the scaling flushes to zero, as the exponential does
    assert exp_nonpos(-1.0e9, log2e, shift, ln2_hi, ln2_lo, poly)[0] == 0.0
