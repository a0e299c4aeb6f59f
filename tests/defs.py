"""Definition checker used by the oracle's pins: exact rational arithmetic (fractions) and
exhaustive nearest-value search over explicit value tables.  It calls nothing under oracle/
and nothing of the HIP path: it is the independent yardstick both are held against.

Tables for E2M1 / E2M3 / E3M2 are the literal ones in tests/golden/ocp_element_values.txt.
E4M3 and the integer formats are enumerated from the format definition (sign | exponent |
mantissa with bias 2^(eta-1)-1; two's complement) and cross-checked against the file's spots.
"""
import functools
import math
import os
from fractions import Fraction

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")

FP_SHAPES = {"e4m3": (4, 3), "e3m3": (3, 3), "e3m2": (3, 2), "e2m3": (2, 3), "e2m2": (2, 2), "e2m1": (2, 1)}
INT_BITS = {"int8": 8, "int7": 7, "int6": 6, "int5": 5, "int4": 4, "int3": 3, "int2": 2}
ALL_FORMATS = list(INT_BITS) + list(FP_SHAPES)


def is_int(fmt):
    return fmt in INT_BITS


def bits_of(fmt):
    return INT_BITS[fmt] if is_int(fmt) else 1 + sum(FP_SHAPES[fmt])


@functools.lru_cache(maxsize=None)
def read_golden_values():
    """{fmt: {code: Fraction or None (NaN)}} from the literal OCP table file."""
    out = {}
    with open(os.path.join(GOLDEN, "ocp_element_values.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            fmt, code, val = line.split()
            out.setdefault(fmt, {})[int(code, 16)] = None if val == "nan" else Fraction(val)
    return out


def fp_value(eta, mu, code):
    """Value of an MXFP code as a Fraction; None for the E4M3 NaN codes."""
    bias = 2 ** (eta - 1) - 1
    m = code & (2 ** mu - 1)
    e = (code >> mu) & (2 ** eta - 1)
    s = (code >> (eta + mu)) & 1
    if (eta, mu) == (4, 3) and e == 15 and m == 7:
        return None
    if e == 0:
        mag = Fraction(m, 2 ** mu) * Fraction(2) ** (1 - bias)
    else:
        mag = (1 + Fraction(m, 2 ** mu)) * Fraction(2) ** (e - bias)
    return -mag if s else mag


@functools.lru_cache(maxsize=None)
def value_table(fmt):
    """[(code, Fraction)] of every finite code of the element format."""
    if is_int(fmt):
        b = INT_BITS[fmt]
        return [(c, Fraction(c if c < 2 ** (b - 1) else c - 2 ** b)) for c in range(2 ** b)]
    eta, mu = FP_SHAPES[fmt]
    golden = read_golden_values().get(fmt, {})
    n = 2 ** (1 + eta + mu)
    if len(golden) * 2 == n:                     # a complete literal table of magnitudes
        sign = n // 2
        return [(c, v) for c, v in golden.items()] + [(c | sign, -v) for c, v in golden.items()]
    tab = []
    for c in range(n):
        v = fp_value(eta, mu, c)
        if v is not None:
            tab.append((c, v))
    return tab


@functools.lru_cache(maxsize=None)
def emax(fmt):
    """Exponent of the largest normal (largest magnitude for MXINT) found from the table itself."""
    top = max(v for _, v in value_table(fmt))
    e = 0
    while Fraction(2) ** (e + 1) <= top:
        e += 1
    return e


def floor_log2(x):
    x = Fraction(x)
    assert x > 0
    e = 0
    while Fraction(2) ** e > x:
        e -= 1
    while Fraction(2) ** (e + 1) <= x:
        e += 1
    return e


@functools.lru_cache(maxsize=None)
def _candidates(fmt, neg):
    tab = value_table(fmt)
    if is_int(fmt):
        b = INT_BITS[fmt]
        return tuple((c, v) for c, v in tab if abs(v) <= 2 ** (b - 1) - 1)
    sign_bit = 2 ** (bits_of(fmt) - 1)
    return tuple((c, v) for c, v in tab if bool(c & sign_bit) == neg)      # keep the sign, also of zero


def nearest_code(fmt, r, tie="default", negative_zero=False):
    """Exhaustive search for the representable value nearest to r (a Fraction).

    Ties: MXINT default = away from zero; MXFP default = even mantissa (even code).
    MXINT uses the symmetric range (the most negative code is never produced).
    Values beyond the largest magnitude fall on it (saturation) by the search itself.
    """
    r = Fraction(r)
    if is_int(fmt):
        rule = "away" if tie in ("default", "away") else "even"
    else:
        rule = "even" if tie in ("default", "even") else "away"
    neg = r < 0 or (r == 0 and negative_zero)
    cand = _candidates(fmt, neg)
    best = min(abs(v - r) for _, v in cand)
    hits = [(c, v) for c, v in cand if abs(v - r) == best]
    if len(hits) == 1:
        return hits[0][0]
    assert len(hits) == 2
    if rule == "away":
        return max(hits, key=lambda cv: abs(cv[1]))[0]
    if is_int(fmt):
        return [c for c, v in hits if v % 2 == 0][0]
    return [c for c, v in hits if c % 2 == 0][0]


def quantize_block(fmt, values, tie="default"):
    """Eq. (1) + Eq. (2) on a list of finite Python floats: (scale byte, [codes])."""
    amax = max(abs(Fraction(float(v))) for v in values)
    shared = -127 if amax == 0 else floor_log2(amax) - emax(fmt)      # log2(0) = -inf clamps to -127
    shared = max(-127, min(127, shared))
    x = Fraction(2) ** shared
    codes = []
    for v in values:
        v = float(v)
        neg_zero = v == 0 and math.copysign(1.0, v) < 0
        codes.append(nearest_code(fmt, Fraction(v) / x, tie, negative_zero=neg_zero))
    return shared + 127, codes


def float_to_fraction(v):
    return Fraction(float(v))
