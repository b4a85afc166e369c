"""Exact-rational helpers for the oracle's pins: format value tables built straight from
Eq. (1) of the paper with `fractions.Fraction`, neighbours by bisection, and the expected
round-up probabilities of each predicate written as counting arguments over integers.
Nothing here calls the oracle or the GPU library."""
import bisect
from fractions import Fraction

import numpy as np

FORMATS = {
    # fmt id: (name, K, P, B, has_inf)
    0: ("bf16", 16, 8, 127, True),
    1: ("e4m3", 8, 4, 7, False),
    2: ("e5m2", 8, 3, 15, True),
}
MAX_FINITE = {0: Fraction(2 ** 8 - 1, 2 ** 7) * Fraction(2) ** 127, 1: Fraction(448), 2: Fraction(57344)}


def pow2(k):
    return Fraction(2) ** k


def code_value(code, fmt):
    """Eq. (1) for a non-negative code; None for inf / NaN encodings."""
    _, K, P, B, has_inf = FORMATS[fmt]
    tbits = P - 1
    e = code >> tbits
    t = code & ((1 << tbits) - 1)
    emax = (1 << (K - 1 - tbits)) - 1
    if has_inf and e == emax:
        return None
    if not has_inf and code == (1 << (K - 1)) - 1:
        return None
    if e == 0:
        return Fraction(t) * pow2(1 - P) * pow2(1 - B)
    return (1 + Fraction(t) * pow2(1 - P)) * pow2(e - B)


_tables = {}


def finite_table(fmt):
    """Sorted (values, codes) of all non-negative finite codes."""
    if fmt not in _tables:
        K = FORMATS[fmt][1]
        pairs = []
        for code in range(1 << (K - 1)):
            v = code_value(code, fmt)
            if v is not None:
                pairs.append((v, code))
        pairs.sort()
        _tables[fmt] = ([p[0] for p in pairs], [p[1] for p in pairs])
    return _tables[fmt]


def neighbours(a, fmt):
    """(lo_code, hi_code) bracketing the non-negative Fraction a <= M (equal if representable)."""
    vals, codes = finite_table(fmt)
    i = bisect.bisect_right(vals, a) - 1
    if vals[i] == a:
        return codes[i], codes[i]
    return codes[i], codes[i + 1]


def f32_fraction(x):
    """Exact value of an fp32 number as a Fraction."""
    return Fraction(float(np.float32(x)))


def delta_of(a, fmt):
    """(floor value code lo, delta) with delta = position of a between its neighbours in [0,1)."""
    vals, codes = finite_table(fmt)
    i = bisect.bisect_right(vals, a) - 1
    if vals[i] == a:
        return codes[i], Fraction(0)
    return codes[i], (a - vals[i]) / (vals[i + 1] - vals[i])


def floor_frac(q):
    return q.numerator // q.denominator


def rne_int(q):
    """Nearest integer to the Fraction q, ties to even."""
    f = floor_frac(q)
    r = q - f
    if r > Fraction(1, 2) or (r == Fraction(1, 2) and f % 2 == 1):
        return f + 1
    return f


def expected_ups(delta, variant, N):
    """Number of n in [0, 2^N) that round up, from the predicates of Sec. II-B / Eq. (7),
    as closed counting arguments (delta a Fraction in [0,1)):
      SRFF: delta + n/2^N >= 1        <=>  n >= 2^N - floor(delta 2^N)      -> floor(delta 2^N)
      SRF : delta + (2n+1)/2^(N+1)>=1 <=>  2n+1 >= 2^(N+1) - floor(delta 2^(N+1))
      SRC : SRFF on h/2^N with h = RNE(delta 2^N)                            -> h
    """
    if variant == 1:
        return floor_frac(delta * 2 ** N)
    if variant == 2:
        g = floor_frac(delta * 2 ** (N + 1))
        # n >= (2^(N+1) - g - 1)/2  -> count of n in [0,2^N)
        need = 2 ** (N + 1) - g - 1          # 2n >= need
        nmin = max(0, -((-need) // 2))       # ceil(need/2)
        return max(0, 2 ** N - nmin)
    if variant == 3:
        return min(rne_int(delta * 2 ** N), 2 ** N)
    raise ValueError(variant)
