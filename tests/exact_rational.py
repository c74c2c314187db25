"""Exact-rational brute-force model of the schedule, for tiny inputs only.

Independent of oracle/: no float addition and no bit-trick rounding.  Every sum is formed
exactly with fractions.Fraction and then rounded to the target format by searching the
sorted table of that format's finite values for the nearest one (ties to the value whose
last significand bit is 0; beyond max + half an ulp gives infinity).  binary32 rounding of
an exact two-term sum goes through Python's correctly rounded Fraction -> float (binary64)
followed by numpy's binary64 -> binary32 cast; the intermediate rounding is harmless
because 53 >= 2*24 + 2.

The expression per element is written out from Algorithm 1 / Section 4.1 of the paper:
  node sum    s(r_n) = bf( f32(..f32(f32(x_0 + x_1) + x_2).. + x_{G-1}) )   local rank order
  step l      v_{l+1}(r_n) = bf( v_l(r_n) + v_l(r_n XOR 2^l) )
  result      v_L(r_n) for every rank of node r_n
where bf() narrows to the message type (identity for fp32 messages).  For N = 2^L + r that is not
a power of two the first 2r node sums are first added pairwise, bf(s(2i) + s(2i+1)), and the
steps run over those r values followed by the remaining nodes' sums.
"""
from __future__ import annotations

import bisect
import math
import struct
from fractions import Fraction

import numpy as np

# ---- bf16 value table -------------------------------------------------------------------


def bf16_bits_to_fraction(b: int) -> Fraction:
    sign = -1 if b & 0x8000 else 1
    e = (b >> 7) & 0xFF
    m = b & 0x7F
    if e == 0xFF:
        raise ValueError("non-finite")
    if e == 0:
        return sign * Fraction(m, 1 << 7) * Fraction(2) ** (-126)
    return sign * (1 + Fraction(m, 1 << 7)) * Fraction(2) ** (e - 127)


_POS = [(bf16_bits_to_fraction(b), b) for b in range(0x0000, 0x7F80)]  # +0 .. max finite
_POS_VALS = [v for v, _ in _POS]
_OVERFLOW = Fraction(2) ** 128  # stands for infinity when searching for the nearest value


def round_fraction_to_bf16(x: Fraction, zero_sign_negative: bool = False) -> int:
    """Nearest bf16 (bit pattern) to the exact value x, ties to even."""
    if x == 0:
        return 0x8000 if zero_sign_negative else 0x0000
    neg = x < 0
    a = -x if neg else x
    i = bisect.bisect_left(_POS_VALS, a)
    if i < len(_POS_VALS) and _POS_VALS[i] == a:
        bits = _POS[i][1]
    else:
        lo_v, lo_b = _POS[i - 1]
        hi_v, hi_b = (_POS[i] if i < len(_POS) else (_OVERFLOW, 0x7F80))
        d_lo, d_hi = a - lo_v, hi_v - a
        if d_lo < d_hi:
            bits = lo_b
        elif d_hi < d_lo:
            bits = hi_b
        else:
            bits = lo_b if (lo_b & 1) == 0 else hi_b
    return bits | (0x8000 if neg else 0)


# ---- binary32 -----------------------------------------------------------------------------


def f32_to_fraction(f) -> Fraction:
    return Fraction(float(np.float32(f)))


def round_fraction_to_f32(x: Fraction, zero_sign_negative: bool = False) -> np.float32:
    if x == 0:
        return np.float32(-0.0 if zero_sign_negative else 0.0)
    with np.errstate(over="ignore"):
        try:
            d = float(x)
        except OverflowError:
            d = math.inf if x > 0 else -math.inf
        return np.float32(d)


def f32_bits(f) -> int:
    return struct.unpack("<I", struct.pack("<f", float(np.float32(f))))[0]


def _is_neg_zero(f) -> bool:
    return float(f) == 0.0 and math.copysign(1.0, float(f)) < 0


def add_f32_exact(a: np.float32, b: np.float32) -> np.float32:
    """Correctly rounded binary32 a + b via exact rationals (an infinite operand passes through)."""
    if math.isinf(float(a)) or math.isinf(float(b)):
        with np.errstate(invalid="ignore"):
            return np.float32(np.float32(a) + np.float32(b))
    s = f32_to_fraction(a) + f32_to_fraction(b)
    return round_fraction_to_f32(s, zero_sign_negative=_is_neg_zero(a) and _is_neg_zero(b))


# ---- the schedule, element by element --------------------------------------------------


def _widen(v, dtype: str) -> np.float32:
    if dtype == "bf16":
        b = int(v)
        if (b & 0x7FFF) == 0x7F80:      # an infinity produced by an earlier narrowing
            return np.float32(-math.inf if b & 0x8000 else math.inf)
        if (b & 0x7FFF) == 0:
            return np.float32(-0.0 if b & 0x8000 else 0.0)
        return np.float32(float(bf16_bits_to_fraction(b)))
    return np.float32(v)


def _narrow(f: np.float32, dtype: str):
    if dtype == "bf16":
        if math.isnan(float(f)):
            return 0x7FC0
        if math.isinf(float(f)):
            return 0xFF80 if f < 0 else 0x7F80
        return round_fraction_to_bf16(f32_to_fraction(f), zero_sign_negative=_is_neg_zero(f))
    return np.float32(f)


def allreduce_element(vals, G: int, dtype: str):
    """vals[p] for p = r_n*G + r_g -> the value every rank ends with for this element."""
    P = len(vals)
    N = P // G
    node = []
    for r_n in range(N):
        acc = _widen(vals[r_n * G], dtype)
        for g in range(1, G):
            acc = add_f32_exact(acc, _widen(vals[r_n * G + g], dtype))
        node.append(_narrow(acc, dtype))
    # N = 2^L + r: fold the first 2r nodes pairwise (even node's value arrives at the odd node)
    L = N.bit_length() - 1
    r = N - (1 << L)
    vals = []
    for v in range(1 << L):
        if v < r:
            vals.append(_narrow(add_f32_exact(_widen(node[2 * v], dtype), _widen(node[2 * v + 1], dtype)), dtype))
        else:
            vals.append(node[v + r])
    for step in range(L):
        nxt = []
        for v in range(1 << L):
            a = _widen(vals[v], dtype)
            b = _widen(vals[v ^ (1 << step)], dtype)
            nxt.append(_narrow(add_f32_exact(a, b), dtype))
        vals = nxt
    # back to nodes: node 2i and 2i+1 (i < r) share value i, node j >= 2r has value j - r
    return [vals[q // 2] if q < 2 * r else vals[q - r] for q in range(N)]


def allreduce(x: np.ndarray, G: int) -> np.ndarray:
    """x[P, n] (uint16 bf16 bits or float32) -> out[P, n], finite inputs only."""
    P, n = x.shape
    dtype = "bf16" if x.dtype == np.uint16 else "f32"
    out = np.empty_like(x)
    for j in range(n):
        per_node = allreduce_element([x[p, j] for p in range(P)], G, dtype)
        for p in range(P):
            out[p, j] = per_node[p // G]
    return out
