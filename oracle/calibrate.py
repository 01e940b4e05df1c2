"""Oracle-side calibration: turns accumulator statistics of a synthetic network
into the per-layer integers (mul, shift, bound) the integer layer needs.

TEST INFRASTRUCTURE, like the rest of oracle/.  Follows Section 3.3 (quantised
BReLU: h_ri -> mul, shift with [h_ri * mul / 2^shift] = max_int), Section 4.1
(ratio synchronisation at residual merges) and Algorithm 2 (concatenation).

Readings fixed here because the paper does not define them:
  * mul_shift(a, b) returns integers with mul / 2^shift ~ b / a: the smallest
    shift in [0, 46] whose rounded multiplier reaches 2^14 (so mul has 15
    significant bits); ratios of 2^15 and above use shift 0.
  * The statistic standing in for the n-sigma bound is the 99.9th percentile
    (nearest rank, at least 1) of all pre-clamp values of a layer on the
    calibration images.
  * A concatenated branch whose ratio is lowered to the common minimum can no
    longer reach max_int; its bound becomes min(max_int, [h_ri * mul / 2^shift]).
"""
import math
from fractions import Fraction

import numpy as np

from . import oracle as O

MAX_INT = 127
MAX_SHIFT = 46


def mul_shift(a, b):
    """Integers (mul, shift) with mul / 2^shift ~ b / a  (a, b positive rationals)."""
    ratio = Fraction(b) / Fraction(a)
    if ratio <= 0:
        raise ValueError("ratio must be positive")
    for s in range(0, MAX_SHIFT + 1):
        m = math.floor(ratio * (1 << s) + Fraction(1, 2))
        if m >= (1 << 14) or s == MAX_SHIFT:
            return max(1, min(m, (1 << 31) - 1)), s
    raise AssertionError


def bound_params(h_ri, max_int=MAX_INT):
    """(mul, shift) for a BReLU bound: [h_ri * mul / 2^shift] == max_int (Section 3.3)."""
    h_ri = max(1, int(h_ri))
    mul, s = mul_shift(h_ri, max_int)
    for _ in range(1 << 16):
        q = O.requant(h_ri, mul, s)
        if q == max_int:
            return mul, s
        mul += 1 if q < max_int else -1
        if mul < 1:
            break
    raise ArithmeticError("no multiplier maps %d to %d at shift %d" % (h_ri, max_int, s))


def percentile_999(values, absolute=False):
    """Nearest-rank 99.9th percentile of an integer array, at least 1."""
    v = np.asarray(values).reshape(-1)
    if absolute:
        v = np.abs(v.astype(np.int64))
    n = v.size
    k = max(0, math.ceil(0.999 * n) - 1)
    return max(1, int(np.partition(v, k)[k]))


def percentile_999_per_channel(values, absolute=False):
    """The same statistic for every channel (last axis) on its own."""
    v = np.asarray(values)
    return [percentile_999(v[..., c], absolute) for c in range(v.shape[-1])]


def sync_concat(h_ri, ratio_y, max_int=MAX_INT):
    """Algorithm 2 for N branches given each branch's bound h_ri[i] (integer, in its
    own Y domain) and ratio_Y[i].  Returns per-branch (mul, shift, bound_q) and the
    common output ratio."""
    own = [bound_params(h, max_int) for h in h_ri]
    ratio_v = [Fraction(ry) * m / (1 << s) for ry, (m, s) in zip(ratio_y, own)]
    ratio_min = min(ratio_v)
    out = []
    for h, ry in zip(h_ri, ratio_y):
        m, s = mul_shift(Fraction(ry), ratio_min)
        bq = min(max_int, O.requant(max(1, int(h)), m, s))
        out.append((m, s, max(1, bq)))
    return out, ratio_min
