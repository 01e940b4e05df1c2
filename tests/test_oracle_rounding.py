"""Pins of the oracle's rounding and requantisation (Section 3.2.1's requantisation
equation, Section 3.3's bound condition) against exact rational arithmetic."""
import math
import os
import random
from fractions import Fraction

import pytest

from oracle import oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))


def closed_form(v, mul, s):
    """floor(v * mul / 2^s + 1/2) with exact rationals (no rounding term when s == 0)."""
    x = Fraction(v * mul, 1 << s)
    return math.floor(x + Fraction(1, 2)) if s > 0 else int(x)


def test_hand_computed_table():
    n = 0
    for line in open(os.path.join(HERE, "golden", "requant_cases.txt")):
        line = line.split("#")[0].split()
        if not line:
            continue
        y, mul, s, want = map(int, line)
        assert O.requant(y, mul, s) == want, (y, mul, s)
        n += 1
    assert n >= 25


def test_rsr_exhaustive_small_grid():
    for s in range(0, 9):
        for v in range(-600, 601):
            assert O.rsr(v, s) == closed_form(v, 1, s), (v, s)


def test_requant_small_grid_against_rationals():
    for mul in (1, 2, 3, 5, 7, 127, 255, 1000, 16384, 32767):
        for s in (0, 1, 2, 3, 7, 8, 14, 15, 16):
            for v in list(range(-130, 131)) + [4095, 4096, 4097, -4095, -4096, -4097]:
                assert O.requant(v, mul, s) == closed_form(v, mul, s), (v, mul, s)


def test_requant_edges_and_random_wide():
    rnd = random.Random(7)
    i31 = (1 << 31) - 1
    cases = [(v, m, s) for v in (0, 1, -1, i31, -i31 - 1, i31 - 1)
             for m in (1, 2, i31, 1 << 30, 23124) for s in (0, 1, 31, 32, 46, 61, 62)]
    for _ in range(20000):
        s = rnd.randint(0, 62)
        cases.append((rnd.randint(-i31 - 1, i31), rnd.randint(1, i31), s))
    for v, m, s in cases:
        assert O.requant(v, m, s) == closed_form(v, m, s), (v, m, s)


def test_exact_ties_round_up_for_both_signs():
    for s in range(1, 40):
        half = 1 << (s - 1)
        for k in (-5, -1, 0, 1, 6):
            v = k * (1 << s) + half          # exactly k + 1/2
            assert O.rsr(v, s) == k + 1
            assert O.rsr(v - 1, s) == k      # just below the tie


def test_monotone_and_identity():
    for mul, s in ((23124, 26), (3, 1), (32767, 15), (1, 7)):
        prev = None
        for v in range(-3000, 3000, 7):
            q = O.requant(v * 1000, mul, s)
            assert prev is None or q >= prev
            prev = q
    for s in (0, 1, 5, 14, 30):
        for v in (-77, -1, 0, 1, 99, 123456):
            assert O.requant(v, 1 << s, s) == v


@pytest.mark.parametrize("mul,shift,max_int", [(23124, 26, 127), (5, 4, 127), (21116, 23, 127),
                                               (3, 3, 15), (32767, 20, 63), (16384, 14, 127)])
def test_brelu_then_quantise_equals_quantise_then_clamp(mul, shift, max_int):
    # Figure 1 orders the layer as BReLU (clamp Y to [0, h_i]) then quantisation; the
    # oracle quantises then clamps to max_int.  Section 3.3 requires h_i to quantise to
    # max_int; with that, both orders agree on every Y.
    h_i = None
    # smallest Y whose quantised value is max_int is a valid h_i; so is [max_int * 2^shift / mul]
    cand = closed_form(max_int << shift, 1, 0) // mul
    for h in range(max(0, cand - 3), cand + 4):
        if O.requant(h, mul, shift) == max_int:
            h_i = h
            break
    assert h_i is not None
    span = min(4 * h_i + 50, 400000)
    step = max(1, span // 50000)
    for y in list(range(-span, span, step)) + [h_i - 1, h_i, h_i + 1, 0, -1, 1]:
        brelu_first = O.requant(min(max(y, 0), h_i), mul, shift)
        clamp_last = min(max(O.requant(y, mul, shift), 0), max_int)
        assert brelu_first == clamp_last, y
