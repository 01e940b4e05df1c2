"""Pins of the oracle's rescaled addition (Sections 3.4.2, 4.1), concatenation
(Algorithm 2) and pooling against identities and library routines."""
from fractions import Fraction
import math

import numpy as np
import torch

from oracle import oracle as O


def rnd(seed):
    return np.random.default_rng(seed)


def test_add_with_zero_operand_is_plain_requantisation():
    g = rnd(1)
    a = g.integers(-300000, 300000, size=(3, 5, 8)).astype(np.int32)
    z = np.zeros_like(a)
    got = O.add_rescale(a, z, b_mul=12345, b_shift=3, mul=23124, shift=26, lo=0, hi=127)
    want = np.clip((a.astype(np.int64) * 23124 + (1 << 25)) >> 26, 0, 127)
    assert (got == want).all()


def test_add_with_unit_rescale_is_exact_integer_addition():
    g = rnd(2)
    a = g.integers(0, 128, size=(4, 4, 16), dtype=np.uint8)
    b = g.integers(0, 128, size=(4, 4, 16), dtype=np.uint8)
    for s in (0, 4, 11):
        got = O.add_rescale(a, b, b_mul=1 << s, b_shift=s, mul=1, shift=0, lo=0, hi=255)
        assert (got == a.astype(np.int64) + b).all()
    raw = O.add_rescale(a, b, out_mode="raw_s32")
    assert raw.dtype == np.int32 and (raw == a.astype(np.int64) + b).all()


def test_add_general_case_against_rationals_and_saturation():
    g = rnd(3)
    a = g.integers(-2**31, 2**31, size=(2, 3, 4)).astype(np.int32)
    b = g.integers(-2**31, 2**31, size=(2, 3, 4)).astype(np.int32)
    bm, bs, m, s = 3, 1, 5, 33
    got = O.add_rescale(a, b, b_mul=bm, b_shift=bs, mul=m, shift=s, out_mode="linear_s8")
    for av, bv, q in zip(a.reshape(-1), b.reshape(-1), got.reshape(-1)):
        skip = math.floor(Fraction(int(bv) * bm, 1 << bs) + Fraction(1, 2))
        t = min(max(int(av) + skip, -2**31), 2**31 - 1)
        want = min(max(math.floor(Fraction(t * m, 1 << s) + Fraction(1, 2)), -128), 127)
        assert int(q) == want


def test_add_mixed_types_matches_conv_merge_arithmetic():
    g = rnd(4)
    y = g.integers(-200000, 200000, size=(1, 4, 4, 8)).astype(np.int32)
    r = g.integers(0, 128, size=(1, 4, 4, 8), dtype=np.uint8)
    got = O.add_rescale(y, r, b_mul=18415, b_shift=5, mul=23187, shift=24, lo=0, hi=127)
    t = y.astype(np.int64) + ((r.astype(np.int64) * 18415 + 16) >> 5)
    assert (got == np.clip((t * 23187 + (1 << 23)) >> 24, 0, 127)).all()


def test_concat_identity_scale_is_numpy_concatenate():
    g = rnd(5)
    xs = [g.integers(0, 128, size=(2, 3, 3, c), dtype=np.uint8) for c in (32, 16, 5)]
    got = O.concat(xs, [1, 1, 1], [0, 0, 0], 127)
    assert (got == np.concatenate(xs, axis=-1)).all()


def test_concat_per_branch_rescale_and_bound():
    g = rnd(6)
    xs = [g.integers(0, 128, size=(7, c), dtype=np.uint8) for c in (4, 6)]
    got = O.concat(xs, [3, 20000], [1, 14], 100)
    w0 = np.clip((xs[0].astype(np.int64) * 3 + 1) >> 1, 0, 100)
    w1 = np.clip((xs[1].astype(np.int64) * 20000 + (1 << 13)) >> 14, 0, 100)
    assert (got[:, :4] == w0).all() and (got[:, 4:] == w1).all() and got.max() == 100


def test_zero_copy_concat_equals_explicit_concat():
    # two conv branches writing channel slices of one buffer == concatenating their outputs
    g = rnd(7)
    x = g.integers(0, 128, size=(1, 6, 6, 16), dtype=np.uint8)
    wa = g.integers(-127, 128, size=(8, 5, 5, 16), dtype=np.int8)
    wb = g.integers(-127, 128, size=(4, 3, 3, 16), dtype=np.int8)
    ba = np.zeros(8, np.int32)
    bb = np.ones(4, np.int32)
    pa = dict(mul=30000, shift=27, bound_q=127)
    pb = dict(mul=18000, shift=27, bound_q=24)
    buf = np.full((1, 6, 6, 12), 255, np.uint8)
    O.conv2d(x, wa, ba, stride=1, pad=2, out=buf, out_c_offset=0, **pa)
    assert (buf[..., 8:] == 255).all()                     # the other slice is untouched
    O.conv2d(x, wb, bb, stride=1, pad=1, out=buf, out_c_offset=8, **pb)
    sep = [O.conv2d(x, wa, ba, stride=1, pad=2, **pa), O.conv2d(x, wb, bb, stride=1, pad=1, **pb)]
    assert (buf == np.concatenate(sep, axis=-1)).all()
    assert (buf == O.concat(sep, [1, 1], [0, 0], 127)).all()


def test_maxpool_matches_library():
    g = rnd(8)
    for (h, w, k, s, p) in ((12, 12, 3, 2, 1), (7, 9, 3, 2, 1), (8, 8, 2, 2, 0)):
        x = g.integers(0, 128, size=(2, h, w, 5), dtype=np.uint8)
        xf = torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2)
        want = torch.nn.functional.max_pool2d(xf, k, s, p).permute(0, 2, 3, 1).numpy()
        assert (O.maxpool2d(x, k, s, p) == want).all()


def test_global_average_against_rationals():
    g = rnd(9)
    x = g.integers(0, 128, size=(3, 7, 7, 6), dtype=np.uint8)
    mul, shift = 21400, 20                       # ~ 1/49
    got = O.avgpool_global(x, mul, shift, 127)
    sums = x.astype(np.int64).sum(axis=(1, 2))
    for s_, q in zip(sums.reshape(-1), got.reshape(-1)):
        want = min(127, math.floor(Fraction(int(s_) * mul, 1 << shift) + Fraction(1, 2)))
        assert int(q) == want
    assert np.abs(got.reshape(3, 6).astype(float) - sums / 49.0).max() <= 0.51


def test_renormalise_is_minus_128_on_every_byte():
    # Section 3.4.1: all 256 byte values against the closed form; as bytes it is a flip of the top bit; and a
    # layer that re-normalises on the fly equals the same layer on the re-normalised picture
    x = np.arange(256, dtype=np.uint8)
    got = O.renormalize(x)
    assert got.dtype == np.int8 and [int(v) for v in got] == [v - 128 for v in range(256)]
    assert (got.view(np.uint8) == (x ^ 0x80)).all()
    g = rnd(10)
    raw = g.integers(0, 256, size=(1, 7, 9, 3), dtype=np.uint8)
    w = g.integers(-127, 128, size=(5, 3, 3, 3), dtype=np.int8)
    b = g.integers(-50, 50, size=5).astype(np.int32)
    fly = O.conv2d(raw, w, b, stride=1, pad=1, in_sub128=True, out_mode="raw_s32")
    pre = O.conv2d(O.renormalize(raw), w, b, stride=1, pad=1, out_mode="raw_s32")
    assert (fly == pre).all()
