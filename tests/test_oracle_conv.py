"""Pins of the oracle's integer convolution layer (Section 3.1 / Figure 1: U = X conv W,
Y = U + b; Section 3.4.1: re-normalisation) against things that are not the oracle:
a seven-loop brute force, a float64 library convolution (exact on these integers),
an int64 matrix product, shifted-copy and box-sum kernels, linearity."""
import numpy as np
import pytest
import torch

from oracle import oracle as O


def rnd(seed):
    return np.random.default_rng(seed)


def brute_force_u(x, w, stride, pad, sub128=False):
    """U[n,ho,wo,co] by seven nested loops over python ints."""
    n_, h, w_, c = x.shape
    co_, kh_, kw_, _ = w.shape
    ho_ = (h + 2 * pad - kh_) // stride + 1
    wo_ = (w_ + 2 * pad - kw_) // stride + 1
    out = np.zeros((n_, ho_, wo_, co_), dtype=np.int64)
    for n in range(n_):
        for ho in range(ho_):
            for wo in range(wo_):
                for co in range(co_):
                    acc = 0
                    for kh in range(kh_):
                        for kw in range(kw_):
                            hi = ho * stride - pad + kh
                            wi = wo * stride - pad + kw
                            if not (0 <= hi < h and 0 <= wi < w_):
                                continue
                            for ci in range(c):
                                xv = int(x[n, hi, wi, ci]) - (128 if sub128 else 0)
                                acc += xv * int(w[co, kh, kw, ci])
                    out[n, ho, wo, co] = acc
    return out


def library_u(x, w, stride, pad, sub128=False):
    """Same U through torch.nn.functional.conv2d in float64 (exact below 2^53)."""
    xf = torch.from_numpy(x.astype(np.float64))
    if sub128:
        xf = xf - 128.0
    xf = xf.permute(0, 3, 1, 2)
    wf = torch.from_numpy(w.astype(np.float64)).permute(0, 3, 1, 2)
    y = torch.nn.functional.conv2d(xf, wf, stride=stride, padding=pad)
    return y.permute(0, 2, 3, 1).numpy().astype(np.int64)


def oracle_u(x, w, stride, pad, sub128=False, bias=None):
    b = np.zeros(w.shape[0], np.int32) if bias is None else bias
    return O.conv2d(x, w, b, stride=stride, pad=pad, in_sub128=sub128,
                    out_mode="raw_s32").astype(np.int64)


GEOMS = [  # (k, stride, pad) used by the five workloads, on odd sizes
    (3, 1, 1), (5, 1, 2), (1, 1, 0), (7, 2, 3), (3, 2, 1), (1, 2, 0)]


@pytest.mark.parametrize("k,stride,pad", GEOMS)
def test_matches_seven_loop_brute_force(k, stride, pad):
    g = rnd(k * 100 + stride)
    x = g.integers(0, 128, size=(2, 7, 9, 3), dtype=np.uint8)
    w = g.integers(-127, 128, size=(4, k, k, 3), dtype=np.int8)
    assert (oracle_u(x, w, stride, pad) == brute_force_u(x, w, stride, pad)).all()


@pytest.mark.parametrize("k,stride,pad", GEOMS)
def test_matches_float64_library_convolution(k, stride, pad):
    g = rnd(k * 7 + stride + 50)
    x = g.integers(0, 128, size=(2, 13, 11, 16), dtype=np.uint8)
    w = g.integers(-127, 128, size=(8, k, k, 16), dtype=np.int8)
    assert (oracle_u(x, w, stride, pad) == library_u(x, w, stride, pad)).all()


def test_renormalised_input_pads_with_zero_after_subtracting_128():
    # raw uint8 picture: the layer sees raw - 128 inside the image and 0 outside it
    g = rnd(11)
    x = g.integers(0, 256, size=(1, 6, 5, 1), dtype=np.uint8)
    w = g.integers(-127, 128, size=(3, 3, 3, 1), dtype=np.int8)
    got = oracle_u(x, w, 1, 1, sub128=True)
    assert (got == brute_force_u(x, w, 1, 1, sub128=True)).all()
    assert (got == library_u(x, w, 1, 1, sub128=True)).all()
    # padding with raw zeros (i.e. -128 after the shift) would differ at the border
    xp = np.zeros((1, 8, 7, 1), np.uint8)
    xp[:, 1:-1, 1:-1] = x
    wrong = library_u(xp, w, 1, 0, sub128=True)
    assert (wrong[:, 1:-1, 1:-1] == got[:, 1:-1, 1:-1]).all() and (wrong != got).any()


def test_signed_int8_input():
    g = rnd(12)
    x = g.integers(-128, 128, size=(1, 5, 6, 4), dtype=np.int8)
    w = g.integers(-127, 128, size=(5, 3, 3, 4), dtype=np.int8)
    assert (oracle_u(x, w, 1, 1) == library_u(x, w, 1, 1)).all()


def test_pointwise_conv_is_an_integer_matrix_product():
    g = rnd(13)
    x = g.integers(0, 128, size=(3, 5, 7, 32), dtype=np.uint8)
    w = g.integers(-127, 128, size=(24, 1, 1, 32), dtype=np.int8)
    want = x.reshape(-1, 32).astype(np.int64) @ w.reshape(24, 32).astype(np.int64).T
    assert (oracle_u(x, w, 1, 0).reshape(-1, 24) == want).all()


def test_delta_kernels_are_shifted_copies():
    g = rnd(14)
    x = g.integers(0, 128, size=(1, 8, 9, 2), dtype=np.uint8)
    for kh in range(3):
        for kw in range(3):
            w = np.zeros((2, 3, 3, 2), np.int8)
            w[0, kh, kw, 0] = 1
            w[1, kh, kw, 1] = 1
            xp = np.zeros((1, 10, 11, 2), np.int64)
            xp[:, 1:-1, 1:-1] = x
            want = xp[:, kh:kh + 8, kw:kw + 9, :]
            assert (oracle_u(x, w, 1, 1) == want).all(), (kh, kw)


def test_all_ones_kernel_is_a_box_sum_with_stride():
    g = rnd(15)
    x = g.integers(0, 128, size=(1, 9, 9, 1), dtype=np.uint8)
    w = np.ones((1, 3, 3, 1), np.int8)
    xp = np.zeros((11, 11), np.int64)
    xp[1:-1, 1:-1] = x[0, :, :, 0]
    got = oracle_u(x, w, 2, 1)[0, :, :, 0]
    for ho in range(5):
        for wo in range(5):
            assert got[ho, wo] == xp[2 * ho:2 * ho + 3, 2 * wo:2 * wo + 3].sum()


def test_linear_in_the_weights_and_bias_is_added():
    g = rnd(16)
    x = g.integers(0, 128, size=(1, 6, 6, 8), dtype=np.uint8)
    w1 = g.integers(-60, 60, size=(4, 3, 3, 8), dtype=np.int8)
    w2 = g.integers(-60, 60, size=(4, 3, 3, 8), dtype=np.int8)
    b = g.integers(-4096, 4097, size=4).astype(np.int32)
    lhs = oracle_u(x, (w1 + w2).astype(np.int8), 1, 1)
    assert (lhs == oracle_u(x, w1, 1, 1) + oracle_u(x, w2, 1, 1)).all()
    assert (oracle_u(x, w1, 1, 1, bias=b) == oracle_u(x, w1, 1, 1) + b).all()


def test_channel_slice_input_and_channel_offset_output():
    g = rnd(17)
    xb = g.integers(0, 128, size=(1, 5, 5, 12), dtype=np.uint8)     # read only 8 of 12 channels
    w = g.integers(-127, 128, size=(3, 3, 3, 8), dtype=np.int8)
    b = np.zeros(3, np.int32)
    a = O.conv2d(xb, w, b, stride=1, pad=1, cin=8, out_mode="raw_s32")
    assert (a == library_u(np.ascontiguousarray(xb[..., :8]), w, 1, 1)).all()
    out = np.full((1, 5, 5, 7), 99, np.uint8)
    O.conv2d(xb, w, b, stride=1, pad=1, cin=8, mul=1, shift=8, bound_q=127, out=out, out_c_offset=2)
    assert (out[..., :2] == 99).all() and (out[..., 5:] == 99).all()
    want = np.clip((a.astype(np.int64) + 128) >> 8, 0, 127)
    assert (out[..., 2:5] == want).all()


def test_full_layer_epilogue_and_invariants():
    g = rnd(18)
    x = g.integers(0, 128, size=(2, 9, 8, 16), dtype=np.uint8)
    w = g.integers(-127, 128, size=(6, 3, 3, 16), dtype=np.int8)
    b = g.integers(-4096, 4097, size=6).astype(np.int32)
    y = library_u(x, w, 1, 1) + b
    mul, shift, bq = 29000, 24, 127
    v = O.conv2d(x, w, b, stride=1, pad=1, mul=mul, shift=shift, bound_q=bq)
    want = np.clip((y * mul + (1 << (shift - 1))) >> shift, 0, bq)
    assert v.dtype == np.uint8 and v.min() >= 0 and v.max() <= bq
    assert (v == want).all() and (v == 0).any() and (v == bq).any()


def test_residual_merge_before_and_after_requantisation():
    g = rnd(19)
    x = g.integers(0, 128, size=(1, 6, 7, 8), dtype=np.uint8)
    w = g.integers(-127, 128, size=(5, 1, 1, 8), dtype=np.int8)
    b = g.integers(-4096, 4097, size=5).astype(np.int32)
    y = library_u(x, w, 1, 0) + b
    r8 = g.integers(0, 128, size=(1, 6, 7, 5), dtype=np.uint8)
    r32 = g.integers(-200000, 200000, size=(1, 6, 7, 5)).astype(np.int32)
    for r, rm, rs in ((r8, 18415, 5), (r32, 20000, 15), (r32, 3, 0)):
        skip = (r.astype(np.int64) * rm + ((1 << (rs - 1)) if rs else 0)) >> rs
        t = O.conv2d(x, w, b, res=r, res_mode="pre", res_mul=rm, res_shift=rs, out_mode="raw_s32")
        assert (t == y + skip).all()
        v = O.conv2d(x, w, b, res=r, res_mode="pre", res_mul=rm, res_shift=rs, mul=20000, shift=24)
        assert (v == np.clip(((y + skip) * 20000 + (1 << 23)) >> 24, 0, 127)).all()
    # regression output: requantise, add the raw picture, clamp to [0, 255]
    raw = g.integers(0, 256, size=(1, 6, 7, 5), dtype=np.uint8)
    v = O.conv2d(x, w, b, res=raw, res_mode="post", res_mul=1, res_shift=0, mul=20050, shift=22,
                 out_mode="clamp_u8", lo=0, hi=255)
    want = np.clip(((y * 20050 + (1 << 21)) >> 22) + raw, 0, 255)
    assert (v == want).all() and (v == 0).any() and (v == 255).any()


def test_accumulator_overflow_is_reported():
    x = np.full((1, 1, 1, 70000), 255, np.uint8).view(np.int8).view(np.uint8)
    w = np.full((1, 1, 1, 70000), 127, np.int8)
    with pytest.raises(ArithmeticError):
        O.conv2d(x, w, np.zeros(1, np.int32), out_mode="raw_s32")      # 255*127*70000 > 2^31


def test_per_channel_requantisation_is_the_per_layer_one_channel_by_channel():
    """Section 3.4.3 (one weight step per output channel): every channel carries its own
    (mul, shift) and skip rescale.  Pinned three ways: numpy arithmetic on the library U,
    the per-layer oracle run once per channel, and constant arrays == per-layer call."""
    g = rnd(23)
    x = g.integers(0, 128, size=(2, 7, 6, 12), dtype=np.uint8)
    w = g.integers(-127, 128, size=(9, 3, 3, 12), dtype=np.int8)
    b = g.integers(-4096, 4097, size=9).astype(np.int32)
    mul_c = g.integers(1 << 14, 1 << 15, size=9).astype(np.int32)
    shift_c = g.integers(20, 27, size=9).astype(np.int32)
    shift_c[0], mul_c[0] = 0, 1                       # a shift of zero adds no rounding term
    rmul_c = g.integers(1, 1 << 15, size=9).astype(np.int32)
    rshift_c = g.integers(0, 9, size=9).astype(np.int32)
    r8 = g.integers(0, 128, size=(2, 7, 6, 9), dtype=np.uint8)
    y = library_u(x, w, 1, 1) + b
    half = np.where(shift_c > 0, (1 << np.maximum(shift_c - 1, 0)), 0).astype(np.int64)
    rhalf = np.where(rshift_c > 0, (1 << np.maximum(rshift_c - 1, 0)), 0).astype(np.int64)
    skip = (r8.astype(np.int64) * rmul_c + rhalf) >> rshift_c
    # no skip operand
    v = O.conv2d(x, w, b, stride=1, pad=1, mul_c=mul_c, shift_c=shift_c)
    assert (v == np.clip((y * mul_c + half) >> shift_c, 0, 127)).all()
    # skip operand joined before and after requantisation
    v_pre = O.conv2d(x, w, b, stride=1, pad=1, mul_c=mul_c, shift_c=shift_c, res=r8, res_mode="pre",
                     res_mul_c=rmul_c, res_shift_c=rshift_c)
    assert (v_pre == np.clip(((y + skip) * mul_c + half) >> shift_c, 0, 127)).all()
    v_post = O.conv2d(x, w, b, stride=1, pad=1, mul_c=mul_c, shift_c=shift_c, res=r8, res_mode="post",
                      res_mul_c=rmul_c, res_shift_c=rshift_c, out_mode="clamp_u8", lo=3, hi=250)
    assert (v_post == np.clip(((y * mul_c + half) >> shift_c) + skip, 3, 250)).all()
    # the per-layer function, one output channel at a time
    for co in range(9):
        one = O.conv2d(x, w[co:co + 1], b[co:co + 1], stride=1, pad=1, mul=int(mul_c[co]), shift=int(shift_c[co]),
                       res=np.ascontiguousarray(r8[..., co:co + 1]), res_mode="pre",
                       res_mul=int(rmul_c[co]), res_shift=int(rshift_c[co]))
        assert (one[..., 0] == v_pre[..., co]).all()
    # constant arrays are the per-layer call; a missing array falls back to the per-layer value
    same = O.conv2d(x, w, b, stride=1, pad=1, mul_c=np.full(9, 23000, np.int32), shift_c=np.full(9, 24, np.int32))
    assert (same == O.conv2d(x, w, b, stride=1, pad=1, mul=23000, shift=24)).all()
    mixed = O.conv2d(x, w, b, stride=1, pad=1, mul_c=mul_c, shift=22, res=r8, res_mode="pre", res_mul=77,
                     res_shift_c=rshift_c)
    skip2 = (r8.astype(np.int64) * 77 + rhalf) >> rshift_c
    assert (mixed == np.clip(((y + skip2) * mul_c + (1 << 21)) >> 22, 0, 127)).all()
