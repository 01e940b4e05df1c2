"""GPU parity of the fused identity bottleneck block (iconv2d_bottleneck_brelu) against the oracle's three
separate layers, bit for bit: the two middle tensors never exist on the GPU, so the block's output is compared
(the oracle computes the middle tensors itself)."""
import numpy as np
import pytest
import torch

from oracle import calibrate as K
from oracle import oracle as O

pytestmark = pytest.mark.gpu


def rnd(seed):
    return np.random.default_rng(seed)


def run_block(seed, n, h, w, c, mid, *, skip="x", c3_mode="brelu", forms=("auto", "auto"), bound12=127, cbuf=None):
    """Returns (gpu output, oracle output).  forms: how the first two layers requantise: "auto" = calibrated
    15-bit multiplier (the 32-bit form), "hi" = a pair only the one-multiply form takes, "wide" = only the general form."""
    from gpu_util import dev
    from paper_2006_11735_amd import binding as B
    g = rnd(seed)
    cbuf = c if cbuf is None else cbuf
    x = g.integers(0, 128, size=(n, h, w, cbuf), dtype=np.uint8)
    w1 = g.integers(-127, 128, size=(mid, 1, 1, c), dtype=np.int8)
    w2 = g.integers(-127, 128, size=(mid, 3, 3, mid), dtype=np.int8)
    w3 = g.integers(-127, 128, size=(c, 1, 1, mid), dtype=np.int8)
    b1, b2, b3 = (g.integers(-4096, 4097, size=k).astype(np.int32) for k in (mid, mid, c))

    def pair(raw, form, bound):
        m, s = K.bound_params(K.percentile_999(raw), bound)
        if form == "hi":            # same ratio, multiplier of 29 bits: too wide for 24-bit factors, fine as a high-word multiply
            return m << 14, s + 14
        if form == "wide":          # shift beyond 32: general 64-bit form
            return m << 16, s + 16 if s + 16 > 32 else 33
        return m, s
    t1_raw = O.conv2d(x, w1, b1, cin=c, out_mode="raw_s32")
    m1, s1 = pair(t1_raw, forms[0], bound12)
    t1 = O.conv2d(x, w1, b1, cin=c, mul=m1, shift=s1, bound_q=bound12)
    t2_raw = O.conv2d(t1, w2, b2, pad=1, out_mode="raw_s32")
    m2, s2 = pair(t2_raw, forms[1], bound12)
    t2 = O.conv2d(t1, w2, b2, pad=1, mul=m2, shift=s2, bound_q=bound12)
    kw3 = {}
    res = None
    if skip == "x":
        res = np.ascontiguousarray(x[..., :c])
    elif skip == "s32":
        res = g.integers(-300000, 300000, size=(n, h, w, c)).astype(np.int32)
    if res is not None:
        y_main = O.conv2d(t2, w3, b3, out_mode="raw_s32")
        rm, rs = K.mul_shift(127 if skip == "x" else 300000, K.percentile_999(y_main))
        kw3.update(res=res, res_mode="pre", res_mul=rm, res_shift=rs)
    t3_raw = O.conv2d(t2, w3, b3, out_mode="raw_s32", **kw3)
    m3, s3 = K.bound_params(K.percentile_999(t3_raw), 127)
    if c3_mode == "raw_s32":
        want = t3_raw
    elif c3_mode == "linear_s8":
        want = O.conv2d(t2, w3, b3, mul=m3, shift=s3, out_mode="linear_s8", **kw3)
    else:
        want = O.conv2d(t2, w3, b3, mul=m3, shift=s3, bound_q=127, **kw3)

    om = {"brelu": B.ICNN_OUT_BRELU_U8, "raw_s32": B.ICNN_OUT_RAW_S32, "linear_s8": B.ICNN_OUT_LINEAR_S8}[c3_mode]
    d1 = B.conv_desc(n=n, h=h, w=w, cin=c, in_c_stride=cbuf, cout=mid, kh=1, kw=1, out_c_stride=mid, mul=m1, shift=s1, bound_q=bound12)
    d2 = B.conv_desc(n=n, h=h, w=w, cin=mid, in_c_stride=mid, cout=mid, kh=3, kw=3, pad_h=1, pad_w=1, out_c_stride=mid, mul=m2,
                     shift=s2, bound_q=bound12)
    d3 = B.conv_desc(n=n, h=h, w=w, cin=mid, in_c_stride=mid, cout=c, kh=1, kw=1, out_c_stride=c, mul=m3, shift=s3, bound_q=127,
                     out_mode=om)
    if res is not None:
        d3.res_mode, d3.res_c_stride = B.ICNN_RES_PRE, c
        d3.res_dtype = B.ICNN_U8 if res.dtype == np.uint8 else B.ICNN_S32
        d3.res_mul, d3.res_shift = rm, rs
    packs = []
    for d, wt in ((d1, w1), (d2, w2), (d3, w3)):
        pk = torch.zeros(B.iconv2d_packed_weight_bytes(d), dtype=torch.uint8, device="cuda:0")
        B.iconv2d_prepack_weights(d, dev(wt), pk)
        packs.append(pk)
    tdt = {np.dtype(np.uint8): torch.uint8, np.dtype(np.int8): torch.int8, np.dtype(np.int32): torch.int32}[want.dtype]
    y = torch.zeros(want.shape, dtype=tdt, device="cuda:0")
    xd = dev(x)
    rd = None if res is None else (dev(res) if (skip != "x" or cbuf != c) else xd)
    B.iconv2d_bottleneck_brelu(d1, xd, packs[0], dev(b1), d2, packs[1], dev(b2), d3, packs[2], dev(b3), rd, y)
    torch.cuda.synchronize()
    return y.cpu().numpy(), want


BLOCKS = [
    # n, h, w, c, mid
    (2, 56, 56, 256, 64),        # stage-1 shape: 28 tiles per image, two workgroups per compute unit
    (3, 28, 28, 512, 128),       # stage-2 shape
    (1, 17, 23, 128, 64),        # ragged tiles on both axes
    (2, 9, 30, 256, 128),
    (1, 5, 6, 64, 64),           # image smaller than a tile
    (5, 14, 14, 192, 64),        # three channel chunks in the last layer, three K steps in the first
    (40, 14, 14, 256, 128),      # more tiles than resident workgroups: every workgroup walks several
    (1, 1, 200, 128, 128),       # one image row
    (1, 150, 1, 64, 64),         # one image column
    (12, 56, 56, 256, 64),       # 336 tiles: more than resident workgroups, both patch buffers in turn
    (3, 30, 41, 128, 64),        # ragged tiles, two slices
]


@pytest.mark.parametrize("ring", [False, True], ids=["default", "lds_ring"])
@pytest.mark.parametrize("shape", BLOCKS, ids=lambda s: "x".join(map(str, s)))
def test_fused_block_equals_three_layers(shape, ring):
    # blocks with 64 middle channels and 64 / 128 / 256 outer ones take the kernel that keeps the weights in registers;
    # ring=True keeps them on the kernel that streams the weights through LDS, like the other shapes
    from paper_2006_11735_amd import binding as B
    n, h, w, c, mid = shape
    if ring and mid != 64:
        pytest.skip("only one kernel takes this shape")
    B.icnn_set_tuning("no_block64", 1 if ring else 0)
    try:
        got, want = run_block(sum(shape), n, h, w, c, mid)
    finally:
        B.icnn_set_tuning("no_block64", 0)
    assert got.shape == want.shape
    assert (got == want).all(), "%d of %d bytes differ" % (int((got != want).sum()), want.size)
    assert want.max() == 127 and want.min() == 0


@pytest.mark.parametrize("mid,c", [(64, 128), (128, 512)])
def test_fused_block_on_the_instantiation_that_holds_every_epilogue_form(mid, c):
    # calibrated layers take the instantiation with the one 32-bit form; the other one must agree on them too
    from paper_2006_11735_amd import binding as B
    B.icnn_set_tuning("no_block64", 1)
    B.icnn_set_tuning("block_any_form", 1)
    try:
        for kw in (dict(), dict(skip=None)):
            got, want = run_block(11 + mid, 3, 14, 14, c, mid, **kw)
            assert (got == want).all(), kw
    finally:
        B.icnn_set_tuning("reset")


@pytest.mark.parametrize("mid,c", [(64, 128), (128, 256)])
def test_fused_block_output_and_skip_modes(mid, c):
    for kw in (dict(skip=None), dict(skip="s32"), dict(c3_mode="raw_s32"), dict(c3_mode="linear_s8", skip=None),
               dict(forms=("hi", "wide")), dict(forms=("wide", "hi")), dict(bound12=15), dict(cbuf=c + 64)):
        got, want = run_block(7 + mid, 2, 11, 13, c, mid, **kw)
        assert (got == want).all(), kw


def test_fused_block_refuses_other_shapes():
    from paper_2006_11735_amd import binding as B

    def descs(**over):
        base = dict(n=1, h=8, w=8, c=128, mid=64, stride=1, k2=3)
        base.update(over)
        c, mid = base["c"], base["mid"]
        d1 = B.conv_desc(n=1, h=8, w=8, cin=c, in_c_stride=c, cout=mid, kh=1, kw=1, out_c_stride=mid, mul=20000, shift=24)
        d2 = B.conv_desc(n=1, h=8, w=8, cin=mid, in_c_stride=mid, cout=mid, kh=base["k2"], kw=base["k2"], pad_h=base["k2"] // 2,
                         pad_w=base["k2"] // 2, stride_h=base["stride"], stride_w=base["stride"], out_c_stride=mid, mul=20000, shift=24)
        d3 = B.conv_desc(n=1, h=8, w=8, cin=mid, in_c_stride=mid, cout=c, kh=1, kw=1, out_c_stride=c, mul=20000, shift=24)
        return d1, d2, d3
    for over in (dict(mid=32), dict(mid=256, c=256), dict(stride=2), dict(k2=5), dict(c=96)):
        d1, d2, d3 = descs(**over)
        with pytest.raises(B.IcnnError) as e:
            B.iconv2d_bottleneck_brelu(d1, 4096, 8192, 12288, d2, 16384, 20480, d3, 24576, 28672, None, 32768, stream=0)
        assert e.value.code in (B.ICNN_E_UNSUPPORTED, B.ICNN_E_SHAPE), over


# ---- first layer + max-pool as one launch
STEMS = [
    # n, h, w, cin, cout, k, pad
    (2, 224, 224, 3, 64, 7, 3),      # the ResNet stem
    (3, 37, 41, 3, 64, 7, 3),        # ragged pooled tiles, odd sizes
    (1, 64, 64, 1, 32, 5, 2),        # one channel, 5x5, 32 output channels
    (2, 19, 150, 4, 64, 8, 3),       # four channels, even kernel
    (1, 7, 9, 3, 64, 7, 3),          # picture smaller than a tile
    (70, 32, 32, 3, 64, 7, 3),       # more tiles than resident workgroups
]


@pytest.mark.parametrize("shape", STEMS, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("raw", [True, False])
def test_first_layer_with_pool_equals_the_two_calls(shape, raw):
    from gpu_util import dev
    from paper_2006_11735_amd import binding as B
    n, h, w, cin, cout, k, pad = shape
    g = rnd(sum(shape) + raw)
    x = g.integers(0, 256 if raw else 128, size=(n, h, w, cin), dtype=np.uint8)
    wt = g.integers(-127, 128, size=(cout, k, k, cin), dtype=np.int8)
    b = g.integers(-4096, 4097, size=cout).astype(np.int32)
    t_raw = O.conv2d(x, wt, b, stride=2, pad=pad, in_sub128=raw, out_mode="raw_s32")
    mul, shift = K.bound_params(K.percentile_999(t_raw))
    t = O.conv2d(x, wt, b, stride=2, pad=pad, in_sub128=raw, mul=mul, shift=shift, bound_q=127)
    want = O.maxpool2d(t, 3, 2, 1)
    d = B.conv_desc(n=n, h=h, w=w, cin=cin, in_c_stride=cin, in_sub128=int(raw), cout=cout, kh=k, kw=k, stride_h=2, stride_w=2,
                    pad_h=pad, pad_w=pad, out_c_stride=cout + 16, out_c_offset=16, mul=mul, shift=shift, bound_q=127)
    wp = torch.zeros(B.iconv2d_packed_weight_bytes(d), dtype=torch.uint8, device="cuda:0")
    B.iconv2d_prepack_weights(d, dev(wt), wp)
    y = torch.full((n,) + want.shape[1:3] + (cout + 16,), 99, dtype=torch.uint8, device="cuda:0")
    B.iconv2d_maxpool_brelu(d, 3, 2, 1, dev(x), wp, dev(b), y)
    torch.cuda.synchronize()
    got = y.cpu().numpy()
    assert (got[..., 16:] == want).all(), "%d of %d bytes differ" % (int((got[..., 16:] != want).sum()), want.size)
    assert (got[..., :16] == 99).all() and want.max() == 127


@pytest.mark.parametrize("cin,pitch", [(3, 4), (3, 7), (1, 2), (2, 2)])
def test_first_layer_with_pool_picture_pitch_wider_than_cin(cin, pitch):
    # pictures whose pixels are `pitch` bytes apart (e.g. RGB in RGBA storage): the kernel reads four bytes per pixel
    # and keeps cin of them; the tensor's last pixels are read early and shifted
    from gpu_util import dev
    from paper_2006_11735_amd import binding as B
    n, h, w, cout, k, pad = 2, 21, 26, 64, 7, 3
    g = rnd(100 * cin + pitch)
    xbuf = g.integers(0, 256, size=(n, h, w, pitch), dtype=np.uint8)
    wt = g.integers(-127, 128, size=(cout, k, k, cin), dtype=np.int8)
    b = g.integers(-4096, 4097, size=cout).astype(np.int32)
    x = np.ascontiguousarray(xbuf[..., :cin])
    t_raw = O.conv2d(x, wt, b, stride=2, pad=pad, in_sub128=True, out_mode="raw_s32")
    mul, shift = K.bound_params(K.percentile_999(t_raw))
    want = O.maxpool2d(O.conv2d(x, wt, b, stride=2, pad=pad, in_sub128=True, mul=mul, shift=shift, bound_q=127), 3, 2, 1)
    d = B.conv_desc(n=n, h=h, w=w, cin=cin, in_c_stride=pitch, in_sub128=1, cout=cout, kh=k, kw=k, stride_h=2, stride_w=2,
                    pad_h=pad, pad_w=pad, out_c_stride=cout, mul=mul, shift=shift, bound_q=127)
    wp = torch.zeros(B.iconv2d_packed_weight_bytes(d), dtype=torch.uint8, device="cuda:0")
    B.iconv2d_prepack_weights(d, dev(wt), wp)
    # the device buffer ends with the last pixel's cin bytes: nothing behind it may be touched
    flat = torch.from_numpy(xbuf.reshape(-1)[: xbuf.size - (pitch - cin)].copy()).to("cuda:0")
    y = torch.zeros(want.shape, dtype=torch.uint8, device="cuda:0")
    B.iconv2d_maxpool_brelu(d, 3, 2, 1, flat, wp, dev(b), y)
    torch.cuda.synchronize()
    assert (y.cpu().numpy() == want).all()


def test_first_layer_with_pool_refuses_other_shapes():
    from paper_2006_11735_amd import binding as B
    base = dict(n=1, h=32, w=32, cin=3, in_c_stride=3, cout=64, kh=7, kw=7, stride_h=2, stride_w=2, pad_h=3, pad_w=3,
                out_c_stride=64, mul=20000, shift=24)
    for over, pool in ((dict(cin=16, in_c_stride=16), (3, 2, 1)), (dict(kw=3, kh=3, pad_h=1, pad_w=1), (3, 2, 1)),
                       (dict(stride_h=1, stride_w=1), (3, 2, 1)), (dict(cout=128, out_c_stride=128), (3, 2, 1)), ({}, (2, 2, 0)),
                       (dict(out_mode=B.ICNN_OUT_RAW_S32), (3, 2, 1))):
        d = B.conv_desc(**dict(base, **over))
        with pytest.raises(B.IcnnError) as e:
            B.iconv2d_maxpool_brelu(d, *pool, 4096, 8192, 12288, 16384, stream=0)
        assert e.value.code == B.ICNN_E_UNSUPPORTED, (over, pool)


# ---------------------------------------------------------------- the block that opens a stage: projection skip included
def run_proj_block(seed, n, h, w, *, cbuf=64, b3_mag=4096, c3_mode="brelu", res_pair=None):
    """64 -> 64 -> 64 -> 256 with a 64 -> 256 projection of the block input.  Returns (gpu y, oracle y)."""
    from gpu_util import dev
    from paper_2006_11735_amd import binding as B
    g = rnd(seed)
    c, mid, co = 64, 64, 256
    x = g.integers(0, 128, size=(n, h, w, cbuf), dtype=np.uint8)
    w1 = g.integers(-127, 128, size=(mid, 1, 1, c), dtype=np.int8)
    w2 = g.integers(-127, 128, size=(mid, 3, 3, mid), dtype=np.int8)
    w3 = g.integers(-127, 128, size=(co, 1, 1, mid), dtype=np.int8)
    wq = g.integers(-127, 128, size=(co, 1, 1, c), dtype=np.int8)
    b1, b2 = (g.integers(-4096, 4097, size=k).astype(np.int32) for k in (mid, mid))
    b3 = g.integers(-b3_mag, b3_mag + 1, size=co).astype(np.int32)
    bq = g.integers(-4096, 4097, size=co).astype(np.int32)
    m1, s1 = K.bound_params(K.percentile_999(O.conv2d(x, w1, b1, cin=c, out_mode="raw_s32")), 127)
    t1 = O.conv2d(x, w1, b1, cin=c, mul=m1, shift=s1, bound_q=127)
    m2, s2 = K.bound_params(K.percentile_999(O.conv2d(t1, w2, b2, pad=1, out_mode="raw_s32")), 127)
    t2 = O.conv2d(t1, w2, b2, pad=1, mul=m2, shift=s2, bound_q=127)
    yq = O.conv2d(x, wq, bq, cin=c, out_mode="raw_s32")
    y_main = O.conv2d(t2, w3, b3, out_mode="raw_s32")
    rm, rs = res_pair or K.mul_shift(K.percentile_999(np.abs(yq)), K.percentile_999(y_main))
    kw3 = dict(res=yq, res_mode="pre", res_mul=rm, res_shift=rs)
    m3, s3 = K.bound_params(K.percentile_999(O.conv2d(t2, w3, b3, out_mode="raw_s32", **kw3)), 127)
    if c3_mode == "linear_s8":
        want = O.conv2d(t2, w3, b3, mul=m3, shift=s3, out_mode="linear_s8", **kw3)
    else:
        want = O.conv2d(t2, w3, b3, mul=m3, shift=s3, bound_q=127, **kw3)
    d1 = B.conv_desc(n=n, h=h, w=w, cin=c, in_c_stride=cbuf, cout=mid, kh=1, kw=1, out_c_stride=mid, mul=m1, shift=s1, bound_q=127)
    d2 = B.conv_desc(n=n, h=h, w=w, cin=mid, in_c_stride=mid, cout=mid, kh=3, kw=3, pad_h=1, pad_w=1, out_c_stride=mid, mul=m2,
                     shift=s2, bound_q=127)
    d3 = B.conv_desc(n=n, h=h, w=w, cin=mid, in_c_stride=mid, cout=co, kh=1, kw=1, out_c_stride=co, mul=m3, shift=s3, bound_q=127,
                     out_mode=B.ICNN_OUT_LINEAR_S8 if c3_mode == "linear_s8" else B.ICNN_OUT_BRELU_U8,
                     res_mode=B.ICNN_RES_PRE, res_dtype=B.ICNN_S32, res_c_stride=co, res_mul=rm, res_shift=rs)
    dq = B.conv_desc(n=n, h=h, w=w, cin=c, in_c_stride=cbuf, cout=co, kh=1, kw=1, out_c_stride=co, out_mode=B.ICNN_OUT_RAW_S32)
    packs = []
    for d, wt in ((d1, w1), (d2, w2), (d3, w3), (dq, wq)):
        pk = torch.zeros(B.iconv2d_packed_weight_bytes(d), dtype=torch.uint8, device="cuda:0")
        B.iconv2d_prepack_weights(d, dev(wt), pk)
        packs.append(pk)
    y = torch.zeros(want.shape, dtype=torch.int8 if c3_mode == "linear_s8" else torch.uint8, device="cuda:0")
    B.iconv2d_bottleneck_dual_brelu(d1, dev(x), packs[0], dev(b1), d2, packs[1], dev(b2), d3, packs[2], dev(b3), dq, packs[3],
                                    dev(bq), y)
    torch.cuda.synchronize()
    return y.cpu().numpy(), want


@pytest.mark.parametrize("shape", [(2, 56, 56), (1, 17, 23), (1, 5, 6), (14, 56, 56), (1, 1, 1), (1, 1, 150)],
                         ids=lambda s: "x".join(map(str, s)))
def test_fused_projection_bottleneck_equals_its_layers(shape):
    got, want = run_proj_block(sum(shape), *shape)
    assert got.shape == want.shape
    assert (got == want).all(), "%d of %d bytes differ" % (int((got != want).sum()), want.size)
    assert want.max() == 127 and want.min() == 0


def test_fused_projection_bottleneck_variants():
    # a wider input buffer; biases near the contract's limit (with a fixed skip ratio the proof accepts); a signed output
    for kw in (dict(cbuf=96), dict(b3_mag=1 << 27, res_pair=(20011, 15)), dict(c3_mode="linear_s8")):
        got, want = run_proj_block(31, 2, 11, 13, **kw)
        assert (got == want).all(), kw


def test_fused_projection_bottleneck_refuses_other_shapes():
    from paper_2006_11735_amd import binding as B

    def descs(**over):
        d1 = B.conv_desc(n=1, h=8, w=8, cin=64, in_c_stride=64, cout=64, kh=1, kw=1, out_c_stride=64, mul=20000, shift=24)
        d2 = B.conv_desc(n=1, h=8, w=8, cin=64, in_c_stride=64, cout=64, kh=3, kw=3, pad_h=1, pad_w=1, out_c_stride=64, mul=20000,
                         shift=26)
        d3 = B.conv_desc(n=1, h=8, w=8, cin=64, in_c_stride=64, cout=256, kh=1, kw=1, out_c_stride=256, mul=20000, shift=24,
                         res_mode=B.ICNN_RES_PRE, res_dtype=B.ICNN_S32, res_c_stride=256, res_mul=20000, res_shift=15)
        dq = B.conv_desc(n=1, h=8, w=8, cin=64, in_c_stride=64, cout=256, kh=1, kw=1, out_c_stride=256, out_mode=B.ICNN_OUT_RAW_S32)
        ds = {"d1": d1, "d2": d2, "d3": d3, "dq": dq}
        for k, v in over.items():
            which, field = k.split("__")
            setattr(ds[which], field, v)
        return d1, d2, d3, dq
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda:0")
    bias = torch.zeros(4096, dtype=torch.int32, device="cuda:0")
    cases = [descs(d3__cout=128, dq__cout=128, d3__out_c_stride=128, d3__res_c_stride=128, dq__out_c_stride=128),
             descs(dq__stride_h=2, dq__stride_w=2), descs(d3__res_dtype=B.ICNN_U8), descs(dq__out_mode=B.ICNN_OUT_BRELU_U8),
             descs(d3__out_mode=B.ICNN_OUT_RAW_S32), descs(d3__res_mul=2 ** 30, d3__res_shift=0), descs(d1__bound_q=255),
             descs(dq__in_c_stride=128)]
    for d1, d2, d3, dq in cases:
        with pytest.raises(B.IcnnError):
            B.iconv2d_bottleneck_dual_brelu(d1, buf, buf, bias, d2, buf, bias, d3, buf, bias, dq, buf, bias, buf)
    torch.cuda.synchronize()
