"""GPU parity of the fused pair of pointwise layers (iconv2d_pair_brelu) against the oracle's two separate layers,
bit for bit, on both outputs."""
import numpy as np
import pytest
import torch

from oracle import calibrate as K
from oracle import oracle as O

pytestmark = pytest.mark.gpu


def run_pair(seed, n, h, w, mid, c, *, skip=True, form3="auto", form1="auto", bound_y=127, bound_z=127, tbuf=None, ybuf=None):
    """Returns ((y, z) from the GPU, (y, z) from the oracle).  form*: how a layer requantises: "auto" = calibrated
    15-bit multiplier (the 32-bit form), "hi" = a pair only the one-multiply form takes, "wide" = only the general form."""
    from gpu_util import dev
    from paper_2006_11735_amd import binding as B
    g = np.random.default_rng(seed)
    tbuf = mid if tbuf is None else tbuf
    ybuf = c if ybuf is None else ybuf
    t = g.integers(0, 128, size=(n, h, w, tbuf), dtype=np.uint8)
    w3 = g.integers(-127, 128, size=(c, 1, 1, mid), dtype=np.int8)
    w1 = g.integers(-127, 128, size=(mid, 1, 1, c), dtype=np.int8)
    b3 = g.integers(-4096, 4097, size=c).astype(np.int32)
    b1 = g.integers(-4096, 4097, size=mid).astype(np.int32)

    def widen(m, s, form):
        if form == "hi":
            return m << 14, s + 14
        if form == "wide":
            return m << 16, s + 16 if s + 16 > 32 else 33
        return m, s
    kw3 = {}
    res = None
    if skip:
        res = g.integers(0, 128, size=(n, h, w, c), dtype=np.uint8)
        y_main = O.conv2d(t, w3, b3, cin=mid, out_mode="raw_s32")
        rm, rs = K.mul_shift(127, K.percentile_999(y_main))
        kw3.update(res=res, res_mode="pre", res_mul=rm, res_shift=rs)
    y_raw = O.conv2d(t, w3, b3, cin=mid, out_mode="raw_s32", **kw3)
    m3, s3 = widen(*K.bound_params(K.percentile_999(y_raw), bound_y), form3)
    y = O.conv2d(t, w3, b3, cin=mid, mul=m3, shift=s3, bound_q=bound_y, **kw3)
    z_raw = O.conv2d(y, w1, b1, out_mode="raw_s32")
    m1, s1 = widen(*K.bound_params(K.percentile_999(z_raw), bound_z), form1)
    z = O.conv2d(y, w1, b1, mul=m1, shift=s1, bound_q=bound_z)

    d3 = B.conv_desc(n=n, h=h, w=w, cin=mid, in_c_stride=tbuf, cout=c, kh=1, kw=1, out_c_stride=ybuf, mul=m3, shift=s3,
                     bound_q=bound_y)
    if skip:
        d3.res_mode, d3.res_c_stride, d3.res_dtype = B.ICNN_RES_PRE, c, B.ICNN_U8
        d3.res_mul, d3.res_shift = rm, rs
    d1 = B.conv_desc(n=n, h=h, w=w, cin=c, in_c_stride=ybuf, cout=mid, kh=1, kw=1, out_c_stride=mid, mul=m1, shift=s1,
                     bound_q=bound_z)
    packs = []
    for d, wt in ((d3, w3), (d1, w1)):
        pk = torch.zeros(B.iconv2d_packed_weight_bytes(d), dtype=torch.uint8, device="cuda:0")
        B.iconv2d_prepack_weights(d, dev(wt), pk)
        packs.append(pk)
    yd = torch.full((n, h, w, ybuf), 0xEE, dtype=torch.uint8, device="cuda:0")
    zd = torch.zeros((n, h, w, mid), dtype=torch.uint8, device="cuda:0")
    B.iconv2d_pair_brelu(d3, dev(t), packs[0], dev(b3), None if res is None else dev(res), yd, d1, packs[1], dev(b1), zd)
    torch.cuda.synchronize()
    yh = yd.cpu().numpy()
    assert (yh[..., c:] == 0xEE).all()            # channels of the buffer beyond the layer's are left alone
    return (yh[..., :c], zd.cpu().numpy()), (y, z)


PAIRS = [
    # n, h, w, mid, c
    (4, 14, 14, 256, 1024),      # stage-3 shape: 784 pixels, 13 tiles with a ragged last one
    (2, 28, 28, 128, 512),       # stage-2 shape
    (1, 56, 56, 64, 256),        # stage-1 shape
    (1, 7, 7, 256, 2048),        # the widest tile the on-chip memory takes
    (1, 1, 1, 64, 256),          # a single pixel
    (3, 5, 9, 128, 768),         # three chunks per wave, ragged tile
    (1, 9, 7, 256, 256),
    (1, 3, 50, 64, 512),
]


@pytest.mark.parametrize("shape", PAIRS, ids=lambda s: "x".join(map(str, s)))
def test_fused_pair_equals_two_layers(shape):
    n, h, w, mid, c = shape
    got, want = run_pair(sum(shape), n, h, w, mid, c)
    for a, b, name in zip(got, want, "yz"):
        assert a.shape == b.shape
        assert (a == b).all(), "%s: %d of %d bytes differ" % (name, int((a != b).sum()), b.size)
    assert want[0].max() == 127 and want[1].max() == 127


@pytest.mark.parametrize("mid,c", [(64, 256), (128, 512), (256, 512)])
def test_fused_pair_epilogue_forms_and_pitches(mid, c):
    for kw in (dict(skip=False), dict(form3="hi"), dict(form3="wide", form1="hi"), dict(form1="wide"), dict(bound_y=15, bound_z=255),
               dict(tbuf=mid + 32, ybuf=c + 48), dict(skip=False, form3="hi", form1="wide")):
        got, want = run_pair(11 + mid, 2, 9, 11, mid, c, **kw)
        assert (got[0] == want[0]).all() and (got[1] == want[1]).all(), kw


def test_fused_pair_refuses_other_shapes():
    from paper_2006_11735_amd import binding as B

    def descs(mid=64, c=256, **over):
        d3 = B.conv_desc(n=1, h=8, w=8, cin=mid, in_c_stride=mid, cout=c, kh=1, kw=1, out_c_stride=c, mul=20000, shift=24)
        d1 = B.conv_desc(n=1, h=8, w=8, cin=c, in_c_stride=c, cout=mid, kh=1, kw=1, out_c_stride=mid, mul=20000, shift=24)
        for k, v in over.items():
            which, field = k.split("__")
            setattr({"d3": d3, "d1": d1}[which], field, v)
        return d3, d1
    buf = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda:0")
    bias = torch.zeros(4096, dtype=torch.int32, device="cuda:0")
    cases = [descs(mid=32, c=256), descs(mid=64, c=128), descs(mid=64, c=2304), descs(d3__bound_q=255),
             descs(d1__res_mode=B.ICNN_RES_PRE, d1__res_c_stride=64), descs(d3__out_mode=B.ICNN_OUT_RAW_S32),
             descs(d1__out_mode=B.ICNN_OUT_LINEAR_S8), descs(d3__in_signed=B.ICNN_IN_U8_FULL), descs(d1__cout=128),
             descs(d3__res_mode=B.ICNN_RES_PRE, d3__res_c_stride=256, d3__res_dtype=B.ICNN_S32, d3__res_mul=3, d3__res_shift=2)]
    for d3, d1 in cases:
        with pytest.raises(B.IcnnError):
            B.iconv2d_pair_brelu(d3, buf, buf, bias, buf, buf, d1, buf, bias, buf)
    torch.cuda.synchronize()
