"""GPU parity of two branches of one input in one launch (iconv2d_twin_brelu) against the oracle's two separate layers,
bit for bit, in the shared output buffer."""
import numpy as np
import pytest
import torch

from oracle import calibrate as K
from oracle import oracle as O

pytestmark = pytest.mark.gpu


def run_twin(seed, n, h, w, cin, ka, cout_a, cout_b, *, off_a=0, off_b=None, cbuf=None, xbuf=None, mode_b="brelu", separate=False):
    """Branch a: ka x ka, cout_a channels at channel off_a of the output buffer; branch b: (ka - 2) x (ka - 2), cout_b
    channels at off_b (default: right behind a).  Returns (GPU buffer, oracle buffer), both [n, h, w, cbuf]; with
    separate=True branch b writes a buffer of its own and a pair of pairs is returned."""
    from gpu_util import dev
    from paper_2006_11735_amd import binding as B
    g = np.random.default_rng(seed)
    kb = ka - 2
    off_b = off_a + cout_a if off_b is None else off_b
    cbuf = max(off_a + cout_a, off_b + cout_b) if cbuf is None else cbuf
    xbuf = cin if xbuf is None else xbuf
    x = g.integers(0, 128, size=(n, h, w, xbuf), dtype=np.uint8)
    wa = g.integers(-127, 128, size=(cout_a, ka, ka, cin), dtype=np.int8)
    wb = g.integers(-127, 128, size=(cout_b, kb, kb, cin), dtype=np.int8)
    ba = g.integers(-4096, 4097, size=cout_a).astype(np.int32)
    bb = g.integers(-4096, 4097, size=cout_b).astype(np.int32)
    # each branch calibrated by itself, as the branches of a concatenation are (their multipliers differ)
    ma, sa = K.bound_params(K.percentile_999(O.conv2d(x, wa, ba, cin=cin, pad=ka // 2, out_mode="raw_s32")))
    mb, sb = K.bound_params(K.percentile_999(O.conv2d(x, wb, bb, cin=cin, pad=kb // 2, out_mode="raw_s32")))
    canvas = g.integers(0, 256, size=(n, h, w, cbuf), dtype=np.uint8)          # canary bytes in the channels no branch owns
    kw_b = dict(out_mode=mode_b)
    if mode_b == "clamp_u8":
        kw_b.update(lo=3, hi=200)
    if separate:
        want_a = O.conv2d(x, wa, ba, cin=cin, pad=ka // 2, mul=ma, shift=sa, out=canvas.copy(), out_c_offset=off_a)
        want_b = O.conv2d(x, wb, bb, cin=cin, pad=kb // 2, mul=mb, shift=sb, **kw_b)
    else:
        want = O.conv2d(x, wa, ba, cin=cin, pad=ka // 2, mul=ma, shift=sa, out=canvas.copy(), out_c_offset=off_a)
        want = O.conv2d(x, wb, bb, cin=cin, pad=kb // 2, mul=mb, shift=sb, out=want, out_c_offset=off_b, **kw_b)

    da = B.conv_desc(n=n, h=h, w=w, cin=cin, in_c_stride=xbuf, cout=cout_a, kh=ka, kw=ka, pad_h=ka // 2, pad_w=ka // 2,
                     out_c_stride=cbuf, out_c_offset=off_a, mul=ma, shift=sa, bound_q=127)
    db = B.conv_desc(n=n, h=h, w=w, cin=cin, in_c_stride=xbuf, cout=cout_b, kh=kb, kw=kb, pad_h=kb // 2, pad_w=kb // 2,
                     out_c_stride=cout_b if separate else cbuf, out_c_offset=0 if separate else off_b, mul=mb, shift=sb, bound_q=127)
    if mode_b == "clamp_u8":
        db.out_mode, db.lo, db.hi = B.ICNN_OUT_CLAMP_U8, 3, 200
    if mode_b == "raw_s32":
        db.out_mode = B.ICNN_OUT_RAW_S32
    packs = []
    for d, wt in ((da, wa), (db, wb)):
        pk = torch.zeros(B.iconv2d_packed_weight_bytes(d), dtype=torch.uint8, device="cuda:0")
        B.iconv2d_prepack_weights(d, dev(wt), pk)
        packs.append(pk)
    yd = dev(canvas)
    yb = torch.zeros((n, h, w, cout_b), dtype=torch.int32 if mode_b == "raw_s32" else torch.uint8, device="cuda:0") if separate else yd
    B.iconv2d_twin_brelu(da, dev(x), packs[0], dev(ba), yd, db, packs[1], dev(bb), yb)
    torch.cuda.synchronize()
    if separate:
        return (yd.cpu().numpy(), yb.cpu().numpy()), (want_a, want_b)
    return yd.cpu().numpy(), want


TWINS = [
    # n, h, w, cin, ka, cout_a, cout_b, off_a, off_b
    (1, 32, 64, 64, 5, 32, 16, 0, 32),       # the restoration network's second layer: 5x5 beside 3x3
    (1, 32, 64, 48, 3, 16, 32, 0, 16),       # its third layer: 3x3 beside 1x1 on 48 channels
    (2, 48, 96, 64, 5, 32, 16, 0, 32),       # several tiles in both directions, two images
    (3, 16, 32, 48, 3, 16, 32, 0, 16),       # one tile per image
    (1, 32, 96, 64, 3, 16, 16, 0, 16),       # 3x3 beside 1x1 on 64 channels
    (1, 64, 64, 64, 5, 24, 8, 8, 32),        # channel counts that are no multiples of 16, a gap before the first branch
    (1, 32, 32, 48, 3, 32, 32, 32, 0),       # the smaller kernel's channels first
    (1, 37, 70, 64, 5, 32, 16, 0, 32),       # pictures that are no multiples of the tile
    (2, 21, 45, 48, 3, 16, 32, 0, 16),
]


@pytest.mark.parametrize("case", TWINS, ids=lambda c: "x".join(map(str, c)))
def test_twin_branches_match_two_layers(case):
    n, h, w, cin, ka, ca, cb, oa, ob = case
    got, want = run_twin(7, n, h, w, cin, ka, ca, cb, off_a=oa, off_b=ob)
    assert (got == want).all()
    assert want[..., oa:oa + ca].max() == 127 and want[..., ob:ob + cb].max() == 127 and want.min() == 0


def test_twin_without_the_pipelined_epilogue():
    from paper_2006_11735_amd import binding as B
    B.icnn_set_tuning("plane_no_pipe", 1)
    try:
        got, want = run_twin(12, 2, 32, 64, 48, 3, 16, 32)
        assert (got == want).all()
    finally:
        B.icnn_set_tuning("reset")


def test_twin_in_a_wider_buffer_and_from_a_wider_input():
    got, want = run_twin(8, 1, 32, 64, 64, 5, 32, 16, off_a=16, cbuf=96, xbuf=80)
    assert (got == want).all()
    got, want = run_twin(9, 2, 16, 64, 48, 3, 16, 32, off_a=0, cbuf=64, xbuf=64)
    assert (got == want).all()


def test_twin_with_outputs_of_their_own_and_a_clamped_branch():
    (ya, yb), (wa, wb) = run_twin(10, 1, 32, 64, 64, 5, 32, 16, separate=True)
    assert (ya == wa).all() and (yb == wb).all()
    got, want = run_twin(11, 1, 32, 64, 48, 3, 16, 32, mode_b="clamp_u8")
    assert (got == want).all()
    # the smaller kernel's branch as raw accumulators (its own int32 buffer), beside a requantised branch
    for shape in ((1, 32, 64, 64, 5, 32, 16), (2, 19, 40, 48, 3, 16, 32)):
        (ya, yb), (wa, wb) = run_twin(13, *shape, separate=True, mode_b="raw_s32")
        assert yb.dtype == np.int32 and (ya == wa).all() and (yb == wb).all()


def test_twin_refuses_what_it_does_not_take():
    from gpu_util import dev
    from paper_2006_11735_amd import binding as B
    x = dev(np.zeros((1, 32, 64, 64), np.uint8))
    y = torch.zeros((1, 32, 64, 48), dtype=torch.uint8, device="cuda:0")
    bias = dev(np.zeros(32, np.int32))

    def desc(k, cout, off, **kw):
        args = dict(n=1, h=32, w=64, cin=64, in_c_stride=64, cout=cout, kh=k, kw=k, pad_h=k // 2, pad_w=k // 2, out_c_stride=48,
                    out_c_offset=off, mul=1, shift=10, bound_q=127)
        args.update(kw)
        return B.conv_desc(**args)

    def packed(d):
        wt = dev(np.zeros((d.cout, d.kh, d.kw, d.cin), np.int8))
        pk = torch.zeros(B.iconv2d_packed_weight_bytes(d), dtype=torch.uint8, device="cuda:0")
        B.iconv2d_prepack_weights(d, wt, pk)
        return pk
    good_a, good_b = desc(5, 32, 0), desc(3, 16, 32)
    B.iconv2d_twin_brelu(good_a, x, packed(good_a), bias, y, good_b, packed(good_b), bias, y)
    for da, db in ((desc(5, 32, 0), desc(5, 16, 32)),                       # kernels of the same size
                   (desc(5, 32, 0, stride_h=2, stride_w=2), desc(3, 16, 32, stride_h=2, stride_w=2)),
                   (desc(5, 64, 0, out_c_stride=80), desc(3, 16, 64, out_c_stride=80)),        # more than 32 channels
                   (desc(7, 32, 0), desc(5, 16, 32))):
        with pytest.raises(B.IcnnError) as e:
            B.iconv2d_twin_brelu(da, x, packed(da), bias, y, db, packed(db), bias, y)
        assert e.value.code == B.ICNN_E_UNSUPPORTED
    torch.cuda.synchronize()
