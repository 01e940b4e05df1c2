"""GPU parity of the bandwidth-bound entry points against the CPU oracle (bit-exact)."""
import numpy as np
import pytest
import torch

from oracle import oracle as O

pytestmark = pytest.mark.gpu


def rnd(seed):
    return np.random.default_rng(seed)


def tensor(g, shape, kind):
    if kind == "u8":
        return g.integers(0, 128, size=shape, dtype=np.uint8)
    if kind == "s8":
        return g.integers(-128, 128, size=shape, dtype=np.int8)
    return g.integers(-400000, 400000, size=shape).astype(np.int32)


@pytest.mark.parametrize("a_kind", ["u8", "s8", "s32"])
@pytest.mark.parametrize("b_kind", ["u8", "s8", "s32"])
@pytest.mark.parametrize("c", [64, 23])
def test_add_rescale_all_operand_types(a_kind, b_kind, c):
    from gpu_util import dev
    from paper_2006_11735_amd import binding as B
    g = rnd(len(a_kind) * 7 + len(b_kind) + c)
    shape = (3, 11, 13, c)
    a, b = tensor(g, shape, a_kind), tensor(g, shape, b_kind)
    dt = {"u8": B.ICNN_U8, "s8": B.ICNN_S8, "s32": B.ICNN_S32}
    px = 3 * 11 * 13
    for out_mode, odt, kw in (("clamp_u8", np.uint8, dict(mul=23187, shift=24 if a_kind == "s32" else 9, lo=0, hi=127)),
                              ("linear_s8", np.int8, dict(mul=3, shift=4)),
                              ("raw_s32", np.int32, dict())):
        want = O.add_rescale(a, b, b_mul=18415, b_shift=5, out_mode=out_mode, **kw)
        d = B.add_desc(count_pixels=px, c=c, a_c_stride=c, b_c_stride=c, out_c_stride=c, a_dtype=dt[a_kind],
                       b_dtype=dt[b_kind], b_mul=18415, b_shift=5,
                       out_mode={"clamp_u8": B.ICNN_OUT_CLAMP_U8, "linear_s8": B.ICNN_OUT_LINEAR_S8,
                                 "raw_s32": B.ICNN_OUT_RAW_S32}[out_mode], **kw)
        out = torch.zeros(shape, dtype={np.uint8: torch.uint8, np.int8: torch.int8, np.int32: torch.int32}[odt],
                          device="cuda:0")
        B.iadd_rescale(d, dev(a), dev(b), out)
        torch.cuda.synchronize()
        assert (out.cpu().numpy() == want).all(), out_mode


def test_add_rescale_channel_offset_and_empty():
    from gpu_util import dev
    from paper_2006_11735_amd import binding as B
    g = rnd(3)
    a, b = tensor(g, (50, 32), "s32"), tensor(g, (50, 32), "u8")
    out = torch.full((50, 80), 77, dtype=torch.uint8, device="cuda:0")
    d = B.add_desc(count_pixels=50, c=32, a_c_stride=32, b_c_stride=32, out_c_stride=80, out_c_offset=16,
                   a_dtype=B.ICNN_S32, b_dtype=B.ICNN_U8, b_mul=18415, b_shift=5, mul=23187, shift=24, lo=0, hi=127)
    B.iadd_rescale(d, dev(a), dev(b), out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want = O.add_rescale(a, b, b_mul=18415, b_shift=5, mul=23187, shift=24, lo=0, hi=127)
    assert (got[:, 16:48] == want).all() and (got[:, :16] == 77).all() and (got[:, 48:] == 77).all()
    d.count_pixels = 0
    B.iadd_rescale(d, None, None, None)              # empty input: nothing to do, no error


@pytest.mark.parametrize("cs", [(32, 16), (5, 7, 4)])
def test_concat_matches_oracle_and_numpy(cs):
    from gpu_util import dev
    from paper_2006_11735_amd import binding as B
    g = rnd(4)
    px = 301
    xs = [g.integers(0, 128, size=(px, c), dtype=np.uint8) for c in cs]
    muls, shifts = [20000 + 1000 * i for i in range(len(cs))], [14 + i for i in range(len(cs))]
    for m, s in ((muls, shifts), ([1] * len(cs), [0] * len(cs))):
        out = torch.zeros((px, sum(cs)), dtype=torch.uint8, device="cuda:0")
        B.iconcat([dev(x) for x in xs], cs, cs, m, s, 100, px, out, sum(cs))
        torch.cuda.synchronize()
        assert (out.cpu().numpy() == O.concat(xs, m, s, 100)).all()
    out = torch.zeros((px, sum(cs)), dtype=torch.uint8, device="cuda:0")
    B.iconcat([dev(x) for x in xs], cs, cs, [1] * len(cs), [0] * len(cs), 127, px, out, sum(cs))
    torch.cuda.synchronize()
    assert (out.cpu().numpy() == np.concatenate(xs, axis=1)).all()


@pytest.mark.parametrize("shape", [(2, 112, 112, 64, 3, 2, 1), (1, 9, 7, 5, 3, 2, 1), (1, 8, 8, 16, 2, 2, 0),
                                   # 3x3 / 2 / 1 beyond the network shape: ragged blocks, odd
                                   # sizes, rows wider than one workgroup, one-pixel images
                                   (3, 13, 17, 32, 3, 2, 1), (1, 30, 200, 64, 3, 2, 1), (2, 7, 7, 16, 3, 2, 1),
                                   (1, 1, 1, 16, 3, 2, 1), (1, 2, 5, 48, 3, 2, 1), (1, 10, 4, 16, 3, 2, 1),
                                   (1, 9, 9, 16, 3, 1, 1), (1, 9, 9, 16, 3, 2, 0)])
def test_maxpool(shape):
    from gpu_util import dev
    from paper_2006_11735_amd import binding as B
    n, h, w, c, k, s, p = shape
    x = rnd(5).integers(0, 256, size=(n, h, w, c), dtype=np.uint8)
    want = O.maxpool2d(x, k, s, p)
    out = torch.zeros(want.shape, dtype=torch.uint8, device="cuda:0")
    B.imaxpool2d_u8(n, h, w, c, k, s, p, dev(x), out)
    torch.cuda.synchronize()
    assert (out.cpu().numpy() == want).all()


def test_global_average_pool_and_renormalise():
    from gpu_util import dev
    from paper_2006_11735_amd import binding as B
    x = rnd(6).integers(0, 128, size=(5, 7, 7, 2048), dtype=np.uint8)
    want = O.avgpool_global(x, 21400, 20, 127)
    out = torch.zeros((5, 1, 1, 2048), dtype=torch.uint8, device="cuda:0")
    B.iavgpool_global_u8(5, 7, 7, 2048, 21400, 20, 127, dev(x), out)
    torch.cuda.synchronize()
    assert (out.cpu().numpy() == want).all()
    # ragged channel counts (one partly filled workgroup; the scalar kernel for c % 4 != 0), odd window sizes,
    # values up to 255, a clamp that bites
    for (n, h, w, c, mul, shift, bound) in ((3, 5, 6, 300, 17476, 19, 127), (2, 3, 3, 7, 29127, 18, 255), (1, 1, 1, 64, 1, 0, 90),
                                            (2, 13, 11, 1028, 30000, 20, 127)):
        x = rnd(60 + c).integers(0, 256, size=(n, h, w, c), dtype=np.uint8)
        want = O.avgpool_global(x, mul, shift, bound)
        out = torch.zeros((n, 1, 1, c), dtype=torch.uint8, device="cuda:0")
        B.iavgpool_global_u8(n, h, w, c, mul, shift, bound, dev(x), out)
        torch.cuda.synchronize()
        assert (out.cpu().numpy() == want).all(), (n, h, w, c)
    for count in (4096, 1001):
        raw = rnd(7).integers(0, 256, size=count, dtype=np.uint8)
        o = torch.zeros(count, dtype=torch.uint8, device="cuda:0")
        B.irenormalize_u8(count, dev(raw), o)
        torch.cuda.synchronize()
        assert (o.cpu().numpy().view(np.int8) == O.renormalize(raw)).all()


@pytest.mark.parametrize("pair", [(8388608, 23), (8421504, 30), (8388607, 23)], ids=lambda p: "%dx2^-%d" % p)
@pytest.mark.parametrize("a_kind", ["s32", "s8", "u8"])
@pytest.mark.parametrize("b_kind", ["u8", "s8"])
def test_add_rescale_multipliers_of_24_bits(pair, a_kind, b_kind):
    """b multipliers with bit 23 set pass the 32-bit gate (255 * b_mul + half < 2^31); the signed 24-bit
    multiply of the fast kernel must not take them."""
    from gpu_util import dev
    from paper_2006_11735_amd import binding as B
    b_mul, b_shift = pair
    g = rnd(sum(pair) + len(a_kind))
    shape = (2, 9, 13, 32)
    a, b = tensor(g, shape, a_kind), tensor(g, shape, b_kind)
    if b_kind == "u8":
        b = g.integers(0, 256, size=shape, dtype=np.uint8)
    dt = {"u8": B.ICNN_U8, "s8": B.ICNN_S8, "s32": B.ICNN_S32}
    for out_mode, tdt, kw in (("clamp_u8", torch.uint8, dict(mul=23187, shift=24 if a_kind == "s32" else 16, lo=0, hi=200)),
                              ("raw_s32", torch.int32, dict())):
        want = O.add_rescale(a, b, b_mul=b_mul, b_shift=b_shift, out_mode=out_mode, **kw)
        d = B.add_desc(count_pixels=2 * 9 * 13, c=32, a_c_stride=32, b_c_stride=32, out_c_stride=32, a_dtype=dt[a_kind],
                       b_dtype=dt[b_kind], b_mul=b_mul, b_shift=b_shift,
                       out_mode={"clamp_u8": B.ICNN_OUT_CLAMP_U8, "raw_s32": B.ICNN_OUT_RAW_S32}[out_mode], **kw)
        out = torch.zeros(shape, dtype=tdt, device="cuda:0")
        B.iadd_rescale(d, dev(a), dev(b), out)
        torch.cuda.synchronize()
        assert (out.cpu().numpy() == want).all(), out_mode


ADD_U8_PARAMS = [
    # b_mul, b_shift, mul, shift, hi
    (18415, 5, 23187, 24, 127), (1, 0, 1, 1, 255), (1, 0, 3, 1, 255), ((1 << 23) - 1, 20, (1 << 24) - 1, 31, 255),
    (40000, 7, 6 << 10, 22, 15), (255, 8, 52429, 19, 63), (8421504, 30, 1 << 20, 21, 200), (7, 1, 999983, 30, 127),
    (1 << 22, 0, 5, 31, 255),        # skip term up to 2^30
]


@pytest.mark.parametrize("params", ADD_U8_PARAMS, ids=lambda p: "-".join(map(str, p)))
@pytest.mark.parametrize("dense", [True, False])
def test_add_of_two_unsigned_maps_in_32_bits(params, dense):
    """The unsigned 8-bit + 8-bit -> 8-bit kernel over full-range bytes, multipliers at the limits of its 24-bit form."""
    from gpu_util import dev
    from paper_2006_11735_amd import binding as B
    b_mul, b_shift, mul, shift, hi = params
    g = rnd(sum(params))
    px, c = 1111, 48
    a = g.integers(0, 256, size=(px, c), dtype=np.uint8)
    b = g.integers(0, 256, size=(px, c), dtype=np.uint8)
    a[0, :4] = [0, 255, 0, 255]
    b[0, :4] = [0, 0, 255, 255]
    want = O.add_rescale(a, b, b_mul=b_mul, b_shift=b_shift, mul=mul, shift=shift, lo=0, hi=hi)
    ocs, oco = (c, 0) if dense else (96, 32)
    out = torch.full((px, ocs), 9, dtype=torch.uint8, device="cuda:0")
    d = B.add_desc(count_pixels=px, c=c, a_c_stride=c, b_c_stride=c, out_c_stride=ocs, out_c_offset=oco, a_dtype=B.ICNN_U8,
                   b_dtype=B.ICNN_U8, b_mul=b_mul, b_shift=b_shift, mul=mul, shift=shift, lo=0, hi=hi)
    B.iadd_rescale(d, dev(a), dev(b), out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert (got[:, oco:oco + c] == want).all()
    if not dense:
        assert (got[:, :oco] == 9).all() and (got[:, oco + c:] == 9).all()


@pytest.mark.parametrize("params", [(20000, 14, 100), (1, 1, 255), ((1 << 24) - 1, 31, 255), (3 << 20, 21, 15), (999983, 18, 63),
                                    (1 << 24, 24, 127), (1 << 30, 31, 127)], ids=lambda p: "-".join(map(str, p)))
def test_concat_requantisation_in_32_bits(params):
    from gpu_util import dev
    from paper_2006_11735_amd import binding as B
    mul, shift, bound = params
    g = rnd(sum(params))
    px = 777
    xs = [g.integers(0, 256, size=(px, c), dtype=np.uint8) for c in (32, 16)]
    out = torch.zeros((px, 48), dtype=torch.uint8, device="cuda:0")
    B.iconcat([dev(x) for x in xs], [32, 16], [32, 16], [mul, mul], [shift, shift], bound, px, out, 48)
    torch.cuda.synchronize()
    assert (out.cpu().numpy() == O.concat(xs, [mul, mul], [shift, shift], bound)).all()


def test_concat_of_several_aligned_branches_in_one_launch():
    """Branches of different widths and pitches, one without channels, one with a pair the 32-bit form does not take;
    the output rows are wider than the concatenation and keep what lies beyond it."""
    from gpu_util import dev
    from paper_2006_11735_amd import binding as B
    g = rnd(11)
    px = 1234
    cs, pitch = [48, 0, 16, 64], [64, 16, 16, 80]
    muls, shifts = [20000, 5, 1, 3 << 20], [14, 3, 0, 22]
    bufs = [g.integers(0, 256, size=(px, p), dtype=np.uint8) for p in pitch]
    xs = [b[:, :c] for b, c in zip(bufs, cs)]
    out = torch.full((px, 160), 201, dtype=torch.uint8, device="cuda:0")
    B.iconcat([dev(b) for b in bufs], cs, pitch, muls, shifts, 127, px, out, 160)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want = O.concat([x for x in xs if x.shape[1]], [m for m, c in zip(muls, cs) if c], [s for s, c in zip(shifts, cs) if c], 127)
    assert (got[:, :128] == want).all() and (got[:, 128:] == 201).all()


def test_every_byte_through_random_requantisation_pairs():
    """iconcat's requantisation over all 256 input bytes for 300 seeded (mul, shift, bound) triples that straddle
    the limits of the 32-bit form (multipliers around 2^24, shifts 0..40, bounds 1..255)."""
    from gpu_util import dev
    from paper_2006_11735_amd import binding as B
    g = rnd(2024)
    x = np.arange(256, dtype=np.uint8).reshape(16, 16)
    xd = dev(x)
    out = torch.zeros((16, 16), dtype=torch.uint8, device="cuda:0")
    for _ in range(300):
        shift = int(g.integers(0, 41))
        bits = int(g.integers(1, 31))
        mul = int(g.integers(1 << (bits - 1), 1 << bits)) if g.integers(0, 4) else int(1 << bits)
        bound = int(g.choice([1, 15, 31, 63, 100, 127, 200, 255]))
        B.iconcat([xd], [16], [16], [mul], [shift], bound, 16, out, 16)
        torch.cuda.synchronize()
        want = O.concat([x], [mul], [shift], bound)
        assert (out.cpu().numpy() == want).all(), (mul, shift, bound)


def test_every_pair_of_bytes_through_random_addition_parameters():
    """iadd_rescale u8 + u8 -> u8 over all 65536 (a, b) byte pairs for 120 seeded parameter sets around the limits
    of the 32-bit kernel (and beyond them, where the general kernel takes over)."""
    from gpu_util import dev
    from paper_2006_11735_amd import binding as B
    g = rnd(2025)
    a = np.repeat(np.arange(256, dtype=np.uint8), 256).reshape(4096, 16)
    b = np.tile(np.arange(256, dtype=np.uint8), 256).reshape(4096, 16)
    ad, bd = dev(a), dev(b)
    out = torch.zeros((4096, 16), dtype=torch.uint8, device="cuda:0")
    for _ in range(120):
        b_shift = int(g.integers(0, 31))
        b_mul = int(g.integers(1, 1 << int(g.integers(1, 25))))
        shift = int(g.integers(0, 36))
        mul = int(g.integers(1, 1 << int(g.integers(1, 27))))
        hi = int(g.choice([1, 15, 63, 127, 128, 255]))
        d = B.add_desc(count_pixels=4096, c=16, a_c_stride=16, b_c_stride=16, out_c_stride=16, a_dtype=B.ICNN_U8,
                       b_dtype=B.ICNN_U8, b_mul=b_mul, b_shift=b_shift, mul=mul, shift=shift, lo=0, hi=hi)
        B.iadd_rescale(d, ad, bd, out)
        torch.cuda.synchronize()
        want = O.add_rescale(a, b, b_mul=b_mul, b_shift=b_shift, mul=mul, shift=shift, lo=0, hi=hi)
        assert (out.cpu().numpy() == want).all(), (b_mul, b_shift, mul, shift, hi)
