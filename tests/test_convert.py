"""The offline float -> integer conversion (the paper's Algorithm 1 without its training steps):
its integer helpers against exact rationals and the paper's post-condition, batch-norm
folding against a library batch norm, the ratio bookkeeping at merges and concatenations, and the
end-to-end property the method exists for: the integer network (run by the CPU oracle) tracks the
BReLU-enabled float network to within a few quantisation steps."""
import numpy as np
import pytest
import torch

from oracle import net as ONet
from oracle import oracle as O
from paper_2006_11735_amd import convert as C
from workloads import nets as W


def float_params(net, seed, bn=False):
    """He-initialised float weights, small biases, optionally a batch norm behind every BReLU conv."""
    g = np.random.default_rng(seed)
    prm = {}
    for op in net["ops"]:
        if op["op"] != "conv":
            continue
        fan = op["kh"] * op["kw"] * op["cin"]
        p = {"w": g.normal(0, (2.0 / fan) ** 0.5, size=(op["cout"], op["kh"], op["kw"], op["cin"])),
             "b": g.normal(0, 0.05, size=op["cout"])}
        if bn and op["out_mode"] == "brelu":
            c = op["cout"]
            p["bn"] = (g.uniform(0.5, 1.5, c), g.normal(0, 0.1, c), g.normal(0, 0.1, c), g.uniform(0.5, 1.5, c), 1e-5)
        prm[op["name"]] = p
    return prm


def test_integer_helpers_against_exact_rationals_and_the_bound_condition():
    """mul_shift: mul / 2^shift within 2^-15 of b / a (half a unit of a 15-bit multiplier), the multiplier has
    15 significant bits and the shift is the smallest that gives them; bound_params: the post-condition of
    Section 3.3, [h_ri * mul / 2^shift] = max_int, with a multiplier that stays next to the rounded ratio."""
    from fractions import Fraction
    g = np.random.default_rng(1)
    cases = [(int(g.integers(1, 1 << 24)), int(g.integers(1, 1 << 24))) for _ in range(3000)]
    cases += [(1, 1), (127, 1), (1, 127), (3, 1 << 20), ((1 << 24) - 1, 1), (1, (1 << 24) - 1), (12345, 12345)]
    for a, b in cases:
        m, s = C.mul_shift(a, b)
        ratio = Fraction(b, a)
        assert 0 <= s <= 46 and 1 <= m < (1 << 31)
        if s < 46 and m < (1 << 31) - 1:
            assert m >= (1 << 14)
            assert abs(Fraction(m, 1 << s) / ratio - 1) <= Fraction(1, 1 << 15), (a, b, m, s)
            assert s == 0 or ratio * (1 << (s - 1)) + Fraction(1, 2) < (1 << 14), (a, b, m, s)     # smallest such shift
            assert abs(Fraction(m) - ratio * (1 << s)) <= Fraction(1, 2)                                # rounded, not truncated
    for max_int in (127, 255, 15):
        for h in list(range(1, 600)) + [int(v) for v in g.integers(600, 1 << 24, size=600)]:
            m, s = C.bound_params(h, max_int)
            assert O.requant(h, m, s) == max_int                                                        # Section 3.3
            exact = (int(h) * m + ((1 << s) >> 1)) >> s                                                 # the same in big integers
            assert exact == max_int
            m0, s0 = C.mul_shift(h, max_int)
            assert s == s0 and abs(m - m0) <= max(1, m0 >> 13), (h, max_int, m, m0)
    x = g.normal(0, 40, size=1000)
    assert (C.rhu(x) == np.floor(x + 0.5)).all() and C.rhu(-2.5) == -2 and C.rhu(2.5) == 3


def test_batch_norm_folding_matches_a_library_batch_norm():
    g = np.random.default_rng(2)
    w, b = g.normal(size=(6, 3, 3, 5)), g.normal(size=6)
    bn = (g.uniform(0.5, 2, 6), g.normal(size=6), g.normal(size=6), g.uniform(0.3, 2, 6), 1e-5)
    x = g.normal(size=(2, 7, 8, 5))
    wf, bf = C.fold_bn(w, b, bn)
    got = C._conv_f(x, wf, 1, 1) + bf
    y = torch.from_numpy(C._conv_f(x, w, 1, 1) + b).permute(0, 3, 1, 2)
    t = [torch.from_numpy(np.asarray(v, np.float64)) for v in bn[:4]]
    want = torch.nn.functional.batch_norm(y, t[2], t[3], t[0], t[1], False, 0.0, bn[4]).permute(0, 2, 3, 1).numpy()
    assert np.allclose(got, want, rtol=1e-9, atol=1e-9)


NETS = [("vdsr", lambda: W.vdsr(40, 52, depth=5), False, False),
        ("vrcnn", lambda: W.vrcnn(36, 44), False, False),
        ("resnet", lambda: W.resnet(4, [2, 1, 1, 1], "tiny", image=64, calib_images=4, classes=10), True, False),
        ("resnet-per-channel", lambda: W.resnet(4, [2, 1, 1, 1], "tiny", image=64, calib_images=4, classes=10), True, True),
        ("resnet-basic", lambda: W.resnet_basic(2, [1, 1, 1, 1], "tiny18", image=64, calib_images=2, classes=10), True, False)]


@pytest.mark.parametrize("name,make,bn,pc", NETS, ids=[n[0] for n in NETS])
def test_integer_network_tracks_the_float_network(name, make, bn, pc):
    net = make()
    raw = W.input_tensor(net, 3)
    calib, weights, info = C.convert(net, float_params(net, 5, bn), raw, per_channel=pc)
    got = ONet.run(net, 0, calib, x_raw=raw, weights=weights)
    for op in W.conv_ops(net):
        w_i, b_i = weights[op["name"]]
        assert w_i.dtype == np.int8 and np.abs(w_i.astype(int)).max() == 127 and b_i.dtype == np.int32
        cal = calib["conv"][op["name"]]
        if op["res_mode"] == "pre":
            # ratio synchronisation (Section 4.1): the rescaled skip ratio IS the main path's ratio_Y
            rs = np.atleast_1d(np.asarray(info["ratio"][op["res"]], float))
            ry = np.atleast_1d(np.asarray(info["ratio_y"][op["name"]], float))
            pairs = list(zip(cal["res_mul_c"], cal["res_shift_c"])) if "res_mul_c" in cal else [(cal["res_mul"], cal["res_shift"])]
            for (m, s), a, b in zip(pairs, np.broadcast_to(rs, (len(pairs),)), np.broadcast_to(ry, (len(pairs),))):
                assert abs(a * m / 2.0 ** s / b - 1) < 1e-9
    for bname, b in net["buffers"].items():
        if bname == "raw":
            continue
        f, r = info["float"][bname], info["ratio"][bname]
        err = np.abs(got[bname].astype(np.float64) / r - f)
        if b["dtype"] == "s32":                       # projections, logits: no activation quantisation of their own
            assert err.mean() < 0.02 * np.abs(f).max(), bname
            continue
        step = 1.0 / float(np.max(r))                # one quantisation step in float units
        if bname == "out":                           # regression output, pixel levels
            assert err.mean() < 1.5 and np.percentile(err, 99) <= 6, (bname, err.mean(), err.max())
        else:
            assert err.mean() < 1.0 * step and err.max() < 12 * step, (bname, err.mean() / step, err.max() / step)
            assert got[bname].max() <= calib["max_int"]
    first = W.conv_ops(net)[0]["dst"]                 # only rounding separates the first layer's two versions
    e0 = np.abs(got[first].astype(np.float64) / info["ratio"][first] - info["float"][first]) * info["ratio"][first]
    assert e0.max() <= 0.51                          # half a step, plus the rounded bias
    if "logits" in got:
        fl, il = info["float"]["logits"].reshape(len(raw), -1), got["logits"].reshape(len(raw), -1).astype(np.float64)
        for a, b in zip(fl, il):
            assert np.corrcoef(a, b)[0, 1] > 0.98


def test_concatenated_branches_share_one_ratio_and_lower_bounds():
    net = W.vrcnn(36, 44)
    raw = W.input_tensor(net, 4)
    calib, weights, info = C.convert(net, float_params(net, 6), raw)
    for a, b in (("conv2a", "conv2b"), ("conv3a", "conv3b")):
        ca, cb = calib["conv"][a], calib["conv"][b]
        ra = info["ratio_y"][a] * ca["mul"] / 2.0 ** ca["shift"]
        rb = info["ratio_y"][b] * cb["mul"] / 2.0 ** cb["shift"]
        assert abs(ra / rb - 1) < 1e-9                      # Algorithm 2: one ratio after the rescale
        assert max(ca["bound_q"], cb["bound_q"]) == 127 and min(ca["bound_q"], cb["bound_q"]) >= 1


def test_other_bit_depths_and_n_sigma():
    net = W.vdsr(32, 36, depth=4)
    raw = W.input_tensor(net, 7)
    prm = float_params(net, 8)
    errs = {}
    for max_int in (255, 127, 15):
        calib, weights, info = C.convert(net, prm, raw, max_int=max_int)
        got = ONet.run(net, 0, calib, x_raw=raw, weights=weights)
        assert got["a2"].max() == max_int
        errs[max_int] = np.abs(got["out"].astype(float) - info["float"]["out"]).mean()
    assert errs[255] < errs[127] < errs[15]                  # fewer activation bits, larger error (the paper's Table 5 trend)
    wide, _, iw = C.convert(net, prm, raw, n_sigma=4.0)
    narrow, _, inn = C.convert(net, prm, raw, n_sigma=2.0)
    assert iw["h_f"]["conv2"] > inn["h_f"]["conv2"]
