"""Pins of the oracle-side calibration (Section 3.3's bound condition, Algorithm 2's
post-condition) and of the workload shapes."""
import json
import random
from fractions import Fraction

import numpy as np
import pytest

from oracle import calibrate as K
from oracle import net as ONet
from oracle import oracle as O
from workloads import nets as W


def test_bound_params_meet_the_papers_postcondition():
    # Section 3.3: max_int = [h_ri * mul / 2^shift]
    hs = list(range(1, 1 << 12)) + list(range(1 << 12, 1 << 16, 37))
    rnd = random.Random(3)
    hs += [rnd.randint(1 << 16, 1 << 24) for _ in range(3000)] + [(1 << 24), (1 << 31) - 1]
    for h in hs:
        mul, s = K.bound_params(h, 127)
        assert 1 <= mul < (1 << 31) and 0 <= s <= K.MAX_SHIFT
        assert O.requant(h, mul, s) == 127, h
        if s < K.MAX_SHIFT:
            assert (1 << 14) <= mul <= (1 << 15) + 1, (h, mul, s)


def test_mul_shift_approximates_the_ratio():
    rnd = random.Random(4)
    for _ in range(2000):
        a, b = rnd.randint(1, 1 << 22), rnd.randint(1, 1 << 22)
        mul, s = K.mul_shift(a, b)
        r = Fraction(b, a)
        if r >= (1 << 15):
            assert s == 0 and abs(mul - r) <= Fraction(1, 2)
        elif mul >= (1 << 14):
            assert abs(Fraction(mul, 1 << s) / r - 1) <= Fraction(1, 1 << 14)
    assert K.mul_shift(49, 1) == (21400, 20)          # 2^20 / 49 = 21399.51
    assert K.mul_shift(1, 1) == (16384, 14)
    assert K.mul_shift(1, 1 << 20) == (1 << 20, 0)


def test_percentile_is_nearest_rank():
    v = np.arange(1, 1001)                              # 1..1000
    assert K.percentile_999(v) == 999                   # ceil(0.999*1000) = 999th smallest
    assert K.percentile_999(np.arange(1, 2001)) == 1998
    assert K.percentile_999(np.array([-5, -3])) == 1    # floor at 1
    assert K.percentile_999(np.array([-5000, 3, 4]), absolute=True) == 5000


def test_concat_sync_postconditions():
    # Algorithm 2: every branch ends at the minimal ratio; no branch can overflow max_int
    rnd = random.Random(5)
    for _ in range(200):
        n = rnd.randint(2, 4)
        h = [rnd.randint(50000, 500000) for _ in range(n)]
        ry = [Fraction(rnd.randint(1000, 9000), 7) for _ in range(n)]
        params, r_min = K.sync_concat(h, ry)
        own_v = [r * Fraction(127, hh) for r, hh in zip(ry, h)]
        assert abs(r_min / min(own_v) - 1) < Fraction(1, 1000)
        hit = 0
        for (m, s, bq), hh, r in zip(params, h, ry):
            assert abs(r * m / (1 << s) / r_min - 1) <= Fraction(1, 1 << 14)
            assert 1 <= bq <= 127 and O.requant(hh, m, s) >= bq
            hit += bq == 127
        assert hit >= 1                                  # the widest branch keeps the full range


def test_network_shapes_and_mac_counts():
    r50 = W.resnet50()
    convs = W.conv_ops(r50)
    assert len(convs) == 54 and sum(c["role"] == "projection" for c in convs) == 4
    assert sum(c["res_mode"] == "pre" for c in convs) == 16
    assert abs(W.conv_macs(r50) / 64 / 1e9 - 4.09) < 0.03          # ~4.09 GMAC per image
    assert r50["buffers"]["logits"]["shape"] == [64, 1, 1, 1000]
    r152 = W.resnet152()
    assert len(W.conv_ops(r152)) == 156
    assert sum(c["res_mode"] == "pre" for c in W.conv_ops(r152)) == 50
    assert abs(W.conv_macs(r152) / 128 / 1e9 - 11.5) < 0.1
    v = W.vdsr()
    assert len(W.conv_ops(v)) == 20 and v["buffers"]["out"]["shape"] == [1, 256, 256, 1]
    c = W.vrcnn()
    assert [o["cout"] for o in W.conv_ops(c)] == [64, 32, 16, 16, 32, 1]
    assert c["buffers"]["a2"]["shape"] == [1, 720, 1280, 48]
    assert W.conv_macs(c) // (720 * 1280) == 70896                 # MACs per pixel
    r18 = W.resnet18()
    convs = W.conv_ops(r18)
    assert len(convs) == 21 and sum(c["role"] == "projection" for c in convs) == 3
    assert sum(c["res_mode"] == "pre" for c in convs) == 8
    assert abs(W.conv_macs(r18) / 64 / 1e9 - 1.81) < 0.02            # ~1.81 GMAC per image
    big = W.vrcnn_2560x1600()
    assert big["buffers"]["out"]["shape"] == [1, 1600, 2560, 1]
    assert W.conv_macs(big) // (1600 * 2560) == 70896


def test_cfg0_calibration_reproduces_stored_integers_and_hits_the_bound_rarely():
    net = W.CONFIGS["cfg0"]()
    calib, bufs = ONet.calibrate(net, 0)
    stored = json.load(open(ONet.stored_calib_path("cfg0", 0)))
    assert stored["conv"] == calib["conv"]
    out = bufs["out"]
    assert out.max() == 127 and out.min() == 0
    frac = float((out == 127).mean())
    assert 0.0005 < frac < 0.002                                   # ~0.1 % by construction
    rerun = ONet.run(net, 0, calib)
    assert (rerun["out"] == out).all()


@pytest.mark.parametrize("seed", [0, 1])
def test_small_vrcnn_calibration_and_concat_branches(seed):
    net = W.vrcnn(24, 32)
    calib, bufs = ONet.calibrate(net, seed)
    a2 = bufs["a2"]
    ca, cb = calib["conv"]["conv2a"], calib["conv"]["conv2b"]
    assert max(ca["bound_q"], cb["bound_q"]) == 127
    assert a2[..., :32].max() <= ca["bound_q"] and a2[..., 32:].max() <= cb["bound_q"]
    assert bufs["out"].shape == (1, 24, 32, 1)
    again = ONet.run(net, seed, calib)
    for k in bufs:
        assert (again[k] == bufs[k]).all(), k


def test_small_resnet_runs_and_merges():
    net = W.resnet(2, [1, 1, 1, 1], "tiny", image=32, calib_images=2, classes=10)
    calib, bufs = ONet.calibrate(net, 0)
    assert bufs["logits"].shape == (2, 1, 1, 10) and bufs["logits"].dtype == np.int32
    assert bufs["s1b0_sk"].dtype == np.int32
    one = ONet.run(net, 0, calib, images=1)               # images are independent
    assert (one["logits"][0] == bufs["logits"][0]).all()


def test_bound_parameters_for_other_activation_bit_depths():
    """Section 3.3's post-condition [h_ri * mul / 2^shift] = max_int for the bit-depths of the paper's
    table (8, 6, 5, 4 bits), and a small VDSR calibrated at each reaches exactly that maximum."""
    g = np.random.default_rng(5)
    for max_int in (255, 63, 31, 15):
        hs = list(range(1, 3000)) + [int(v) for v in g.integers(3000, 1 << 24, size=1500)]
        for h in hs:
            m, s = K.bound_params(h, max_int)
            assert O.requant(h, m, s) == max_int and 1 <= m < (1 << 31) and 0 <= s <= K.MAX_SHIFT
        net = W.vdsr(24, 28, depth=4)
        calib, bufs = ONet.calibrate(net, 0, max_int=max_int)
        assert calib["max_int"] == max_int
        assert all(c.get("bound_q", max_int) == max_int for c in calib["conv"].values())
        assert max(int(bufs[n].max()) for n in ("a1", "a2", "a3")) == max_int
