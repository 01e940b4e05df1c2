"""GPU parity on whole synthetic networks: every stored buffer of every layer must
equal the oracle's, so compensating errors cannot hide."""
import json
import os

import numpy as np
import torch
import pytest

from oracle import net as ONet
from workloads import nets as W

pytestmark = pytest.mark.gpu


def compare_all(net, gpu, want):
    for name in net["buffers"]:
        if name in gpu.fused:            # int32 skip tensor of a fused block: never materialised
            continue
        got = gpu.result(name)
        assert got.shape == want[name].shape, name
        assert (got == want[name]).all(), "buffer %s differs at %d elements" % (
            name, int((got != want[name]).sum()))


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_small_vdsr_vrcnn_resnet(seed):
    from paper_2006_11735_amd.netrun import GpuNet
    for net in (W.vdsr(40, 52, depth=5), W.vrcnn(36, 44),
                W.resnet(3, [2, 1, 1, 1], "tiny", image=64, calib_images=2, classes=10)):
        calib, _ = ONet.calibrate(net, seed)
        want = ONet.run(net, seed, calib)
        for fuse in (False, True):
            g = GpuNet(net, seed, calib, fuse=fuse)
            assert bool(g.fused) == (fuse and net["name"] == "tiny")
            assert bool(g.fused_block) == (fuse and net["name"] == "tiny")
            g.set_input()
            g.run()
            compare_all(net, g, want)


@pytest.mark.parametrize("seed", [0, 1])
def test_small_resnet_with_per_channel_requantisation(seed):
    # Section 3.4.3: every output channel its own (mul, shift) and skip rescale
    from paper_2006_11735_amd.netrun import GpuNet
    net = W.resnet(3, [2, 1, 1, 1], "tiny", image=64, calib_images=2, classes=10)
    calib, _ = ONet.calibrate(net, seed, per_channel=True)
    assert "mul_c" in calib["conv"]["stem"] and "res_mul_c" in calib["conv"]["s1b0_c3"]
    want = ONet.run(net, seed, calib)
    for fuse in (False, True):
        g = GpuNet(net, seed, calib, fuse=fuse)
        assert any(st[0] == "conv_pc" for st in g.steps)
        assert any(st[0] == "dual_pc" for st in g.steps) == fuse      # the block whose sum provably fits int32
        g.set_input()
        g.run()
        compare_all(net, g, want)


def test_resnet50_shape_per_channel_batch_8():
    from paper_2006_11735_amd.netrun import GpuNet
    net = W.resnet(8, [3, 4, 6, 3], "r50b8", calib_images=2)
    calib, _ = ONet.calibrate(net, 0, per_channel=True)
    g = GpuNet(net, 0, calib)
    g.set_input()
    g.run()
    x = W.input_tensor(net, 0)
    for img in (0, 5):
        want = ONet.run(net, 0, calib, images=1, x_raw=np.ascontiguousarray(x[img:img + 1]))
        for name in net["buffers"]:
            if name in g.fused:
                continue
            got = g.result(name)[img:img + 1]
            assert (got == want[name]).all(), (img, name)


@pytest.mark.parametrize("floor_channels", ["layer", "own"])
def test_config3_per_channel_full_batch_sampled_images(floor_channels):
    # both stored per-channel calibrations: channels without a positive calibration value keep the layer's pair, or
    # get the wide pair of their own statistic (which only the epilogue's general form takes)
    from paper_2006_11735_amd.netrun import GpuNet
    net = W.CONFIGS["cfg3"]()
    calib = json.load(open(ONet.stored_calib_path("cfg3", 0, per_channel=True, floor_channels=floor_channels)))
    g = GpuNet(net, 0, calib)
    g.set_input()
    g.run()
    x = W.input_tensor(net, 0)
    for img in (1, 62):
        want = ONet.run(net, 0, calib, images=1, x_raw=np.ascontiguousarray(x[img:img + 1]))
        for name in net["buffers"]:
            if name in g.fused:
                continue
            got = g.result(name)[img:img + 1]
            assert (got == want[name]).all(), (img, name)
    assert len(g.fused_proj) == 4 and not g.fused_block       # per-channel layers are not taken by the block kernel


def stored(cfg):
    return json.load(open(ONet.stored_calib_path(cfg, 0)))


def test_config1_vdsr_full_size():
    from paper_2006_11735_amd.netrun import GpuNet
    net, calib = W.CONFIGS["cfg1"](), stored("cfg1")
    want = ONet.run(net, 0, calib)
    g = GpuNet(net, 0, calib)
    g.set_input()
    g.run()
    compare_all(net, g, want)


def test_config2_vrcnn_full_size():
    from paper_2006_11735_amd.netrun import GpuNet
    net, calib = W.CONFIGS["cfg2"](), stored("cfg2")
    want = ONet.run(net, 0, calib)
    g = GpuNet(net, 0, calib)
    g.set_input()
    g.run()
    compare_all(net, g, want)
    ca, cb = calib["conv"]["conv2a"], calib["conv"]["conv2b"]
    a2 = g.result("a2")
    assert a2[..., :32].max() <= ca["bound_q"] and a2[..., 32:].max() <= cb["bound_q"]


def test_config3_resnet50_full_batch_sampled_images():
    # The GPU runs the full batch of 64 in the launch configuration the benchmark times;
    # images are independent, so the oracle checks a sample of them layer by layer.
    from paper_2006_11735_amd.netrun import GpuNet
    net, calib = W.CONFIGS["cfg3"](), stored("cfg3")
    g = GpuNet(net, 0, calib)
    g.set_input()
    g.run()
    x = W.input_tensor(net, 0)
    for img in (0, 37, 63):
        want = ONet.run(net, 0, calib, images=1, x_raw=np.ascontiguousarray(x[img:img + 1]))
        for name in net["buffers"]:
            if name in g.fused:
                continue
            got = g.buf[name][img:img + 1].cpu().numpy()
            assert (got == want[name]).all(), (img, name)
    # the first layer with its pool, four projection blocks and the five identity blocks of stages 1 and 2 run as
    # single launches
    assert len(g.fused_proj) == 4 and len(g.fused_block) == 5 and len(g.fused_pool) == 1 and len(g.fused) == 4 + 2 * 5 + 1 + 2
    assert len(g.fused_projblock) == 1     # stage 1's opening block: stride 1, 64 -> 64 -> 64 -> 256
    assert len(g.fused_pair) == 4          # stage 3: blocks 1..5 share four block boundaries
    logits = g.result("logits")
    assert logits.dtype == np.int32 and logits.shape == (64, 1, 1, 1000)


@pytest.mark.parametrize("max_int", [255, 63, 15])
def test_small_nets_at_other_activation_bit_depths(max_int):
    # the paper's bit-depth table: 8-, 6- and 4-bit activations (255 needs the full-range unsigned input kind)
    from paper_2006_11735_amd.netrun import GpuNet
    for net in (W.vdsr(40, 52, depth=5), W.vrcnn(36, 44),
                W.resnet(3, [2, 1, 1, 1], "tiny", image=64, calib_images=2, classes=10)):
        calib, _ = ONet.calibrate(net, 1, max_int=max_int)
        want = ONet.run(net, 1, calib)
        top = max(int(want[name].max()) for name, b in net["buffers"].items() if b["dtype"] == "u8" and name not in ("raw", "out"))
        assert top == max_int
        g = GpuNet(net, 1, calib)
        g.set_input()
        g.run()
        compare_all(net, g, want)


def test_config1_vdsr_with_8_bit_activations():
    from paper_2006_11735_amd.netrun import GpuNet
    net = W.CONFIGS["cfg1"]()
    calib = json.load(open(ONet.stored_calib_path("cfg1", 0, max_int=255)))
    assert calib["max_int"] == 255
    want = ONet.run(net, 0, calib)
    g = GpuNet(net, 0, calib)
    g.set_input()
    g.run()
    compare_all(net, g, want)
    assert want["a5"].max() == 255


@pytest.mark.parametrize("per_channel", [False, True])
def test_converted_float_networks(per_channel):
    """Networks produced by the offline float -> integer conversion (real weight distributions, folded
    batch norms, synchronised ratios): the library's result equals the oracle's bit for bit, and both
    track the float network."""
    from paper_2006_11735_amd import convert as C
    from paper_2006_11735_amd.netrun import GpuNet
    from test_convert import float_params
    for net, bn in ((W.vdsr(40, 52, depth=5), False), (W.vrcnn(36, 44), False),
                    (W.resnet(4, [2, 1, 1, 1], "tiny", image=64, calib_images=4, classes=10), True),
                    (W.resnet_basic(2, [1, 1, 1, 1], "tiny18", image=64, calib_images=2, classes=10), True)):
        raw = W.input_tensor(net, 3)
        calib, weights, info = C.convert(net, float_params(net, 5, bn), raw, per_channel=per_channel)
        want = ONet.run(net, 0, calib, x_raw=raw, weights=weights)
        g = GpuNet(net, 0, calib, weights=weights)
        g.set_input(raw)
        g.run()
        compare_all(net, g, want)
        out = net["outputs"][0]
        r = info["ratio"][out]
        err = np.abs(g.result(out).astype(np.float64) / r - info["float"][out])
        assert err.mean() < 0.02 * np.abs(info["float"][out]).max()


def test_config5_resnet18_full_batch_sampled_images():
    # basic blocks: 3x3 convs with the skip merge in their epilogue, int32 projections unfused
    from paper_2006_11735_amd.netrun import GpuNet
    net, calib = W.CONFIGS["cfg5"](), stored("cfg5")
    g = GpuNet(net, 0, calib)
    g.set_input()
    g.run()
    x = W.input_tensor(net, 0)
    for img in (3, 60):
        want = ONet.run(net, 0, calib, images=1, x_raw=np.ascontiguousarray(x[img:img + 1]))
        for name in net["buffers"]:
            if name in g.fused:
                continue
            got = g.buf[name][img:img + 1].cpu().numpy()
            assert (got == want[name]).all(), (img, name)
    # only the first layer's output stays on chip (fused with its max-pool)
    assert len(g.fused_pool) == 1 and len(g.fused) == 1 and not g.fused_block and not g.fused_proj


def test_config6_vrcnn_2560x1600_frame():
    # the picture size the paper times VRCNN on; every layer of the whole frame is compared
    from paper_2006_11735_amd.netrun import GpuNet
    net, calib = W.CONFIGS["cfg6"](), stored("cfg6")
    g = GpuNet(net, 0, calib)
    g.set_input()
    g.run()
    want = ONet.run(net, 0, calib)
    compare_all(net, g, want)


def test_config4_resnet152_full_batch_sampled_images():
    # ResNet-152-shaped at its full batch of 128, i.e. the tile choices, persistent grids and pixel counts of the
    # launch configuration that is timed; images are independent, so the oracle checks a sample of them on every
    # buffer of every layer (about 12 GMAC per image).
    from paper_2006_11735_amd.netrun import GpuNet
    net, calib = W.CONFIGS["cfg4"](), stored("cfg4")
    g = GpuNet(net, 0, calib)
    assert g.images == 128
    g.set_input()
    g.run()
    x = W.input_tensor(net, 0)
    for img in (0, 77, 127):
        want = ONet.run(net, 0, calib, images=1, x_raw=np.ascontiguousarray(x[img:img + 1]))
        for name in net["buffers"]:
            if name in g.fused:
                continue
            got = g.buf[name][img:img + 1].cpu().numpy()
            assert (got == want[name]).all(), (img, name)
    assert len(g.fused_proj) == 4 and len(g.fused_block) == 2 + 7
    assert g.result("logits").shape == (128, 1, 1, 1000)


def test_two_steps_in_flight_on_two_streams():
    # two instances of the same network (own activation buffers, own copies of the weights) issued alternately on
    # two streams: the library keeps no per-call state that concurrent launches could share, so both must reproduce
    # the one-stream result
    from paper_2006_11735_amd.netrun import GpuNet
    net, calib = W.CONFIGS["cfg5"](), stored("cfg5")
    nets = [GpuNet(net, 0, calib, images=16) for _ in range(2)]
    for g in nets:
        g.set_input()
    nets[0].run()
    torch.cuda.synchronize()
    ref = {k: v.clone() for k, v in nets[0].buf.items() if k not in nets[0].fused}
    for g in nets:
        for k, v in g.buf.items():
            if k != net["input"] and k not in g.fused:
                v.zero_()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for i in range(6):
        with torch.cuda.stream(streams[i & 1]):
            nets[i & 1].run()
    torch.cuda.synchronize()
    for g in nets:
        for k, v in ref.items():
            assert torch.equal(v, g.buf[k]), k
