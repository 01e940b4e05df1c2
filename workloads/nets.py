"""Shapes of the five synthetic workloads: one integer conv layer, and VDSR-,
VRCNN-, ResNet-50- and ResNet-152-shaped integer networks.

A network is a plain dict:
    {"name", "input": buffer name, "buffers": {name: {"shape": [N,H,W,C], "dtype"}},
     "ops": [op, ...], "outputs": [buffer names], "calib_images": int}
Every op is a dict with "op" in {"conv", "maxpool", "avgpool"}.  A conv op
names its source and destination buffers, its geometry, how its result is
written (channel offset inside the destination, for concatenation) and which
buffer, if any, is merged in as a skip operand.  The per-layer integers
(mul, shift, bound, skip multiplier...) are not here: calibration produces
them from a run over the calibration images.

Only topology and sizes live in this file; it performs no arithmetic on
tensor values.
"""
import numpy as np

from .rng import uniform_int

# value ranges of the synthetic tensors
ACT_MAX = 127            # quantised BReLU bound of every stored activation
W_ABS_MAX = 127          # weights lie in [-127, 127]
BIAS_ABS_MAX = 1 << 12   # biases lie in [-4096, 4096]


def _out_hw(h, w, k, s, p):
    return (h + 2 * p - k) // s + 1, (w + 2 * p - k) // s + 1


class _Builder:
    def __init__(self, name, n, h, w, c, calib_images):
        self.net = {"name": name, "input": "raw", "buffers": {}, "ops": [],
                    "outputs": [], "calib_images": calib_images}
        self.net["buffers"]["raw"] = {"shape": [n, h, w, c], "dtype": "u8"}
        self.nconv = 0

    def buf(self, name, shape, dtype="u8"):
        b = self.net["buffers"]
        if name in b:
            assert b[name]["shape"] == list(shape) and b[name]["dtype"] == dtype, name
        else:
            b[name] = {"shape": list(shape), "dtype": dtype}

    def shape(self, name):
        return self.net["buffers"][name]["shape"]

    def conv(self, name, src, dst, cout, k, stride=1, pad=None, src_c=None,
             in_sub128=False, out_mode="brelu", res=None, res_mode="none",
             dst_c_total=None, dst_c_offset=0, group=None, role=None):
        n, h, w, c_buf = self.shape(src)
        cin = c_buf if src_c is None else src_c
        if pad is None:
            pad = k // 2
        ho, wo = _out_hw(h, w, k, stride, pad)
        ctot = cout if dst_c_total is None else dst_c_total
        self.buf(dst, [n, ho, wo, ctot], "s32" if out_mode == "raw_s32" else "u8")
        res_dtype = None
        if res is not None:
            res_dtype = self.net["buffers"][res]["dtype"]
            assert self.shape(res)[:3] == [n, ho, wo] and self.shape(res)[3] == cout
        self.net["ops"].append({
            "op": "conv", "name": name, "idx": self.nconv, "src": src, "dst": dst,
            "cin": cin, "cout": cout, "kh": k, "kw": k, "stride": stride, "pad": pad,
            "in_sub128": bool(in_sub128), "out_mode": out_mode,
            "res": res, "res_mode": res_mode, "res_dtype": res_dtype,
            "dst_c_offset": dst_c_offset, "group": group, "role": role})
        self.nconv += 1
        return dst

    def maxpool(self, src, dst, k=3, stride=2, pad=1):
        n, h, w, c = self.shape(src)
        ho, wo = _out_hw(h, w, k, stride, pad)
        self.buf(dst, [n, ho, wo, c])
        self.net["ops"].append({"op": "maxpool", "src": src, "dst": dst, "k": k,
                                "stride": stride, "pad": pad})
        return dst

    def avgpool(self, src, dst):
        n, h, w, c = self.shape(src)
        self.buf(dst, [n, 1, 1, c])
        self.net["ops"].append({"op": "avgpool", "src": src, "dst": dst})
        return dst


def single_conv(n=1, h=56, w=56, cin=64, cout=64, k=3, stride=1, pad=1):
    """Config 0: one integer conv layer with a fused BReLU epilogue."""
    b = _Builder("conv%dx%d_%dx%dx%dx%d_%d" % (k, k, n, h, w, cin, cout), n, h, w, cin, n)
    b.net["input_range"] = [0, ACT_MAX]
    b.conv("conv", "raw", "out", cout, k, stride, pad)
    b.net["outputs"] = ["out"]
    return b.net


def vdsr(h=256, w=256, depth=20, width=64):
    """Config 1: `depth` conv3x3 layers on one luma plane, first layer re-normalises
    the raw picture, last layer adds the raw picture back (regression output)."""
    b = _Builder("vdsr_%dx%d" % (h, w), 1, h, w, 1, 1)
    b.net["input_range"] = [0, 255]
    cur = b.conv("conv1", "raw", "a1", width, 3, in_sub128=True)
    for i in range(2, depth):
        cur = b.conv("conv%d" % i, cur, "a%d" % i, width, 3)
    b.conv("conv%d" % depth, cur, "out", 1, 3, out_mode="clamp_u8", res="raw",
           res_mode="post", role="regression_out")
    b.net["outputs"] = ["out"]
    return b.net


def vrcnn(h=720, w=1280):
    """Config 2: four conv layers, the middle two made of two branches with
    different kernel sizes whose outputs share one buffer (concatenation)."""
    b = _Builder("vrcnn_%dx%d" % (h, w), 1, h, w, 1, 1)
    b.net["input_range"] = [0, 255]
    b.conv("conv1", "raw", "a1", 64, 5, in_sub128=True)
    b.conv("conv2a", "a1", "a2", 32, 5, dst_c_total=48, dst_c_offset=0, group="cat2")
    b.conv("conv2b", "a1", "a2", 16, 3, dst_c_total=48, dst_c_offset=32, group="cat2")
    b.conv("conv3a", "a2", "a3", 16, 3, dst_c_total=48, dst_c_offset=0, group="cat3")
    b.conv("conv3b", "a2", "a3", 32, 1, dst_c_total=48, dst_c_offset=16, group="cat3")
    b.conv("conv4", "a3", "out", 1, 3, out_mode="clamp_u8", res="raw",
           res_mode="post", role="regression_out")
    b.net["outputs"] = ["out"]
    return b.net


def resnet(batch, blocks, name, image=224, calib_images=4, classes=1000):
    """Configs 3 and 4: bottleneck ResNet.  Stem conv7x7/2 + max-pool, four stages
    of 1x1 / 3x3 / 1x1 blocks (stride 2 on the 3x3 of each later stage's first
    block and on its projection), a skip merge per block (identity: the stored
    8-bit block input; projection: an int32 1x1 conv of it), global average
    pool, and a fully connected layer that emits raw int32 logits."""
    b = _Builder(name, batch, image, image, 3, min(calib_images, batch))
    b.net["input_range"] = [0, 255]
    b.conv("stem", "raw", "stem", 64, 7, stride=2, pad=3, in_sub128=True)
    cur = b.maxpool("stem", "pool0")
    widths = [64, 128, 256, 512]
    for si, (nb, wd) in enumerate(zip(blocks, widths)):
        for bi in range(nb):
            p = "s%db%d" % (si + 1, bi)
            stride = 2 if (bi == 0 and si > 0) else 1
            b.conv(p + "_c1", cur, p + "_a1", wd, 1)
            b.conv(p + "_c2", p + "_a1", p + "_a2", wd, 3, stride=stride)
            if bi == 0:
                b.conv(p + "_proj", cur, p + "_sk", 4 * wd, 1, stride=stride, pad=0,
                       out_mode="raw_s32", role="projection")
                skip = p + "_sk"
            else:
                skip = cur
            cur = b.conv(p + "_c3", p + "_a2", p + "_out", 4 * wd, 1, res=skip, res_mode="pre")
    cur = b.avgpool(cur, "gap")
    b.conv("fc", cur, "logits", classes, 1, pad=0, out_mode="raw_s32", role="logits")
    b.net["outputs"] = ["logits"]
    return b.net


def resnet_basic(batch, blocks, name, image=224, calib_images=4, classes=1000):
    """Basic-block ResNet (the block of the paper's residual figure, Section 4.1): stem and pools as
    in `resnet`, four stages of two 3x3 convs per block, the skip joining the second one before
    BReLU (identity: the stored 8-bit block input; first block of stages 2-4: an int32 1x1/2
    projection of it)."""
    b = _Builder(name, batch, image, image, 3, min(calib_images, batch))
    b.net["input_range"] = [0, 255]
    b.conv("stem", "raw", "stem", 64, 7, stride=2, pad=3, in_sub128=True)
    cur = b.maxpool("stem", "pool0")
    widths = [64, 128, 256, 512]
    for si, (nb, wd) in enumerate(zip(blocks, widths)):
        for bi in range(nb):
            p = "s%db%d" % (si + 1, bi)
            stride = 2 if (bi == 0 and si > 0) else 1
            b.conv(p + "_c1", cur, p + "_a1", wd, 3, stride=stride)
            if bi == 0 and si > 0:
                b.conv(p + "_proj", cur, p + "_sk", wd, 1, stride=stride, pad=0,
                       out_mode="raw_s32", role="projection")
                skip = p + "_sk"
            else:
                skip = cur
            cur = b.conv(p + "_c2", p + "_a1", p + "_out", wd, 3, res=skip, res_mode="pre")
    cur = b.avgpool(cur, "gap")
    b.conv("fc", cur, "logits", classes, 1, pad=0, out_mode="raw_s32", role="logits")
    b.net["outputs"] = ["logits"]
    return b.net


def resnet18(batch=64, **kw):
    return resnet_basic(batch, [2, 2, 2, 2], "resnet18_b%d" % batch, **kw)


def vrcnn_2560x1600():
    """The one 2560x1600 picture the paper times VRCNN on (its Table 6)."""
    return vrcnn(1600, 2560)


def resnet50(batch=64, **kw):
    return resnet(batch, [3, 4, 6, 3], "resnet50_b%d" % batch, **kw)


def resnet152(batch=128, **kw):
    return resnet(batch, [3, 8, 36, 3], "resnet152_b%d" % batch, **kw)


CONFIGS = {
    "cfg0": single_conv,
    "cfg1": vdsr,
    "cfg2": vrcnn,
    "cfg3": resnet50,
    "cfg4": resnet152,
    "cfg5": resnet18,             # second workloads: basic-block ResNet, batch 64
    "cfg6": vrcnn_2560x1600,      # and the large VRCNN frame
}


def conv_ops(net):
    return [op for op in net["ops"] if op["op"] == "conv"]


def conv_macs(net):
    """Multiply-accumulates of all conv ops (true, unpadded sizes)."""
    total = 0
    for op in conv_ops(net):
        n, ho, wo, _ = net["buffers"][op["dst"]]["shape"]
        total += n * ho * wo * op["cout"] * op["kh"] * op["kw"] * op["cin"]
    return total


# ---- seeded tensors -------------------------------------------------------
# tensor ids: 0 = network input, 4*idx+1 = weights of conv idx, 4*idx+2 = its
# bias, 4*idx+3 = its synthetic float weight magnitude (calibration of
# concatenated branches only).

def input_tensor(net, seed, images=None):
    """Raw network input, uint8 NHWC.  `images` limits it to the first images
    (element indices are unchanged, so it is a prefix of the full tensor)."""
    n, h, w, c = net["buffers"]["raw"]["shape"]
    if images is not None:
        n = min(n, images)
    lo, hi = net["input_range"]
    return uniform_int(seed, 0, n * h * w * c, lo, hi, np.uint8).reshape(n, h, w, c)


def weight_tensor(op, seed):
    """int8 weights [cout][kh][kw][cin] of a conv op."""
    shape = (op["cout"], op["kh"], op["kw"], op["cin"])
    cnt = int(np.prod(shape))
    return uniform_int(seed, 4 * op["idx"] + 1, cnt, -W_ABS_MAX, W_ABS_MAX, np.int8).reshape(shape)


def bias_tensor(op, seed):
    """int32 bias [cout] of a conv op."""
    return uniform_int(seed, 4 * op["idx"] + 2, op["cout"], -BIAS_ABS_MAX, BIAS_ABS_MAX, np.int32)


def float_weight_absmax(op, seed):
    """Synthetic max|W_f| of the float kernel a conv stands for, in [0.050, 0.500];
    only its ratio between concatenated branches matters."""
    r = uniform_int(seed, 4 * op["idx"] + 3, 1, 50, 500, np.int64)[0]
    return float(r) / 1000.0
