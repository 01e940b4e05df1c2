"""Runs a synthetic integer network (workloads.nets) on the GPU through the C
boundary.  This is harness code: it owns the device buffers (torch tensors),
prepacks the weights once, and then issues one library call per layer.  All
arithmetic happens inside the library.
"""
import numpy as np
import torch

from workloads import nets as W
from . import binding as B

_OUT = {"brelu": B.ICNN_OUT_BRELU_U8, "clamp_u8": B.ICNN_OUT_CLAMP_U8,
        "linear_s8": B.ICNN_OUT_LINEAR_S8, "raw_s32": B.ICNN_OUT_RAW_S32}
_RES = {"none": B.ICNN_RES_NONE, "pre": B.ICNN_RES_PRE, "post": B.ICNN_RES_POST}
_DT = {"u8": B.ICNN_U8, "s8": B.ICNN_S8, "s32": B.ICNN_S32}


class GpuNet:
    def __init__(self, net, seed, calib, images=None, device="cuda:0", fuse=True, weights=None, fuse_blocks=None):
        """fuse: run a projection conv and the block's last conv that consumes it as one
        iconv2d_dual_brelu launch where the library accepts that (the int32 skip buffer then
        stays untouched).  fuse_blocks (default: as fuse): run an identity bottleneck block (1x1, 3x3, 1x1 with
        the block input as skip operand) as one iconv2d_bottleneck_brelu launch where the library accepts
        that (its two middle buffers then stay untouched).  weights: optional {layer: (int8 [cout,kh,kw,cin], int32 [cout])}, e.g.
        from paper_2006_11735_amd.convert, instead of the seeded synthetic tensors."""
        self.weights = weights
        if not torch.cuda.is_available():
            raise RuntimeError("GpuNet needs a GPU: there is no CPU fallback")
        self.net, self.seed, self.calib = net, seed, calib
        self.device = torch.device(device)
        n_full = net["buffers"]["raw"]["shape"][0]
        self.images = n_full if images is None else min(images, n_full)
        self.buf = {}
        for name, b in net["buffers"].items():
            shape = [self.images] + b["shape"][1:]
            dt = torch.int32 if b["dtype"] == "s32" else torch.uint8
            self.buf[name] = torch.zeros(shape, dtype=dt, device=self.device)
        self.steps = []
        self.fused = []                     # names of int32 skip buffers that are never written
        self.fused_proj = {}                # main conv name -> the projection op fused into it
        self.fused_block = {}               # last conv name -> (first, middle) conv ops fused into its launch
        self.fused_pool = {}                # first conv name -> the max-pool op fused into its launch
        self.fused_pair = {}                # block-closing conv name -> the next block's opening conv op in its launch
        self.fused_twin = {}                # branch name -> the other branch's op in its launch
        self.fused_projblock = {}           # last conv name -> (first, middle, projection) conv ops fused into its launch
        pending = {}                        # skip buffer name -> prepared projection step
        for op in net["ops"]:
            if op["op"] == "conv":
                step = self._prep_conv(op)
                if fuse and op["role"] == "projection" and op["out_mode"] == "raw_s32":
                    pending[op["dst"]] = step
                    continue
                if op["res"] in pending:
                    proj = pending.pop(op["res"])
                    dual = self._try_fuse(step, proj)
                    if dual is not None:
                        self.fused.append(op["res"])
                        self.fused_proj[op["name"]] = proj[1]
                        self.steps.append(dual)
                        continue
                    self.steps.append(proj)
                self.steps.append(step)
            elif op["op"] == "maxpool":
                n, h, w, c = self.buf[op["src"]].shape
                args = (n, h, w, c, op["k"], op["stride"], op["pad"], self.buf[op["src"]], self.buf[op["dst"]])
                self.steps.append(("maxpool", op, args))
            elif op["op"] == "avgpool":
                n, h, w, c = self.buf[op["src"]].shape
                cal = calib["avgpool"][op["dst"]]
                args = (n, h, w, c, cal["mul"], cal["shift"], cal["bound_q"], self.buf[op["src"]],
                        self.buf[op["dst"]])
                self.steps.append(("avgpool", op, args))
            else:
                raise ValueError(op["op"])
        if fuse if fuse_blocks is None else fuse_blocks:
            self._fuse_blocks()
            self._fuse_projection_blocks()
            self._fuse_first_layer()
            self._fuse_pairs()
            self._fuse_twins()
        torch.cuda.synchronize(self.device)

    def _fuse_first_layer(self):
        """A picture convolution followed by the max-pool of its output, nothing else reading that output: one
        iconv2d_maxpool_brelu launch where the library accepts it (the convolution's buffer then stays untouched)."""
        readers = {}
        for op in self.net["ops"]:
            readers.setdefault(op["src"], []).append(op)
            if op.get("res") is not None:
                readers.setdefault(op["res"], []).append(op)
        steps, i = [], 0
        while i < len(self.steps):
            pair = self.steps[i:i + 2]
            if len(pair) == 2 and pair[0][0] == "conv" and pair[1][0] == "maxpool":
                oc, op_ = pair[0][1], pair[1][1]
                if op_["src"] == oc["dst"] and readers.get(oc["dst"]) == [op_] and oc["dst"] not in self.net["outputs"]:
                    d, x, wp, bias, _res, _y, _ws = pair[0][2]
                    dd = B.conv_desc(**{k: getattr(d, k) for k, _ in d._fields_})
                    pooled = self.buf[op_["dst"]]
                    dd.out_c_stride, dd.out_c_offset = pooled.shape[3], 0
                    args = (dd, op_["k"], op_["stride"], op_["pad"], x, wp, bias, pooled)
                    try:
                        B.iconv2d_maxpool_brelu(*args)
                    except B.IcnnError as e:
                        if e.code != B.ICNN_E_UNSUPPORTED:
                            raise
                    else:
                        self.fused.append(oc["dst"])
                        self.fused_pool[oc["name"]] = op_
                        steps.append(("convpool", oc, args))
                        i += 2
                        continue
            steps.append(self.steps[i])
            i += 1
        self.steps = steps

    # The fused pair streams both layers' weights through every workgroup's 64-pixel tile: it wins where the tiles
    # fit the chip in about one round and the wide tensor is at most 1024 channels (measured at batch 64: 17.6 us
    # against 23.8 us for 12544 pixels of 256 -> 1024 -> 256; level at 50176 pixels of 128 -> 512 -> 128; a loss,
    # 22.9 us against 19.0 us, at 3136 pixels of 512 -> 2048 -> 512).
    PAIR_MAX_PIXELS = 64 * 512
    PAIR_MAX_WIDE = 1024

    def _fuse_pairs(self):
        """The 1x1 convolution that closes a block followed by the 1x1 convolution that opens the next one: one
        iconv2d_pair_brelu launch where the library accepts it and the shape is one the fused kernel wins on.  Both
        outputs are still written (the first is the next block's skip operand)."""
        steps, i = [], 0
        while i < len(self.steps):
            two = self.steps[i:i + 2]
            if len(two) == 2 and two[0][0] == "conv" and two[1][0] == "conv":
                o3, o1 = two[0][1], two[1][1]
                (d3, t, w3, b3, res, y, _ws3), (d1, _y, w1, b1, _r1, z, _ws1) = two[0][2], two[1][2]
                if (o1["src"] == o3["dst"] and o3["kh"] == 1 and o1["kh"] == 1 and o3["dst_c_offset"] == 0 and
                        o1["cout"] == o3["cin"] and o1["cin"] == o3["cout"] and
                        d3.n * d3.h * d3.w <= self.PAIR_MAX_PIXELS and o3["cout"] <= self.PAIR_MAX_WIDE):
                    args = (d3, t, w3, b3, res, y, d1, w1, b1, z)
                    try:
                        B.iconv2d_pair_brelu(*args)                # also a warm-up launch
                    except B.IcnnError as e:
                        if e.code != B.ICNN_E_UNSUPPORTED:
                            raise
                    else:
                        self.fused_pair[o3["name"]] = o1
                        steps.append(("pair", o3, args))
                        i += 2
                        continue
            steps.append(self.steps[i])
            i += 1
        self.steps = steps

    # The twin launch reads the input once and writes whole pixels of the shared buffer; below a few tiles per compute
    # unit the two-dimensional-tile kernel it runs on is not the library's own choice for either branch.
    TWIN_MIN_PIXELS = 1024 * 512

    def _fuse_twins(self):
        """Two consecutive convolutions of the same input whose kernels differ by two pixels (the branches of a
        concatenation): one iconv2d_twin_brelu launch where the library accepts it."""
        steps, i = [], 0
        while i < len(self.steps):
            two = self.steps[i:i + 2]
            if len(two) == 2 and two[0][0] == "conv" and two[1][0] == "conv":
                (da, xa, wa, ba, ra, ya, _wsa), (db, xb, wb, bb, rb, yb, _wsb) = two[0][2], two[1][2]
                oa, ob = two[0][1], two[1][1]
                if oa["kh"] < ob["kh"]:
                    (da, wa, ba, ya, oa), (db, wb, bb, yb, ob) = (db, wb, bb, yb, ob), (da, wa, ba, ya, oa)
                if (oa["src"] == ob["src"] and oa["kh"] == ob["kh"] + 2 and ra is None and rb is None and
                        oa["dst"] != oa["src"] and ob["dst"] != ob["src"] and da.n * da.h * da.w >= self.TWIN_MIN_PIXELS):
                    args = (da, xa, wa, ba, ya, db, wb, bb, yb)
                    try:
                        B.iconv2d_twin_brelu(*args)                # also a warm-up launch
                    except B.IcnnError as e:
                        if e.code != B.ICNN_E_UNSUPPORTED:
                            raise
                    else:
                        self.fused_twin[oa["name"]] = ob
                        steps.append(("twin", oa, args))
                        i += 2
                        continue
            steps.append(self.steps[i])
            i += 1
        self.steps = steps

    def _fuse_projection_blocks(self):
        """A stage's opening bottleneck block whose last layer already runs with its projection as one dual step: the
        two layers before it join that launch (iconv2d_bottleneck_dual_brelu) where the library accepts it; the block's
        two middle buffers then stay untouched as well."""
        readers = {}
        for op in self.net["ops"]:
            readers.setdefault(op["src"], []).append(op)
            if op.get("res") is not None:
                readers.setdefault(op["res"], []).append(op)
        steps, i = [], 0
        while i < len(self.steps):
            trio = self.steps[i:i + 3]
            if len(trio) == 3 and trio[0][0] == "conv" and trio[1][0] == "conv" and trio[2][0] == "dual":
                o1, o2, o3 = (st[1] for st in trio)
                proj = self.fused_proj[o3["name"]]
                chain = (o2["src"] == o1["dst"] and o3["src"] == o2["dst"] and proj["src"] == o1["src"] and
                         readers.get(o1["dst"]) == [o2] and readers.get(o2["dst"]) == [o3] and
                         o1["dst"] not in self.net["outputs"] and o2["dst"] not in self.net["outputs"] and
                         o1["dst_c_offset"] == 0 and o2["dst_c_offset"] == 0)
                if chain:
                    (d1, x, w1, b1, _r1, _y1, _ws1), (d2, _x2, w2, b2, _r2, _y2, _ws2) = trio[0][2], trio[1][2]
                    dm, _xm, wm, bm, dp, _xp, wp, bp, y = trio[2][2]
                    args = (d1, x, w1, b1, d2, w2, b2, dm, wm, bm, dp, wp, bp, y)
                    try:
                        B.iconv2d_bottleneck_dual_brelu(*args)     # also a warm-up launch
                    except B.IcnnError as e:
                        if e.code != B.ICNN_E_UNSUPPORTED:
                            raise
                    else:
                        self.fused += [o1["dst"], o2["dst"]]
                        self.fused_projblock[o3["name"]] = (o1, o2, proj)
                        steps.append(("projblock", o3, args))
                        i += 3
                        continue
            steps.append(self.steps[i])
            i += 1
        self.steps = steps

    def _fuse_blocks(self):
        """Replaces every run of three per-layer conv steps that forms an identity bottleneck block by one fused step."""
        readers = {}
        for op in self.net["ops"]:
            readers.setdefault(op["src"], []).append(op)
            if op.get("res") is not None:
                readers.setdefault(op["res"], []).append(op)
        steps, i = [], 0
        while i < len(self.steps):
            trio = self.steps[i:i + 3]
            if len(trio) == 3 and all(st[0] == "conv" for st in trio):
                o1, o2, o3 = (st[1] for st in trio)
                chain = (o2["src"] == o1["dst"] and o3["src"] == o2["dst"] and o3["res"] == o1["src"] and
                         readers.get(o1["dst"]) == [o2] and readers.get(o2["dst"]) == [o3] and
                         o1["dst"] not in self.net["outputs"] and o2["dst"] not in self.net["outputs"] and
                         o1["dst_c_offset"] == 0 and o2["dst_c_offset"] == 0)
                if chain:
                    (d1, x, w1, b1, _r1, _y1, _ws1), (d2, _x2, w2, b2, _r2, _y2, _ws2), (d3, _x3, w3, b3, res, y, _ws3) = (
                        st[2] for st in trio)
                    args = (d1, x, w1, b1, d2, w2, b2, d3, w3, b3, res, y)
                    try:
                        B.iconv2d_bottleneck_brelu(*args)          # also a warm-up launch
                    except B.IcnnError as e:
                        if e.code != B.ICNN_E_UNSUPPORTED:
                            raise
                    else:
                        self.fused += [o1["dst"], o2["dst"]]
                        self.fused_block[o3["name"]] = (o1, o2)
                        steps.append(("block", o3, args))
                        i += 3
                        continue
            steps.append(self.steps[i])
            i += 1
        self.steps = steps

    def _prep_conv(self, op):
        cal = self.calib["conv"][op["name"]]
        src, dst = self.buf[op["src"]], self.buf[op["dst"]]
        n, h, w, cbuf = src.shape
        # bytes above 127 can occur in activations bounded above 127, or in a full-range input that is
        # not re-normalised
        top = self.calib.get("max_int", 127) if op["src"] != self.net["input"] else self.net["input_range"][1]
        in_kind = B.ICNN_IN_U8_FULL if (top > 127 and not op["in_sub128"]) else B.ICNN_IN_U8_LE127
        d = B.conv_desc(
            n=n, h=h, w=w, cin=op["cin"], in_c_stride=cbuf, in_signed=in_kind, in_sub128=int(op["in_sub128"]),
            cout=op["cout"], kh=op["kh"], kw=op["kw"], stride_h=op["stride"], stride_w=op["stride"],
            pad_h=op["pad"], pad_w=op["pad"], out_c_stride=dst.shape[3], out_c_offset=op["dst_c_offset"],
            mul=cal.get("mul", 1), shift=cal.get("shift", 0), bound_q=cal.get("bound_q", 127),
            lo=cal.get("lo", 0), hi=cal.get("hi", 255), out_mode=_OUT[op["out_mode"]],
            res_mode=_RES[op["res_mode"]])
        res = None
        if op["res"] is not None:
            res = self.buf[op["res"]]
            d.res_dtype = _DT[op["res_dtype"]]
            d.res_c_stride = res.shape[3]
            d.res_mul, d.res_shift = cal.get("res_mul", 1), cal.get("res_shift", 0)
        w_np = self.weights[op["name"]][0] if self.weights is not None else W.weight_tensor(op, self.seed)
        w_dev = torch.from_numpy(np.ascontiguousarray(w_np, dtype=np.int8)).to(self.device)
        wp = torch.empty(B.iconv2d_packed_weight_bytes(d), dtype=torch.uint8, device=self.device)
        B.iconv2d_prepack_weights(d, w_dev, wp)
        b_np = self.weights[op["name"]][1] if self.weights is not None else W.bias_tensor(op, self.seed)
        bias = torch.from_numpy(np.ascontiguousarray(b_np, dtype=np.int32)).to(self.device)
        ws_bytes = B.iconv2d_workspace_bytes(d)
        ws = torch.zeros(ws_bytes, dtype=torch.uint8, device=self.device) if ws_bytes else None       # zero-filled once: its counter block
        torch.cuda.synchronize(self.device)       # w_dev may be released after the prepack ran
        if "mul_c" in cal or "res_mul_c" in cal:
            # per-output-channel requantisation: the integers go to the device as they are
            def col(key, fallback):
                v = cal.get(key)
                if v is None:
                    v = [cal.get(fallback[0], fallback[1])] * op["cout"]
                return torch.tensor(v, dtype=torch.int32, device=self.device)
            arrs = [col("mul_c", ("mul", 1)), col("shift_c", ("shift", 0))]
            if res is not None:
                arrs += [col("res_mul_c", ("res_mul", 1)), col("res_shift_c", ("res_shift", 0))]
            pcp = torch.empty(B.iconv2d_packed_channel_params_bytes(d), dtype=torch.uint8, device=self.device)
            B.iconv2d_prepack_channel_params(d, B.channel_params(*arrs), pcp)
            if res is not None:
                # the descriptor's own pair bounds the per-channel skip ratios (what the fused block's
                # overflow proof needs; the plain per-channel call does not read it)
                rm, rs = max(zip(cal["res_mul_c"], cal["res_shift_c"]), key=lambda t: t[0] / 2.0 ** t[1])
                d.res_mul, d.res_shift = rm, rs
            torch.cuda.synchronize(self.device)   # the arrays may be released after the prepack ran
            return ("conv_pc", op, (d, src, wp, bias, pcp, res, dst, ws))
        return ("conv", op, (d, src, wp, bias, res, dst, ws))

    def _try_fuse(self, main, proj):
        if proj[0] != "conv":
            return None
        dp, xp, wp, bp, _r, _sk, _w = proj[2]
        if main[0] == "conv_pc":
            dm, xm, wm, bm, pcp, _res, y, _ws = main[2]
            kind, fn, args = "dual_pc", B.iconv2d_dual_brelu_pc, (dm, xm, wm, bm, pcp, dp, xp, wp, bp, y)
        else:
            dm, xm, wm, bm, _res, y, _ws = main[2]
            kind, fn, args = "dual", B.iconv2d_dual_brelu, (dm, xm, wm, bm, dp, xp, wp, bp, y)
        try:
            fn(*args)                       # also a warm-up launch
        except B.IcnnError as e:
            if e.code == B.ICNN_E_UNSUPPORTED:
                return None
            raise
        return (kind, main[1], args)

    def set_input(self, x_raw=None):
        if x_raw is None:
            x_raw = W.input_tensor(self.net, self.seed, self.images)
        self.buf["raw"].copy_(torch.from_numpy(np.ascontiguousarray(x_raw)).to(self.device))

    def run(self, stream=None):
        for i in range(len(self.steps)):
            self.run_step(i, stream)

    def run_step(self, i, stream=None):
        kind, _, args = self.steps[i]
        if kind == "conv":
            B.iconv2d_brelu(*args, stream=stream)
        elif kind == "conv_pc":
            B.iconv2d_brelu_pc(*args, stream=stream)
        elif kind == "dual":
            B.iconv2d_dual_brelu(*args, stream=stream)
        elif kind == "dual_pc":
            B.iconv2d_dual_brelu_pc(*args, stream=stream)
        elif kind == "pair":
            B.iconv2d_pair_brelu(*args, stream=stream)
        elif kind == "twin":
            B.iconv2d_twin_brelu(*args, stream=stream)
        elif kind == "projblock":
            B.iconv2d_bottleneck_dual_brelu(*args, stream=stream)
        elif kind == "block":
            B.iconv2d_bottleneck_brelu(*args, stream=stream)
        elif kind == "convpool":
            B.iconv2d_maxpool_brelu(*args, stream=stream)
        elif kind == "maxpool":
            B.imaxpool2d_u8(*args, stream=stream)
        else:
            B.iavgpool_global_u8(*args, stream=stream)

    def result(self, name):
        return self.buf[name].cpu().numpy()
