"""Runs a synthetic integer network (workloads.nets) through the CPU oracle, and
calibrates it.  TEST INFRASTRUCTURE (see oracle/icnn_oracle.c).

`calibrate(net, seed)` walks the layers once over the calibration images and
fixes every layer's integers from the statistics it sees (Section 3.3, Section
4.1, Algorithm 2); `run(net, seed, calib)` then evaluates the network with
those integers.  Both return every intermediate buffer so the HIP path can be
compared layer by layer.
"""
from fractions import Fraction

import numpy as np

from workloads import nets as W
from . import calibrate as K
from . import oracle as O

INPUT_RATIO = 256            # raw - 128 stands for a float input in [-0.5, 0.5)
REGRESSION_LEVELS = 32       # 99.9th-percentile |residual| maps to this many pixel levels


def _alloc(net, name, images):
    b = net["buffers"][name]
    shape = [min(b["shape"][0], images)] + b["shape"][1:]
    return np.zeros(shape, dtype=np.int32 if b["dtype"] == "s32" else np.uint8)


def _conv(op, bufs, w, bias, cal, out, out_mode=None, use_res=True):
    om = op["out_mode"] if out_mode is None else out_mode
    kw = dict(stride=op["stride"], pad=op["pad"], in_sub128=op["in_sub128"], cin=op["cin"],
              out_mode=om, mul=cal.get("mul", 1), shift=cal.get("shift", 0),
              bound_q=cal.get("bound_q", K.MAX_INT), lo=cal.get("lo", 0), hi=cal.get("hi", 255))
    if "mul_c" in cal:
        kw.update(mul_c=cal["mul_c"], shift_c=cal["shift_c"])
    if op["res"] is not None and use_res:
        kw.update(res=bufs[op["res"]], res_mode=op["res_mode"],
                  res_mul=cal.get("res_mul", 1), res_shift=cal.get("res_shift", 0))
        if "res_mul_c" in cal:
            kw.update(res_mul_c=cal["res_mul_c"], res_shift_c=cal["res_shift_c"])
    if out is None:
        return O.conv2d(bufs[op["src"]], w, bias, **kw)
    return O.conv2d(bufs[op["src"]], w, bias, out=out, out_c_offset=op["dst_c_offset"], **kw)


def run(net, seed, calib, images=None, x_raw=None, weights=None):
    """Evaluate `net` with stored calibration integers; returns {buffer: array}.
    weights: optional {layer: (int8 weights, int32 bias)} replacing the seeded synthetic ones."""
    n_img = net["buffers"]["raw"]["shape"][0] if images is None else images
    bufs = {"raw": W.input_tensor(net, seed, n_img) if x_raw is None else x_raw}
    for op in net["ops"]:
        if op["dst"] not in bufs:
            bufs[op["dst"]] = _alloc(net, op["dst"], n_img)
        if op["op"] == "conv":
            w, b = weights[op["name"]] if weights is not None else (W.weight_tensor(op, seed), W.bias_tensor(op, seed))
            _conv(op, bufs, w, b, calib["conv"][op["name"]], bufs[op["dst"]])
        elif op["op"] == "maxpool":
            bufs[op["dst"]] = O.maxpool2d(bufs[op["src"]], op["k"], op["stride"], op["pad"])
        elif op["op"] == "avgpool":
            c = calib["avgpool"][op["dst"]]
            bufs[op["dst"]] = O.avgpool_global(bufs[op["src"]], c["mul"], c["shift"], c["bound_q"])
        else:
            raise ValueError(op["op"])
    return bufs


def calibrate(net, seed, per_channel=False, max_int=K.MAX_INT, floor_channels="layer"):
    """Returns (calib, buffers on the calibration images).

    calib = {"conv": {name: {...integers...}}, "avgpool": {dst: {...}}, "ratio": {...}}
    per_channel: BReLU layers and their residual merges get one (mul, shift) and one skip
    rescale per output channel ("mul_c", "shift_c", "res_mul_c", "res_shift_c"), each from
    that channel's own statistic (Section 3.4.3: one weight step per output channel).
    Concatenated branches, regression outputs and raw int32 outputs stay per layer.
    floor_channels: what a channel without a positive value in the calibration sample gets (its statistic is the
    floor, 1, and Section 3.3's bound needs positive activations to exist): "layer" = the layer's pair; "own" = the
    pair of its own statistic all the same, i.e. a ratio of max_int per unit (pairs of 20+ bits, the widest the
    method produces).  Both are valid integer networks; the second exists so that the per-channel path is also
    checked and timed on parameters that were not chosen with any kernel in mind.
    max_int: the largest quantised activation (Section 3.3), 2^bits - 1: 127 for the 7-bit
    activations of the main experiments, 255 / 63 / 31 / 15 for the other bit-depths the paper tries.
    """
    n_img = net["calib_images"]
    bufs = {"raw": W.input_tensor(net, seed, n_img)}
    ratio = {"raw": Fraction(INPUT_RATIO)}      # ratio_V of every stored buffer
    calib = {"conv": {}, "avgpool": {}, "max_int": int(max_int)}
    ops = net["ops"]
    i = 0
    while i < len(ops):
        op = ops[i]
        if op["op"] == "maxpool":
            bufs[op["dst"]] = O.maxpool2d(bufs[op["src"]], op["k"], op["stride"], op["pad"])
            ratio[op["dst"]] = ratio[op["src"]]
            i += 1
            continue
        if op["op"] == "avgpool":
            _, h, w, _ = bufs[op["src"]].shape
            m, s = K.mul_shift(h * w, 1)
            calib["avgpool"][op["dst"]] = {"mul": m, "shift": s, "bound_q": max_int}
            bufs[op["dst"]] = O.avgpool_global(bufs[op["src"]], m, s, max_int)
            ratio[op["dst"]] = ratio[op["src"]]
            i += 1
            continue
        # conv ops; the branches of one concatenation are calibrated together
        group = [op]
        if op["group"] is not None:
            while i + len(group) < len(ops) and ops[i + len(group)].get("group") == op["group"]:
                group.append(ops[i + len(group)])
        wts = [W.weight_tensor(g, seed) for g in group]
        bss = [W.bias_tensor(g, seed) for g in group]
        ratio_y = [ratio[g["src"]] * Fraction(K.MAX_INT) / Fraction(W.float_weight_absmax(g, seed))     # weights: 8 bits
                   for g in group]
        if op["dst"] not in bufs:
            bufs[op["dst"]] = _alloc(net, op["dst"], n_img)
        if op["group"] is not None:
            h_ri = []
            for g, w, b in zip(group, wts, bss):
                t = _conv(g, bufs, w, b, {}, None, out_mode="raw_s32")
                h_ri.append(K.percentile_999(t))
            params, r_min = K.sync_concat(h_ri, ratio_y, max_int)
            for g, w, b, (m, s, bq), h in zip(group, wts, bss, params, h_ri):
                cal = {"mul": m, "shift": s, "bound_q": bq, "h_ri": h}
                calib["conv"][g["name"]] = cal
                _conv(g, bufs, w, b, cal, bufs[g["dst"]])
            ratio[op["dst"]] = r_min
            i += len(group)
            continue
        w, b, ry = wts[0], bss[0], ratio_y[0]
        cal = {}
        if op["res_mode"] == "pre":
            # first the main path alone fixes the skip rescale, then the merged sum fixes the bound
            y = _conv(op, bufs, w, b, {}, None, out_mode="raw_s32", use_res=False)
            h_main = K.percentile_999(y)
            if op["res_dtype"] == "s32":
                h_skip = K.percentile_999(bufs[op["res"]])
            else:
                h_skip = max_int
            cal["res_mul"], cal["res_shift"] = K.mul_shift(h_skip, h_main)
            if per_channel and op["out_mode"] == "brelu":
                cout = y.shape[-1]
                hm = K.percentile_999_per_channel(y)
                # an int32 skip operand is not clamped, so a channel is scaled by its magnitude (a channel
                # whose values are mostly negative would otherwise get a bound of 1 and a huge rescale)
                hs = (K.percentile_999_per_channel(bufs[op["res"]][..., :cout], absolute=True)
                      if op["res_dtype"] == "s32" else [max_int] * cout)
                pairs = [K.mul_shift(a, b) for a, b in zip(hs, hm)]
                cal["res_mul_c"] = [m for m, _ in pairs]
                cal["res_shift_c"] = [s for _, s in pairs]
        if op["out_mode"] == "raw_s32":
            calib["conv"][op["name"]] = cal
            _conv(op, bufs, w, b, cal, bufs[op["dst"]])
            ratio[op["dst"]] = ry
        elif op["role"] == "regression_out":
            y = _conv(op, bufs, w, b, {}, None, out_mode="raw_s32", use_res=False)
            h = K.percentile_999(y, absolute=True)
            m, s = K.mul_shift(h, REGRESSION_LEVELS)
            cal.update(mul=m, shift=s, lo=0, hi=255, res_mul=1, res_shift=0, h_ri=h)
            calib["conv"][op["name"]] = cal
            _conv(op, bufs, w, b, cal, bufs[op["dst"]])
            ratio[op["dst"]] = Fraction(1)
        else:
            t = _conv(op, bufs, w, b, cal, None, out_mode="raw_s32")
            h = K.percentile_999(t)
            m, s = K.bound_params(h, max_int)
            cal.update(mul=m, shift=s, bound_q=max_int, h_ri=h)
            if per_channel:
                # a channel without positive values in the sample (statistic 1, the floor) has no bound
                # of its own: it keeps the layer's pair instead of a ratio of max_int per unit
                pairs = [K.bound_params(hc, max_int) if hc > 1 or floor_channels == "own" else (m, s)
                         for hc in K.percentile_999_per_channel(t)]
                cal["mul_c"] = [mc for mc, _ in pairs]
                cal["shift_c"] = [sc for _, sc in pairs]
            calib["conv"][op["name"]] = cal
            _conv(op, bufs, w, b, cal, bufs[op["dst"]])
            ratio[op["dst"]] = ry * m / (1 << s)
        i += 1
    calib["ratio"] = {k: float(v) for k, v in ratio.items()}
    return calib, bufs


def stored_calib_path(cfg, seed, per_channel=False, max_int=K.MAX_INT, floor_channels="layer"):
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    tag = ("_pc" if per_channel else "") + ("_own" if per_channel and floor_channels == "own" else "") + (
        "_a%d" % max_int if max_int != K.MAX_INT else "")
    return os.path.join(root, "workloads", "calib", "%s_seed%d%s.json" % (cfg, seed, tag))


def write_stored_calib(cfg, seed, per_channel=False, max_int=K.MAX_INT, floor_channels="layer"):
    """Calibrate config `cfg` with the oracle and store the integers for bench and tests."""
    import json
    net = W.CONFIGS[cfg]()
    calib, _ = calibrate(net, seed, per_channel, max_int, floor_channels)
    calib["net"] = net["name"]
    calib["seed"] = seed
    calib["written_by"] = "oracle/net.py write_stored_calib (calls only oracle/)"
    path = stored_calib_path(cfg, seed, per_channel, max_int, floor_channels)
    with open(path, "w") as f:
        if per_channel:
            json.dump(calib, f, sort_keys=True, separators=(",", ":"))
        else:
            json.dump(calib, f, indent=1, sort_keys=True)
    return path


if __name__ == "__main__":
    import sys
    import time
    # `python -m oracle.net [cfgN ...]` writes the per-layer files, `cfgN:pc` the per-channel one (`cfgN:pc_own`: floor
    # channels keep a pair of their own), `cfgN:a255` the one with 8-bit activations
    for name in sys.argv[1:] or ["cfg0", "cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "cfg6", "cfg3:pc", "cfg3:pc_own", "cfg1:a255"]:
        t0 = time.time()
        cfg, _, kind = name.partition(":")
        mi = int(kind[1:]) if kind.startswith("a") else K.MAX_INT
        print(write_stored_calib(cfg, 0, kind.startswith("pc"), mi, "own" if kind == "pc_own" else "layer"),
              "%.1fs" % (time.time() - t0), flush=True)
