"""Offline conversion of a float32 CNN into the integer layer records the library runs
(the paper's Algorithm 1 without its training steps: given trained float weights and a
calibration batch it performs steps 1, 3, 6 and 7 once).

What is computed, per layer, in the paper's notation:

  * batch normalisation is folded into the convolution (Section 3.4.3);
  * weights:  Delta = max|W_f| / 127 per layer (or per output channel), W_i = [W_f / Delta],
    ratio_W = 1 / Delta, and the float network continues with the discretised W_d = W_i * Delta
    (Section 3.1, Section 3.4.3 "Training");
  * ratio_Y = ratio_X * ratio_W, b_i = [b_f * ratio_Y]   (Section 3.1);
  * BReLU bound by the n-sigma rule, h_rf = mu + n * sigma of the layer's pre-activation values on
    the calibration batch (Section 3.2.2), h_ri = [h_rf * ratio_Y], (mul, shift) with
    [h_ri * mul / 2^shift] = max_int, ratio_V = ratio_Y * mul / 2^shift, h_f = max_int / ratio_V
    (Section 3.3);
  * input re-normalisation: raw uint8 - 128, i.e. X_f = raw / 256 - 0.5 and ratio_X = 256
    (Section 3.4.1);
  * residual merge: the skip operand is brought to the main path's ratio by (res_mul, res_shift),
    then the main conv's Delta is adjusted so that both ratios are exactly equal (Section 4.1);
  * concatenation: every branch is rescaled to the smallest branch ratio (Algorithm 2);
  * a regression network's last layer resets the ratio to pixel units (Section 3.1).

The network description is the plain op list of `workloads.nets` (shapes only).  Everything here is
host-side, offline, float64 numpy / torch-CPU arithmetic; nothing of it runs in the inference path.
`[.]` is round half up, as everywhere in this package.
"""
import math
from fractions import Fraction

import numpy as np
import torch

MAX_SHIFT = 46
INPUT_RATIO = 256.0


def rhu(x):
    """[x]: round half up, element-wise."""
    return np.floor(np.asarray(x, dtype=np.float64) + 0.5)


def mul_shift(a, b):
    """Integers (mul, shift) with mul / 2^shift ~ b / a: the smallest shift in [0, 46] whose rounded
    multiplier reaches 2^14 (the paper's mul_shift() is not spelled out; this is the reading used
    throughout)."""
    ratio = Fraction(b) / Fraction(a)
    if ratio <= 0:
        raise ValueError("ratio must be positive")
    for s in range(MAX_SHIFT + 1):
        m = math.floor(ratio * (1 << s) + Fraction(1, 2))
        if m >= (1 << 14) or s == MAX_SHIFT:
            return max(1, min(m, (1 << 31) - 1)), s
    raise AssertionError


def _requant(v, mul, shift):
    return (int(v) * int(mul) + ((1 << shift) >> 1)) >> shift


def bound_params(h_ri, max_int):
    """(mul, shift) with [h_ri * mul / 2^shift] == max_int (Section 3.3)."""
    h_ri = max(1, int(h_ri))
    mul, s = mul_shift(h_ri, max_int)
    for _ in range(1 << 16):
        q = _requant(h_ri, mul, s)
        if q == max_int:
            return mul, s
        mul += 1 if q < max_int else -1
        if mul < 1:
            break
    raise ArithmeticError("no multiplier maps %d to %d" % (h_ri, max_int))


def fold_bn(w, b, bn):
    """Conv followed by batch normalisation as one conv (w: [cout, kh, kw, cin])."""
    gamma, beta, mean, var, eps = bn
    k = np.asarray(gamma, np.float64) / np.sqrt(np.asarray(var, np.float64) + eps)
    return w * k[:, None, None, None], (b - mean) * k + beta


def _conv_f(x, w, stride, pad):
    """float64 NHWC convolution, weights [cout, kh, kw, cin]."""
    xt = torch.from_numpy(np.ascontiguousarray(x)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(np.ascontiguousarray(w)).permute(0, 3, 1, 2)
    return torch.nn.functional.conv2d(xt, wt, stride=stride, padding=pad).permute(0, 2, 3, 1).numpy()


def _maxpool_f(x, k, stride, pad):
    xt = torch.from_numpy(np.ascontiguousarray(x)).permute(0, 3, 1, 2)
    return torch.nn.functional.max_pool2d(xt, k, stride, pad).permute(0, 2, 3, 1).numpy()


def convert(net, float_params, raw, n_sigma=3.0, max_int=127, per_channel=False):
    """Returns (calib, weights, info).

    net: op list as built by workloads.nets.  float_params[name] = {"w": [cout,kh,kw,cin], "b": [cout],
    optional "bn": (gamma, beta, mean, var, eps)}.  raw: uint8 calibration batch [N,H,W,C].
    calib: the integers of every layer in the layout the runners take ({"conv": {name: {...}},
    "avgpool": {...}, "max_int": ...}); weights[name] = (int8 [cout,kh,kw,cin], int32 [cout]).
    info: {"ratio": {buffer: ratio_V}, "ratio_y": {layer: ratio_Y}, "float": {buffer: float activations
    of the BReLU-enabled, weight-discretised float network on `raw`}, "h_f": {layer: bound}} for
    checking the conversion.
    """
    raw = np.ascontiguousarray(raw, dtype=np.uint8)
    fl = {"raw": raw.astype(np.float64) / INPUT_RATIO - 0.5}      # re-normalised float input
    ratio = {"raw": INPUT_RATIO}
    calib = {"conv": {}, "avgpool": {}, "max_int": int(max_int)}
    weights, h_fs = {}, {"__ratio_y": {}}
    ops = net["ops"]
    i = 0
    while i < len(ops):
        op = ops[i]
        if op["op"] == "maxpool":
            fl[op["dst"]] = _maxpool_f(fl[op["src"]], op["k"], op["stride"], op["pad"])
            ratio[op["dst"]] = ratio[op["src"]]
            i += 1
            continue
        if op["op"] == "avgpool":
            x = fl[op["src"]]
            m, s = mul_shift(x.shape[1] * x.shape[2], 1)
            calib["avgpool"][op["dst"]] = {"mul": m, "shift": s, "bound_q": int(max_int)}
            fl[op["dst"]] = x.mean(axis=(1, 2), keepdims=True)
            ratio[op["dst"]] = ratio[op["src"]] * x.shape[1] * x.shape[2] * m / float(1 << s)
            i += 1
            continue
        group = [op]
        if op["group"] is not None:
            while i + len(group) < len(ops) and ops[i + len(group)].get("group") == op["group"]:
                group.append(ops[i + len(group)])
        done = [_convert_conv(g, net, float_params[g["name"]], fl, ratio, n_sigma, max_int,
                              per_channel and g["group"] is None and g["role"] != "regression_out") for g in group]
        if op["group"] is not None:
            _sync_concat(done, max_int)                     # Algorithm 2
        for g, d in zip(group, done):
            _finish_conv(net, g, d, fl, ratio, calib, weights, h_fs, max_int)
        i += len(group)
    ratio_y = h_fs.pop("__ratio_y")
    return calib, weights, {"ratio": ratio, "ratio_y": ratio_y, "float": fl, "h_f": h_fs}


def _quantise_weights(w, delta):
    """W_i = [W_f / Delta], kept inside [-127, 127]; delta scalar or per output channel."""
    d = np.asarray(delta, np.float64).reshape(-1, 1, 1, 1) if np.ndim(delta) else float(delta)
    return np.clip(rhu(w / d), -127, 127).astype(np.int8)


def _convert_conv(op, net, prm, fl, ratio, n_sigma, max_int, per_channel):
    w = np.asarray(prm["w"], np.float64)
    b = np.asarray(prm["b"], np.float64)
    if prm.get("bn") is not None:
        w, b = fold_bn(w, b, prm["bn"])
    x = fl[op["src"]][..., :op["cin"]]
    absmax = np.abs(w).reshape(w.shape[0], -1).max(axis=1) if per_channel else np.abs(w).max()
    delta = np.maximum(absmax, 1e-30) / 127.0
    d = {"op": op, "w_f": w, "b_f": b, "delta": delta, "ratio_x": float(ratio[op["src"]]), "x": x, "n_sigma": n_sigma}
    # skip operand: fix (res_mul, res_shift), then adjust Delta so that the two ratios agree exactly
    if op["res_mode"] == "pre":
        ratio_y = d["ratio_x"] / delta                              # scalar or [cout]
        n = w.shape[0] if (np.ndim(ratio_y) or np.ndim(ratio[op["res"]])) else 1
        rs = np.broadcast_to(np.atleast_1d(np.asarray(ratio[op["res"]], np.float64)), (n,))
        ry = np.broadcast_to(np.atleast_1d(np.asarray(ratio_y, np.float64)), (n,))
        pairs = [mul_shift(Fraction(float(a)), Fraction(float(b_))) for a, b_ in zip(rs, ry)]
        exact = np.array([a * m / float(1 << s) for a, (m, s) in zip(rs, pairs)])
        d["delta"] = (d["ratio_x"] / exact) if n > 1 else float(d["ratio_x"] / exact[0])
        d["res"] = pairs
    return d


def _sync_concat(done, max_int):
    """Algorithm 2: bring every branch to the smallest branch ratio; each branch's Delta is corrected so
    that its rescaled ratio equals that minimum exactly."""
    for d in done:
        _measure(d, d["n_sigma"], max_int)
    r_min = min(d["ratio_v"] for d in done)
    for d in done:
        m, s = mul_shift(Fraction(float(d["ratio_y"])), Fraction(float(r_min)))
        factor = d["ratio_y"] * m / float(1 << s) / r_min            # ~ 1
        d["delta"] = d["delta"] * factor
        d["concat"] = (m, s, r_min)


def _measure(d, n_sigma, max_int):
    """Discretise the weights, run the float layer, take the n-sigma bound and the BReLU integers."""
    op = d["op"]
    w_i = _quantise_weights(d["w_f"], d["delta"])
    dl = np.asarray(d["delta"], np.float64)
    w_d = w_i.astype(np.float64) * (dl.reshape(-1, 1, 1, 1) if dl.ndim else float(dl))
    y = _conv_f(d["x"], w_d, op["stride"], op["pad"]) + d["b_f"]
    d["w_i"], d["y_main"] = w_i, y
    d["ratio_y"] = d["ratio_x"] / dl if dl.ndim else d["ratio_x"] / float(dl)
    h_rf = float(y.mean() + n_sigma * y.std())
    d["h_rf"] = max(h_rf, 1e-12)
    ry = float(np.max(d["ratio_y"])) if dl.ndim else float(d["ratio_y"])
    h_ri = max(1, int(rhu(d["h_rf"] * ry)))
    m, s = bound_params(h_ri, max_int)
    d["ratio_v"] = ry * m / float(1 << s)


def _finish_conv(net, op, d, fl, ratio, calib, weights, h_fs, max_int):
    cal = {}
    n_sigma = d["n_sigma"]
    # (re)discretise with the final Delta and run the float layer
    w_i = _quantise_weights(d["w_f"], d["delta"])
    dl = np.asarray(d["delta"], np.float64)
    pc = dl.ndim > 0
    w_d = w_i.astype(np.float64) * (dl.reshape(-1, 1, 1, 1) if pc else float(dl))
    ratio_y = d["ratio_x"] / dl if pc else d["ratio_x"] / float(dl)
    y = _conv_f(d["x"], w_d, op["stride"], op["pad"]) + d["b_f"]
    b_i = rhu(d["b_f"] * ratio_y)
    if np.abs(b_i).max() > 2 ** 30:
        raise ArithmeticError("bias of %s does not fit the int32 contract" % op["name"])
    weights[op["name"]] = (w_i, b_i.astype(np.int32))
    h_fs["__ratio_y"][op["name"]] = ratio_y
    if op["res_mode"] == "pre":
        y = y + fl[op["res"]][..., :op["cout"]]
        if pc:
            cal["res_mul_c"] = [m for m, _ in d["res"]]
            cal["res_shift_c"] = [s for _, s in d["res"]]
        cal["res_mul"], cal["res_shift"] = max(d["res"], key=lambda t: t[0] / 2.0 ** t[1])
    if op["out_mode"] == "raw_s32":
        fl[op["dst"]] = y
        ratio[op["dst"]] = ratio_y                             # a vector with per-channel weight steps
    elif op["role"] == "regression_out":
        # pixel units: out = clamp([Y_i * mul / 2^shift] + raw, 0, 255), mul / 2^shift = 256 / ratio_Y
        m, s = mul_shift(Fraction(float(ratio_y)), Fraction(INPUT_RATIO))
        cal.update(mul=m, shift=s, lo=0, hi=255, res_mul=1, res_shift=0)
        fl[op["dst"]] = np.clip(rhu(y * INPUT_RATIO) + (fl["raw"] + 0.5) * INPUT_RATIO, 0, 255)
        ratio[op["dst"]] = 1.0
    elif "concat" in d:
        m, s, r_min = d["concat"]
        h_ri = max(1, int(rhu(d["h_rf"] * float(ratio_y))))
        bq = max(1, min(int(max_int), _requant(h_ri, m, s)))
        cal.update(mul=m, shift=s, bound_q=bq)
        h_f = bq / r_min
        out = fl.setdefault(op["dst"], np.zeros(y.shape[:3] + (net["buffers"][op["dst"]]["shape"][3],), np.float64))
        out[..., op["dst_c_offset"]:op["dst_c_offset"] + op["cout"]] = np.clip(y, 0, h_f)
        ratio[op["dst"]] = r_min
        h_fs[op["name"]] = h_f
    else:
        h_rf = max(float(y.mean() + n_sigma * y.std()), 1e-12)
        if pc:
            # one float bound for the layer; every channel gets the (mul, shift) that maps it to max_int
            pairs = [bound_params(max(1, int(rhu(h_rf * ry))), max_int) for ry in ratio_y]
            cal["mul_c"] = [m for m, _ in pairs]
            cal["shift_c"] = [s for _, s in pairs]
            rv = np.array([ry * m / float(1 << s) for ry, (m, s) in zip(ratio_y, pairs)])
            ratio_v = float(np.median(rv))
            cal.update(mul=pairs[0][0], shift=pairs[0][1])
        else:
            m, s = bound_params(max(1, int(rhu(h_rf * float(ratio_y)))), max_int)
            cal.update(mul=m, shift=s)
            ratio_v = float(ratio_y) * m / float(1 << s)
        cal["bound_q"] = int(max_int)
        h_f = max_int / ratio_v                               # the bound the float network continues with
        fl[op["dst"]] = np.clip(y, 0, h_f)
        ratio[op["dst"]] = ratio_v
        h_fs[op["name"]] = h_f
    calib["conv"][op["name"]] = cal


def dequantise(buf, ratio_v):
    """Integer activations back to the float network's units."""
    return np.asarray(buf, np.float64) / ratio_v
