"""numpy front end of the C oracle (oracle/icnn_oracle.c).

TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's
CPU-baseline leg import this.  Arrays are numpy, NHWC; weights are
[cout][kh][kw][cin].  See the C file's header for what is computed and which
passages of the paper each function follows.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

U8, S8, S32 = 0, 1, 2
OUT_BRELU_U8, OUT_CLAMP_U8, OUT_LINEAR_S8, OUT_RAW_S32 = 0, 1, 2, 3
RES_NONE, RES_PRE, RES_POST = 0, 1, 2

_OUT_MODES = {"brelu": OUT_BRELU_U8, "clamp_u8": OUT_CLAMP_U8, "linear_s8": OUT_LINEAR_S8,
              "raw_s32": OUT_RAW_S32}
_RES_MODES = {"none": RES_NONE, "pre": RES_PRE, "post": RES_POST}
_DT = {np.dtype(np.uint8): U8, np.dtype(np.int8): S8, np.dtype(np.int32): S32}


class ConvParams(C.Structure):
    _fields_ = [(k, C.c_int32) for k in (
        "n", "h", "w", "cin", "in_c_stride", "in_signed", "in_sub128",
        "cout", "kh", "kw", "stride_h", "stride_w", "pad_h", "pad_w",
        "out_c_stride", "out_c_offset", "mul", "shift", "bound_q", "lo", "hi",
        "out_mode", "res_mode", "res_dtype", "res_c_stride", "res_mul", "res_shift")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        L = C.CDLL(path)
        L.orc_rsr.restype = C.c_int64
        L.orc_rsr.argtypes = [C.c_int64, C.c_int32]
        L.orc_requant.restype = C.c_int64
        L.orc_requant.argtypes = [C.c_int64, C.c_int32, C.c_int32]
        L.orc_conv2d.restype = C.c_int
        L.orc_conv2d.argtypes = [C.POINTER(ConvParams)] + [C.c_void_p] * 5
        L.orc_conv2d_pc.restype = C.c_int
        L.orc_conv2d_pc.argtypes = [C.POINTER(ConvParams)] + [C.c_void_p] * 9
        L.orc_add_rescale.restype = C.c_int
        L.orc_add_rescale.argtypes = [C.c_int64, C.c_int32,
                                      C.c_void_p, C.c_int32, C.c_int32,
                                      C.c_void_p, C.c_int32, C.c_int32,
                                      C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                      C.c_int32, C.c_int32, C.c_int32,
                                      C.c_void_p, C.c_int32, C.c_int32]
        L.orc_concat.restype = C.c_int
        L.orc_concat.argtypes = [C.c_int32, C.POINTER(C.c_void_p), C.POINTER(C.c_int32),
                                 C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                 C.c_int32, C.c_int64, C.c_void_p, C.c_int32]
        L.orc_maxpool2d_u8.restype = C.c_int
        L.orc_maxpool2d_u8.argtypes = [C.c_int32] * 7 + [C.c_void_p, C.c_void_p]
        L.orc_avgpool_global_u8.restype = C.c_int
        L.orc_avgpool_global_u8.argtypes = [C.c_int32] * 7 + [C.c_void_p, C.c_void_p]
        L.orc_renormalize_u8.restype = C.c_int
        L.orc_renormalize_u8.argtypes = [C.c_int64, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def _mode(m, table):
    return table[m] if isinstance(m, str) else int(m)


def num_threads():
    """Threads the C oracle's parallel loops use."""
    L = lib()
    L.orc_num_threads.restype = C.c_int
    return int(L.orc_num_threads())


def rsr(v, s):
    """[v / 2^s], round half up."""
    return int(lib().orc_rsr(int(v), int(s)))


def requant(t, mul, shift):
    """[t * mul / 2^shift], round half up (activation requantisation)."""
    return int(lib().orc_requant(int(t), int(mul), int(shift)))


def conv_out_hw(h, w, kh, kw, stride, pad):
    return (h + 2 * pad - kh) // stride + 1, (w + 2 * pad - kw) // stride + 1


def conv2d(x, w, bias, *, stride=1, pad=0, mul=1, shift=0, bound_q=127, lo=0, hi=255,
           out_mode="brelu", res=None, res_mode="none", res_mul=1, res_shift=0,
           in_sub128=False, cin=None, out=None, out_c_offset=0,
           mul_c=None, shift_c=None, res_mul_c=None, res_shift_c=None):
    """One integer conv layer; returns the output buffer [N,Ho,Wo,Ctot].

    x: uint8 or int8 [N,H,W,Cbuf]; the first `cin` channels of each pixel are read.
    out: optional existing buffer whose channels out_c_offset..+cout are written.
    mul_c, shift_c, res_mul_c, res_shift_c: optional int32 [cout] arrays that replace the
    per-layer value of the same name channel by channel (Section 3.4.3).
    """
    x = np.ascontiguousarray(x)
    w = np.ascontiguousarray(w, dtype=np.int8)
    bias = np.ascontiguousarray(bias, dtype=np.int32)
    n, h, ww, cbuf = x.shape
    cout, kh, kw, wc = w.shape
    cin = wc if cin is None else cin
    assert wc == cin and cin <= cbuf and bias.shape == (cout,)
    om = _mode(out_mode, _OUT_MODES)
    rm = _mode(res_mode, _RES_MODES)
    ho, wo = conv_out_hw(h, ww, kh, kw, stride, pad)
    odt = {OUT_RAW_S32: np.int32, OUT_LINEAR_S8: np.int8}.get(om, np.uint8)
    if out is None:
        out = np.zeros((n, ho, wo, out_c_offset + cout), dtype=odt)
    assert out.flags.c_contiguous and out.dtype == odt and out.shape[:3] == (n, ho, wo)
    assert out_c_offset + cout <= out.shape[3]
    p = ConvParams()
    p.n, p.h, p.w, p.cin, p.in_c_stride = n, h, ww, cin, cbuf
    p.in_signed = int(x.dtype == np.int8)
    p.in_sub128 = int(bool(in_sub128))
    assert x.dtype in (np.uint8, np.int8) and not (p.in_sub128 and p.in_signed)
    p.cout, p.kh, p.kw = cout, kh, kw
    p.stride_h = p.stride_w = stride
    p.pad_h = p.pad_w = pad
    p.out_c_stride, p.out_c_offset = out.shape[3], out_c_offset
    p.mul, p.shift, p.bound_q, p.lo, p.hi = int(mul), int(shift), int(bound_q), int(lo), int(hi)
    p.out_mode, p.res_mode = om, rm
    rp = None
    if rm != RES_NONE:
        res = np.ascontiguousarray(res)
        assert res.shape[:3] == (n, ho, wo) and res.shape[3] >= cout
        p.res_dtype, p.res_c_stride = _DT[res.dtype], res.shape[3]
        p.res_mul, p.res_shift = int(res_mul), int(res_shift)
        rp = _ptr(res)
    pcs = []
    for arr in (mul_c, shift_c, res_mul_c, res_shift_c):
        if arr is not None:
            arr = np.ascontiguousarray(arr, dtype=np.int32)
            assert arr.shape == (cout,)
        pcs.append(arr)
    if any(a is not None for a in pcs):
        rc = lib().orc_conv2d_pc(C.byref(p), _ptr(x), _ptr(w), _ptr(bias), rp, _ptr(out),
                                 *[None if a is None else _ptr(a) for a in pcs])
    else:
        rc = lib().orc_conv2d(C.byref(p), _ptr(x), _ptr(w), _ptr(bias), rp, _ptr(out))
    if rc != 0:
        raise ArithmeticError("orc_conv2d failed: %d" % rc)
    return out


def add_rescale(a, b, *, b_mul=1, b_shift=0, mul=1, shift=0, lo=0, hi=127,
                out_mode="brelu", out=None, out_c_offset=0):
    """out = clamp([sat32(a + [b*b_mul/2^b_shift]) * mul / 2^shift], lo, hi); arrays [...,C]."""
    a = np.ascontiguousarray(a)
    b = np.ascontiguousarray(b)
    assert a.shape == b.shape
    c = a.shape[-1]
    px = a.size // c if c else 0
    om = _mode(out_mode, _OUT_MODES)
    if om == OUT_BRELU_U8:
        om = OUT_CLAMP_U8
    odt = {OUT_RAW_S32: np.int32, OUT_LINEAR_S8: np.int8}.get(om, np.uint8)
    if om == OUT_LINEAR_S8:
        lo, hi = -128, 127
    if out is None:
        out = np.zeros(a.shape[:-1] + (out_c_offset + c,), dtype=odt)
    assert out.dtype == odt and out.flags.c_contiguous
    rc = lib().orc_add_rescale(px, c, _ptr(a), _DT[a.dtype], c, _ptr(b), _DT[b.dtype], c,
                               int(b_mul), int(b_shift), int(mul), int(shift), int(lo), int(hi),
                               om, _ptr(out), out.shape[-1], out_c_offset)
    if rc != 0:
        raise ArithmeticError("orc_add_rescale failed: %d" % rc)
    return out


def concat(inputs, muls, shifts, bound_q=127):
    """Explicit concatenation on the channel axis with per-input requantisation."""
    inputs = [np.ascontiguousarray(t, dtype=np.uint8) for t in inputs]
    k = len(inputs)
    lead = inputs[0].shape[:-1]
    assert all(t.shape[:-1] == lead for t in inputs)
    cs = [t.shape[-1] for t in inputs]
    px = int(np.prod(lead))
    out = np.zeros(lead + (sum(cs),), dtype=np.uint8)
    ptrs = (C.c_void_p * k)(*[t.ctypes.data for t in inputs])
    arr = lambda v: (C.c_int32 * k)(*[int(q) for q in v])  # noqa: E731
    rc = lib().orc_concat(k, ptrs, arr(cs), arr(cs), arr(muls), arr(shifts), int(bound_q),
                          px, _ptr(out), out.shape[-1])
    if rc != 0:
        raise ArithmeticError("orc_concat failed: %d" % rc)
    return out


def maxpool2d(x, k=3, stride=2, pad=1):
    x = np.ascontiguousarray(x, dtype=np.uint8)
    n, h, w, c = x.shape
    ho, wo = conv_out_hw(h, w, k, k, stride, pad)
    out = np.zeros((n, ho, wo, c), dtype=np.uint8)
    rc = lib().orc_maxpool2d_u8(n, h, w, c, k, stride, pad, _ptr(x), _ptr(out))
    assert rc == 0
    return out


def avgpool_global(x, mul, shift, bound_q=127):
    x = np.ascontiguousarray(x, dtype=np.uint8)
    n, h, w, c = x.shape
    out = np.zeros((n, 1, 1, c), dtype=np.uint8)
    rc = lib().orc_avgpool_global_u8(n, h, w, c, int(mul), int(shift), int(bound_q),
                                     _ptr(x), _ptr(out))
    assert rc == 0
    return out


def renormalize(x):
    """Raw uint8 picture -> int8 samples x - 128 (Section 3.4.1)."""
    x = np.ascontiguousarray(x, dtype=np.uint8)
    out = np.zeros(x.shape, dtype=np.int8)
    rc = lib().orc_renormalize_u8(x.size, _ptr(x), _ptr(out))
    assert rc == 0
    return out
