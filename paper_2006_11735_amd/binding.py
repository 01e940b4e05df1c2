"""ctypes binding of libicnn_mi355.so: the same names and arguments as
include/icnn.h, with torch tensors (or raw device addresses) marshalled to
pointers.  Argument marshalling only -- no arithmetic happens here.
"""
import ctypes as C
import os

import torch  # noqa: F401  (first, so that the library below binds to the HIP runtime torch has loaded: two runtimes
#                            in one process do not see the device)

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libicnn_mi355.so")

ICNN_OK = 0
ICNN_IN_U8_LE127, ICNN_IN_S8, ICNN_IN_U8_FULL = 0, 1, 2
ICNN_E_NULL, ICNN_E_SHAPE, ICNN_E_PARAM, ICNN_E_ALIGN, ICNN_E_UNSUPPORTED, ICNN_E_LAUNCH = -1, -2, -3, -4, -5, -6
ICNN_U8, ICNN_S8, ICNN_S32 = 0, 1, 2
ICNN_OUT_BRELU_U8, ICNN_OUT_CLAMP_U8, ICNN_OUT_LINEAR_S8, ICNN_OUT_RAW_S32 = 0, 1, 2, 3
ICNN_RES_NONE, ICNN_RES_PRE, ICNN_RES_POST = 0, 1, 2


class icnn_conv_desc(C.Structure):
    _fields_ = [(k, C.c_int32) for k in (
        "n", "h", "w", "cin", "in_c_stride", "in_signed", "in_sub128",
        "cout", "kh", "kw", "stride_h", "stride_w", "pad_h", "pad_w",
        "out_c_stride", "out_c_offset", "mul", "shift", "bound_q", "lo", "hi",
        "out_mode", "res_mode", "res_dtype", "res_c_stride", "res_mul", "res_shift")]


class icnn_add_desc(C.Structure):
    _fields_ = [("count_pixels", C.c_int64)] + [(k, C.c_int32) for k in (
        "c", "a_c_stride", "b_c_stride", "out_c_stride", "out_c_offset",
        "a_dtype", "b_dtype", "out_mode", "b_mul", "b_shift", "mul", "shift", "lo", "hi")]


class icnn_channel_params(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("mul", "shift", "res_mul", "res_shift")]


class IcnnError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("icnn error %d: %s" % (code, msg))
        self.code = code


if not os.path.exists(LIB_PATH):
    raise ImportError("%s is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                      "(there is no CPU fallback)" % LIB_PATH)

_lib = C.CDLL(LIB_PATH)
_vp, _i32, _i64 = C.c_void_p, C.c_int32, C.c_int64
_lib.icnn_version.restype = C.c_int
_lib.icnn_last_error.restype = C.c_char_p
_lib.icnn_set_tuning.argtypes = [C.c_char_p, _i32]
_lib.iconv2d_validate.argtypes = [C.POINTER(icnn_conv_desc)]
_lib.iconv2d_out_hw.argtypes = [C.POINTER(icnn_conv_desc), C.POINTER(_i32), C.POINTER(_i32)]
_lib.iconv2d_workspace_bytes.argtypes = [C.POINTER(icnn_conv_desc), C.POINTER(C.c_size_t)]
_lib.iconv2d_packed_weight_bytes.argtypes = [C.POINTER(icnn_conv_desc), C.POINTER(C.c_size_t)]
_lib.iconv2d_prepack_weights.argtypes = [C.POINTER(icnn_conv_desc), _vp, _vp, _vp]
_lib.iconv2d_brelu.argtypes = [C.POINTER(icnn_conv_desc), _vp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.iconv2d_brelu_static_ws.argtypes = [C.POINTER(icnn_conv_desc), _vp, _vp, _vp, _vp, _vp, _vp]
_lib.iconv2d_packed_channel_params_bytes.argtypes = [C.POINTER(icnn_conv_desc), C.POINTER(C.c_size_t)]
_lib.iconv2d_prepack_channel_params.argtypes = [C.POINTER(icnn_conv_desc), C.POINTER(icnn_channel_params), _vp, _vp]
_lib.iconv2d_brelu_pc.argtypes = [C.POINTER(icnn_conv_desc), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.iconv2d_dual_brelu.argtypes = [C.POINTER(icnn_conv_desc), _vp, _vp, _vp, C.POINTER(icnn_conv_desc), _vp, _vp, _vp,
                                    _vp, _vp]
_lib.iconv2d_dual_brelu_pc.argtypes = [C.POINTER(icnn_conv_desc), _vp, _vp, _vp, _vp, C.POINTER(icnn_conv_desc), _vp, _vp,
                                       _vp, _vp, _vp]
_lib.iconv2d_maxpool_brelu.argtypes = [C.POINTER(icnn_conv_desc), _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp]
_lib.iconv2d_bottleneck_brelu.argtypes = [C.POINTER(icnn_conv_desc), _vp, _vp, _vp, C.POINTER(icnn_conv_desc), _vp, _vp,
                                          C.POINTER(icnn_conv_desc), _vp, _vp, _vp, _vp, _vp]
_lib.iconv2d_bottleneck_dual_brelu.argtypes = [C.POINTER(icnn_conv_desc), _vp, _vp, _vp, C.POINTER(icnn_conv_desc), _vp, _vp,
                                               C.POINTER(icnn_conv_desc), _vp, _vp, C.POINTER(icnn_conv_desc), _vp, _vp, _vp, _vp]
_lib.iconv2d_pair_brelu.argtypes = [C.POINTER(icnn_conv_desc), _vp, _vp, _vp, _vp, _vp, C.POINTER(icnn_conv_desc), _vp, _vp, _vp, _vp]
_lib.iconv2d_twin_brelu.argtypes = [C.POINTER(icnn_conv_desc), _vp, _vp, _vp, _vp, C.POINTER(icnn_conv_desc), _vp, _vp, _vp, _vp]
_lib.iadd_rescale.argtypes = [C.POINTER(icnn_add_desc), _vp, _vp, _vp, _vp]
_lib.iconcat.argtypes = [_i32, C.POINTER(_vp), C.POINTER(_i32), C.POINTER(_i32), C.POINTER(_i32),
                         C.POINTER(_i32), _i32, _i64, _vp, _i32, _vp]
_lib.imaxpool2d_u8.argtypes = [_i32] * 7 + [_vp, _vp, _vp]
_lib.iavgpool_global_u8.argtypes = [_i32] * 7 + [_vp, _vp, _vp]
_lib.irenormalize_u8.argtypes = [_i64, _vp, _vp, _vp]
_lib.icnn_peak_mfma_i8.argtypes = [_i32, _i32, _vp, _vp]
_lib.icnn_peak_copy.argtypes = [_vp, _vp, C.c_size_t, _vp]

EXPORTS = ["icnn_version", "icnn_last_error", "icnn_set_tuning", "iconv2d_validate", "iconv2d_out_hw",
           "iconv2d_workspace_bytes", "iconv2d_packed_weight_bytes", "iconv2d_prepack_weights",
           "iconv2d_brelu", "iconv2d_brelu_static_ws", "iconv2d_packed_channel_params_bytes", "iconv2d_prepack_channel_params", "iconv2d_brelu_pc",
           "iconv2d_dual_brelu", "iconv2d_dual_brelu_pc", "iconv2d_bottleneck_brelu", "iconv2d_bottleneck_dual_brelu", "iconv2d_pair_brelu", "iconv2d_twin_brelu", "iconv2d_maxpool_brelu", "iadd_rescale", "iconcat", "imaxpool2d_u8", "iavgpool_global_u8",
           "irenormalize_u8", "icnn_peak_mfma_i8", "icnn_peak_copy"]


def _ptr(t):
    """Device address of a torch tensor, or an int / None passed through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _check(rc):
    if rc != 0:
        raise IcnnError(rc, icnn_last_error())
    return rc


def icnn_version():
    return _lib.icnn_version()


def icnn_last_error():
    return _lib.icnn_last_error().decode()


def icnn_set_tuning(name, value=0):
    return _check(_lib.icnn_set_tuning(name.encode(), int(value)))


def conv_desc(**kw):
    d = icnn_conv_desc()
    d.stride_h = d.stride_w = 1
    d.mul, d.bound_q, d.hi, d.res_mul = 1, 127, 255, 1
    for k, v in kw.items():
        if not hasattr(d, k):
            raise AttributeError(k)
        setattr(d, k, int(v))
    return d


def add_desc(**kw):
    d = icnn_add_desc()
    d.b_mul = d.mul = 1
    d.hi = 255
    d.out_mode = ICNN_OUT_CLAMP_U8
    for k, v in kw.items():
        if not hasattr(d, k):
            raise AttributeError(k)
        setattr(d, k, int(v))
    return d


def iconv2d_validate(desc):
    return _lib.iconv2d_validate(C.byref(desc))


def iconv2d_out_hw(desc):
    ho, wo = _i32(), _i32()
    _check(_lib.iconv2d_out_hw(C.byref(desc), C.byref(ho), C.byref(wo)))
    return ho.value, wo.value


def iconv2d_workspace_bytes(desc):
    b = C.c_size_t()
    _check(_lib.iconv2d_workspace_bytes(C.byref(desc), C.byref(b)))
    return b.value


def iconv2d_packed_weight_bytes(desc):
    b = C.c_size_t()
    _check(_lib.iconv2d_packed_weight_bytes(C.byref(desc), C.byref(b)))
    return b.value


def iconv2d_prepack_weights(desc, w_ohwi, w_packed, stream=None):
    return _check(_lib.iconv2d_prepack_weights(C.byref(desc), _ptr(w_ohwi), _ptr(w_packed), _stream(stream)))


def iconv2d_brelu(desc, x, w_packed, bias, res, y, workspace=None, stream=None):
    return _check(_lib.iconv2d_brelu(C.byref(desc), _ptr(x), _ptr(w_packed), _ptr(bias), _ptr(res),
                                     _ptr(y), _ptr(workspace), _stream(stream)))


ICNN_STATIC_WORKSPACE_BYTES = 16 << 20


def iconv2d_brelu_static_ws(desc, x, w_packed, bias, res, y, stream=None):
    return _check(_lib.iconv2d_brelu_static_ws(C.byref(desc), _ptr(x), _ptr(w_packed), _ptr(bias), _ptr(res),
                                               _ptr(y), _stream(stream)))


def channel_params(mul=None, shift=None, res_mul=None, res_shift=None):
    """icnn_channel_params over device int32 tensors (or addresses); the caller keeps them alive."""
    pc = icnn_channel_params()
    pc.mul, pc.shift, pc.res_mul, pc.res_shift = _ptr(mul), _ptr(shift), _ptr(res_mul), _ptr(res_shift)
    return pc


def iconv2d_packed_channel_params_bytes(desc):
    b = C.c_size_t()
    _check(_lib.iconv2d_packed_channel_params_bytes(C.byref(desc), C.byref(b)))
    return b.value


def iconv2d_prepack_channel_params(desc, pc, packed, stream=None):
    return _check(_lib.iconv2d_prepack_channel_params(C.byref(desc), C.byref(pc), _ptr(packed), _stream(stream)))


def iconv2d_brelu_pc(desc, x, w_packed, bias, pc_packed, res, y, workspace=None, stream=None):
    return _check(_lib.iconv2d_brelu_pc(C.byref(desc), _ptr(x), _ptr(w_packed), _ptr(bias), _ptr(pc_packed), _ptr(res),
                                        _ptr(y), _ptr(workspace), _stream(stream)))


def iconv2d_dual_brelu(main_desc, x_main, w_main_packed, bias_main, proj_desc, x_proj, w_proj_packed, bias_proj, y,
                       stream=None):
    return _check(_lib.iconv2d_dual_brelu(C.byref(main_desc), _ptr(x_main), _ptr(w_main_packed), _ptr(bias_main),
                                          C.byref(proj_desc), _ptr(x_proj), _ptr(w_proj_packed), _ptr(bias_proj),
                                          _ptr(y), _stream(stream)))


def iconv2d_dual_brelu_pc(main_desc, x_main, w_main_packed, bias_main, pc_packed_main, proj_desc, x_proj, w_proj_packed,
                          bias_proj, y, stream=None):
    return _check(_lib.iconv2d_dual_brelu_pc(C.byref(main_desc), _ptr(x_main), _ptr(w_main_packed), _ptr(bias_main),
                                             _ptr(pc_packed_main), C.byref(proj_desc), _ptr(x_proj), _ptr(w_proj_packed),
                                             _ptr(bias_proj), _ptr(y), _stream(stream)))


def iconv2d_maxpool_brelu(desc, pool_k, pool_stride, pool_pad, x, w_packed, bias, y, stream=None):
    return _check(_lib.iconv2d_maxpool_brelu(C.byref(desc), pool_k, pool_stride, pool_pad, _ptr(x), _ptr(w_packed), _ptr(bias),
                                             _ptr(y), _stream(stream)))


def iconv2d_bottleneck_brelu(c1, x, w1_packed, bias1, c2, w2_packed, bias2, c3, w3_packed, bias3, res, y, stream=None):
    return _check(_lib.iconv2d_bottleneck_brelu(C.byref(c1), _ptr(x), _ptr(w1_packed), _ptr(bias1), C.byref(c2), _ptr(w2_packed),
                                                _ptr(bias2), C.byref(c3), _ptr(w3_packed), _ptr(bias3), _ptr(res), _ptr(y),
                                                _stream(stream)))


def iconv2d_bottleneck_dual_brelu(c1, x, w1_packed, bias1, c2, w2_packed, bias2, c3, w3_packed, bias3, cp, wp_packed, biasp, y, stream=None):
    return _check(_lib.iconv2d_bottleneck_dual_brelu(C.byref(c1), _ptr(x), _ptr(w1_packed), _ptr(bias1), C.byref(c2), _ptr(w2_packed),
                                                     _ptr(bias2), C.byref(c3), _ptr(w3_packed), _ptr(bias3), C.byref(cp),
                                                     _ptr(wp_packed), _ptr(biasp), _ptr(y), _stream(stream)))


def iconv2d_pair_brelu(c3, t, w3_packed, bias3, res, y, c1, w1_packed, bias1, z, stream=None):
    return _check(_lib.iconv2d_pair_brelu(C.byref(c3), _ptr(t), _ptr(w3_packed), _ptr(bias3), _ptr(res), _ptr(y), C.byref(c1),
                                          _ptr(w1_packed), _ptr(bias1), _ptr(z), _stream(stream)))


def iconv2d_twin_brelu(ca, x, wa_packed, bias_a, ya, cb, wb_packed, bias_b, yb, stream=None):
    return _check(_lib.iconv2d_twin_brelu(C.byref(ca), _ptr(x), _ptr(wa_packed), _ptr(bias_a), _ptr(ya), C.byref(cb),
                                          _ptr(wb_packed), _ptr(bias_b), _ptr(yb), _stream(stream)))


def iadd_rescale(desc, a, b, out, stream=None):
    return _check(_lib.iadd_rescale(C.byref(desc), _ptr(a), _ptr(b), _ptr(out), _stream(stream)))


def iconcat(inputs, c_in, in_c_stride, mul, shift, bound_q, count_pixels, out, out_c_stride, stream=None):
    n = len(inputs)
    arr = lambda v: (_i32 * n)(*[int(q) for q in v])  # noqa: E731
    ptrs = (_vp * n)(*[_ptr(t) for t in inputs])
    return _check(_lib.iconcat(n, ptrs, arr(c_in), arr(in_c_stride), arr(mul), arr(shift), int(bound_q),
                               int(count_pixels), _ptr(out), int(out_c_stride), _stream(stream)))


def imaxpool2d_u8(n, h, w, c, k, stride, pad, x, out, stream=None):
    return _check(_lib.imaxpool2d_u8(n, h, w, c, k, stride, pad, _ptr(x), _ptr(out), _stream(stream)))


def iavgpool_global_u8(n, h, w, c, mul, shift, bound_q, x, out, stream=None):
    return _check(_lib.iavgpool_global_u8(n, h, w, c, mul, shift, bound_q, _ptr(x), _ptr(out), _stream(stream)))


def irenormalize_u8(count, x, out, stream=None):
    return _check(_lib.irenormalize_u8(count, _ptr(x), _ptr(out), _stream(stream)))


def icnn_peak_mfma_i8(blocks, iters, sink, stream=None):
    return _check(_lib.icnn_peak_mfma_i8(int(blocks), int(iters), _ptr(sink), _stream(stream)))


def icnn_peak_copy(src, dst, nbytes, stream=None):
    return _check(_lib.icnn_peak_copy(_ptr(src), _ptr(dst), int(nbytes), _stream(stream)))
