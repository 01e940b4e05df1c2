"""Host-side checks of the C boundary that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def binding():
    from paper_2006_11735_amd import binding as B
    return B


def header_functions():
    text = open(os.path.join(ROOT, "include", "icnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b(i[a-z0-9_]+)\s*\(", text)) - {"int32_t", "int64_t", "int8_t"}


def test_library_exports_every_declared_symbol():
    B = binding()
    names = header_functions()
    assert {"iconv2d_brelu", "iadd_rescale", "iconcat", "icnn_last_error"} <= names
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert names == set(B.EXPORTS)
    assert B.icnn_version() >= 100


def good(B, **kw):
    base = dict(n=1, h=56, w=56, cin=64, in_c_stride=64, cout=64, kh=3, kw=3, pad_h=1, pad_w=1,
                out_c_stride=64, mul=23124, shift=26, bound_q=127)
    base.update(kw)
    return B.conv_desc(**base)


def test_conv_descriptor_validation():
    B = binding()
    assert B.iconv2d_validate(good(B)) == 0
    assert B.iconv2d_out_hw(good(B, stride_h=2, stride_w=2)) == (28, 28)
    bad = [
        (dict(n=0), B.ICNN_E_SHAPE), (dict(cin=0), B.ICNN_E_SHAPE), (dict(kh=0), B.ICNN_E_SHAPE),
        (dict(stride_h=0), B.ICNN_E_SHAPE), (dict(pad_h=-1), B.ICNN_E_SHAPE),
        (dict(h=1, w=1, pad_h=0, pad_w=0), B.ICNN_E_SHAPE),
        (dict(in_c_stride=63), B.ICNN_E_SHAPE), (dict(out_c_stride=63), B.ICNN_E_SHAPE),
        (dict(out_c_offset=1), B.ICNN_E_SHAPE), (dict(out_c_offset=-1, out_c_stride=128), B.ICNN_E_SHAPE),
        (dict(cin=8192, in_c_stride=8192), B.ICNN_E_SHAPE),          # K = 73728 > 65535
        (dict(mul=0), B.ICNN_E_PARAM), (dict(mul=-5), B.ICNN_E_PARAM),
        (dict(shift=-1), B.ICNN_E_PARAM), (dict(shift=63), B.ICNN_E_PARAM),
        (dict(bound_q=0), B.ICNN_E_PARAM), (dict(bound_q=256), B.ICNN_E_PARAM),
        (dict(out_mode=7), B.ICNN_E_PARAM), (dict(res_mode=3), B.ICNN_E_PARAM),
        (dict(in_signed=1, in_sub128=1), B.ICNN_E_PARAM), (dict(in_signed=3), B.ICNN_E_PARAM),
        (dict(in_signed=2, in_sub128=1), B.ICNN_E_PARAM),
        (dict(in_signed=2, cin=4096, in_c_stride=4096), B.ICNN_E_SHAPE),    # K = 36864 > 32767 with inputs up to 255
        (dict(out_mode=B.ICNN_OUT_CLAMP_U8, lo=5, hi=4), B.ICNN_E_PARAM),
        (dict(out_mode=B.ICNN_OUT_CLAMP_U8, lo=0, hi=256), B.ICNN_E_PARAM),
        (dict(res_mode=B.ICNN_RES_PRE, res_dtype=5, res_c_stride=64), B.ICNN_E_PARAM),
        (dict(res_mode=B.ICNN_RES_PRE, res_c_stride=32), B.ICNN_E_SHAPE),
        (dict(res_mode=B.ICNN_RES_PRE, res_c_stride=64, res_mul=0), B.ICNN_E_PARAM),
        (dict(res_mode=B.ICNN_RES_PRE, res_c_stride=64, res_shift=63), B.ICNN_E_PARAM),
        (dict(res_mode=B.ICNN_RES_POST, res_c_stride=64, out_mode=B.ICNN_OUT_RAW_S32), B.ICNN_E_PARAM),
    ]
    for kw, code in bad:
        assert B.iconv2d_validate(good(B, **kw)) == code, kw
        assert B.icnn_last_error() != ""
    # raw int32 output ignores mul / shift / bound
    assert B.iconv2d_validate(good(B, out_mode=B.ICNN_OUT_RAW_S32, mul=0, shift=99, bound_q=0)) == 0
    assert B.iconv2d_packed_weight_bytes(good(B)) == 4 * 9 * 2048 + 128 * 4      # fragments + one weight sum per padded channel
    assert B.iconv2d_workspace_bytes(good(B)) == 0


def test_entry_points_reject_bad_arguments_before_any_launch():
    B = binding()
    d = good(B)
    with pytest.raises(B.IcnnError) as e:
        B.iconv2d_brelu(d, None, None, None, None, None, None, stream=0)
    assert e.value.code == B.ICNN_E_NULL
    with pytest.raises(B.IcnnError) as e:
        B.iconv2d_brelu(d, 4096, 4096 + 8, 8192, None, 12288, None, stream=0)     # packed weights misaligned
    assert e.value.code == B.ICNN_E_ALIGN
    with pytest.raises(B.IcnnError) as e:
        B.iconv2d_brelu(good(B, res_mode=B.ICNN_RES_PRE, res_c_stride=64), 4096, 8192, 12288, None, 16384,
                        None, stream=0)
    assert e.value.code == B.ICNN_E_NULL
    with pytest.raises(B.IcnnError) as e:
        B.iconv2d_prepack_weights(d, None, 4096, stream=0)
    assert e.value.code == B.ICNN_E_NULL
    a = B.add_desc(count_pixels=10, c=16, a_c_stride=16, b_c_stride=16, out_c_stride=16, hi=127)
    for kw, code in ((dict(b_mul=0), B.ICNN_E_PARAM), (dict(shift=63), B.ICNN_E_PARAM),
                     (dict(a_c_stride=8), B.ICNN_E_SHAPE), (dict(count_pixels=-1), B.ICNN_E_SHAPE),
                     (dict(out_mode=B.ICNN_OUT_BRELU_U8), B.ICNN_E_PARAM), (dict(a_dtype=9), B.ICNN_E_PARAM),
                     (dict(lo=9, hi=3), B.ICNN_E_PARAM)):
        bad = B.add_desc(count_pixels=10, c=16, a_c_stride=16, b_c_stride=16, out_c_stride=16, hi=127)
        for k, v in kw.items():
            setattr(bad, k, v)
        with pytest.raises(B.IcnnError) as e:
            B.iadd_rescale(bad, 4096, 8192, 12288, stream=0)
        assert e.value.code == code, kw
    with pytest.raises(B.IcnnError) as e:
        B.iadd_rescale(a, None, 8192, 12288, stream=0)
    assert e.value.code == B.ICNN_E_NULL
    with pytest.raises(B.IcnnError) as e:
        B.iconcat([4096] * 17, [1] * 17, [1] * 17, [1] * 17, [0] * 17, 127, 4, 8192, 17, stream=0)
    assert e.value.code == B.ICNN_E_SHAPE
    with pytest.raises(B.IcnnError) as e:
        B.iconcat([4096, 8192], [8, 8], [8, 8], [1, 1], [0, 0], 127, 4, 12288, 15, stream=0)
    assert e.value.code == B.ICNN_E_SHAPE
    with pytest.raises(B.IcnnError) as e:
        B.iconcat([4096, 8192], [8, 8], [8, 8], [1, 0], [0, 0], 127, 4, 12288, 16, stream=0)
    assert e.value.code == B.ICNN_E_PARAM
    with pytest.raises(B.IcnnError) as e:
        B.imaxpool2d_u8(1, 8, 8, 16, 3, 2, 3, 4096, 8192, stream=0)
    assert e.value.code == B.ICNN_E_SHAPE
    with pytest.raises(B.IcnnError) as e:
        B.iavgpool_global_u8(1, 7, 7, 16, 0, 20, 127, 4096, 8192, stream=0)
    assert e.value.code == B.ICNN_E_PARAM
    with pytest.raises(B.IcnnError) as e:
        B.irenormalize_u8(16, None, 4096, stream=0)
    assert e.value.code == B.ICNN_E_NULL


def test_twin_layers_are_refused_on_the_host_where_the_fused_kernel_does_not_take_them():
    """iconv2d_twin_brelu checks both descriptors, the pointers and the pair's shape before anything is launched."""
    B = binding()

    def branch(k, cout, off, **kw):
        args = dict(h=32, w=64, cout=cout, kh=k, kw=k, pad_h=k // 2, pad_w=k // 2, out_c_stride=48, out_c_offset=off)
        args.update(kw)
        return good(B, **args)
    x, wa, wb, ba, bb, y = 4096, 8192, 12288, 16384, 20480, 24576
    cases = [
        ((branch(5, 32, 0), branch(5, 16, 32)), B.ICNN_E_UNSUPPORTED),                      # kernels of one size
        ((branch(7, 32, 0), branch(5, 16, 32)), B.ICNN_E_UNSUPPORTED),                      # no 7x7 form
        ((branch(5, 32, 0), branch(3, 16, 32, h=16)), B.ICNN_E_SHAPE),                      # different pictures
        ((branch(5, 32, 0), branch(3, 16, 32, cin=48, in_c_stride=48)), B.ICNN_E_SHAPE),    # different inputs
        ((branch(5, 32, 0, res_mode=B.ICNN_RES_PRE, res_c_stride=32), branch(3, 16, 32)), B.ICNN_E_UNSUPPORTED),
        ((branch(5, 32, 0, in_signed=B.ICNN_IN_U8_FULL), branch(3, 16, 32, in_signed=B.ICNN_IN_U8_FULL)), B.ICNN_E_UNSUPPORTED),
        ((branch(5, 32, 0, cin=32, in_c_stride=32), branch(3, 16, 32, cin=32, in_c_stride=32)), B.ICNN_E_UNSUPPORTED),
    ]
    for (da, db), code in cases:
        with pytest.raises(B.IcnnError) as e:
            B.iconv2d_twin_brelu(da, x, wa, ba, y, db, wb, bb, y, stream=0)
        assert e.value.code == code, (da.kh, db.kh, e.value.code)
    with pytest.raises(B.IcnnError) as e:
        B.iconv2d_twin_brelu(branch(5, 32, 0), x, wa, ba, y, branch(3, 16, 32), wb, bb, None, stream=0)
    assert e.value.code == B.ICNN_E_NULL
    with pytest.raises(B.IcnnError) as e:
        B.iconv2d_twin_brelu(branch(5, 32, 0), x + 8, wa, ba, y, branch(3, 16, 32), wb, bb, y, stream=0)
    assert e.value.code == B.ICNN_E_UNSUPPORTED                                              # misaligned input


def test_tuning_overrides_are_validated():
    B = binding()
    try:
        B.icnn_set_tuning("tile", 3)
        B.icnn_set_tuning("halo_always", 1)
        for name, value in (("tile", 5), ("tile", -2), ("stages", 1), ("stages", 7), ("no_fc", 2), ("colour", 1)):
            with pytest.raises(B.IcnnError) as e:
                B.icnn_set_tuning(name, value)
            assert e.value.code == B.ICNN_E_PARAM, (name, value)
    finally:
        B.icnn_set_tuning("reset")
