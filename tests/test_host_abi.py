"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol
include/fscnn.h declares, and its argument validation answers before any device work."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2212_08815_amd import fscnn
    if not os.path.exists(fscnn.LIB_PATH):
        from paper_2212_08815_amd import build
        build.build()
    return fscnn.lib()


def test_every_declared_symbol_is_exported(L):
    from paper_2212_08815_amd import fscnn
    text = open(os.path.join(ROOT, "include", "fscnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(fscnn_[a-z0-9_]+)\s*\(", text))
    assert declared == set(fscnn.EXPORTS)
    for name in declared:
        assert getattr(L, name) is not None


def test_out_shape_and_status_strings(L):
    from paper_2212_08815_amd import fscnn
    assert fscnn.conv2d_out_shape(224, 224, 3, 3, (1, 1), (1, 1)) == (224, 224)
    assert fscnn.conv2d_out_shape(7, 8, 3, 3, (2, 2), (0, 0)) == (3, 3)
    assert fscnn.conv2d_out_shape(5, 9, 5, 1, (1, 3), (0, 0)) == (1, 3)
    for bad in [(0, 5, 3, 3, 1, 1, 0, 0), (5, 5, 3, 3, 0, 1, 0, 0), (5, 5, 3, 3, 1, 1, -1, 0),
                (2, 5, 3, 3, 1, 1, 0, 0)]:
        ho, wo = ctypes.c_int(), ctypes.c_int()
        assert L.fscnn_conv2d_out_shape(*bad, ctypes.byref(ho), ctypes.byref(wo)) == 2
    assert L.fscnn_conv2d_out_shape(5, 5, 3, 3, 1, 1, 0, 0, None, None) == 1
    for s in range(8):
        assert len(L.fscnn_status_string(s)) > 0
    assert L.fscnn_status_string(99) == L.fscnn_status_string(-1) != L.fscnn_status_string(7)   # any int is answered
    n = fscnn.sf_variant_count()
    assert n >= 1 and all(fscnn.sf_variant_name(v) for v in range(1, n + 1))
    assert fscnn.sf_variant_name(0) == "" and fscnn.sf_variant_name(n + 1) == ""


def test_argument_checks_come_before_device_work(L):
    h = ctypes.c_void_p()
    fake = ctypes.c_void_p(256)
    assert L.fscnn_filter_compress(None, 1, 1, 1, 1, None, ctypes.byref(h)) == 1
    assert L.fscnn_filter_compress(fake, 1, 1, 1, 1, None, None) == 1
    assert L.fscnn_filter_compress(fake, 0, 1, 3, 3, None, ctypes.byref(h)) == 2
    assert L.fscnn_filter_compress(fake, 1 << 16, 1 << 16, 3, 3, None, ctypes.byref(h)) == 2
    assert L.fscnn_input_compress(None, 1, 1, 1, 1, None, ctypes.byref(h)) == 1
    assert L.fscnn_input_compress(fake, 1, 1, 0, 1, None, ctypes.byref(h)) == 2
    assert L.fscnn_input_compress(fake, 1, 8193, 2, 2, None, ctypes.byref(h)) == 4      # more than 8192 channels
    assert L.fscnn_filter_destroy(None) == 1 and L.fscnn_input_destroy(None) == 1
    assert L.fscnn_conv2d_sparse_filter_emit(None, fake, 1, 1, 4, 4, 1, 1, 0, 0, None, 0, None, None,
                                             ctypes.byref(h)) == 1
    assert L.fscnn_conv2d_sparse_filter_emit(fake, fake, 1, 1, 4, 4, 1, 1, 0, 0, None, 0, None, None, None) == 1
    assert L.fscnn_maxpool2x2(None, 1, 1, 2, 2, fake, None) == 1
    assert L.fscnn_maxpool2x2(fake, 1, 1, 1, 2, fake, None) == 2
    assert L.fscnn_conv2d_sparse_filter(None, fake, 1, 1, 4, 4, 1, 1, 0, 0, None, 0, fake, None) == 1
    assert L.fscnn_conv2d_sparse_input(None, fake, 1, 3, 3, 1, 1, 0, 0, None, 0, fake, None) == 1
    assert L.fscnn_conv2d_sparse_filter_leaky(None, fake, 1, 1, 4, 4, 1, 1, 0, 0, None, ctypes.c_float(0.1), fake,
                                              0, 0, 0, None) == 1
    # a block of host memory that is not a handle is rejected by its magic word
    junk = (ctypes.c_ubyte * 512)()
    assert L.fscnn_filter_info(ctypes.byref(junk), None, None, None, None, None) == 7
    assert L.fscnn_conv2d_sparse_filter(ctypes.byref(junk), fake, 1, 1, 4, 4, 1, 1, 0, 0, None, 0,
                                        fake, None) == 7
    assert L.fscnn_input_info(ctypes.byref(junk), None, None, None, None, None) == 7
    assert L.fscnn_conv2d_sparse_filter_leaky(ctypes.byref(junk), fake, 1, 1, 4, 4, 1, 1, 0, 0, None,
                                              ctypes.c_float(2.0), fake, 0, 0, 0, None) == 2   # slope outside [0, 1]
    # transposes: workspace size is host arithmetic; argument checks precede any device work
    wsz = lambda rows, nnz: L.fscnn_sparse_transpose_workspace(ctypes.c_longlong(rows), ctypes.c_longlong(nnz))
    assert wsz(10, 0) >= 4 * 2 * 10 and wsz(10, 100) - wsz(10, 0) == 8 * 100    # O(new rows) + 8 bytes per node
    assert wsz(1 << 20, 1 << 20) < 64 << 20                                     # no rows x columns term
    assert wsz(0, 5) == -1 and wsz(10, -1) == -1 and wsz(1 << 40, 1 << 40) == -1
    ll = ctypes.c_longlong
    assert L.fscnn_sparse_transpose(None, fake, fake, 2, 2, ll(1), fake, fake, fake, fake, ll(1 << 20), None) == 1
    assert L.fscnn_sparse_transpose(fake, fake, fake, 0, 2, ll(1), fake, fake, fake, fake, ll(1 << 20), None) == 2
    assert L.fscnn_sparse_transpose(fake, fake, fake, 2, 2, ll(-1), fake, fake, fake, fake, ll(1 << 20), None) == 2
    assert L.fscnn_sparse_transpose(fake, fake, fake, 2, 2, ll(1), fake, fake, fake, fake, ll(8), None) == 4
    assert L.fscnn_sparse_tensor_transpose(fake, fake, fake, 2, 0, 2, ll(1), fake, fake, fake, fake, ll(1 << 20), None) == 2
    assert L.fscnn_sparse_tensor_transpose(fake, None, fake, 2, 2, 2, ll(1), fake, fake, fake, fake, ll(1 << 20), None) == 1
    assert L.fscnn_dense_filter_prepare(None, 1, 1, 3, 3, None, ctypes.byref(h)) == 1
    assert L.fscnn_dense_filter_prepare(fake, 1, 0, 3, 3, None, ctypes.byref(h)) == 2
    assert L.fscnn_dense_filter_destroy(None) == 1 and L.fscnn_dense_filter_destroy(ctypes.byref(junk)) == 7
    assert L.fscnn_conv2d_sparse_input_prepared(None, fake, 1, 1, 0, 0, None, 0, fake, 0, None) == 1
    assert L.fscnn_conv2d_sparse_input_prepared(ctypes.byref(junk), ctypes.byref(junk), 1, 1, 0, 0, None, 0,
                                                fake, 0, None) == 7
    assert L.fscnn_si_variant_count() >= 1
    v = ctypes.c_int()
    assert L.fscnn_sf_variant_choice(None, 1, 4, 4, 1, 1, 0, 0, ctypes.byref(v)) == 1
    assert L.fscnn_sf_variant_choice(ctypes.byref(junk), 1, 4, 4, 1, 1, 0, 0, None) == 1
    assert L.fscnn_sf_variant_choice(ctypes.byref(junk), 1, 4, 4, 1, 1, 0, 0, ctypes.byref(v)) == 7


def test_argument_checks_of_the_remaining_entry_points(L):
    fake = ctypes.c_void_p(256)
    odd = ctypes.c_void_p(260)          # not 16-byte aligned: the N4 layout needs float4 accesses
    junk = (ctypes.c_ubyte * 512)()
    jp = ctypes.byref(junk)
    ll = ctypes.c_longlong
    conv = (1, 1, 4, 4, 1, 1, 0, 0, None, 0)                    # N, C, H, W, stride, pad, bias, relu
    for fn in (L.fscnn_conv2d_sparse_filter_ex, L.fscnn_conv2d_sparse_filter_pool2x2):
        assert fn(None, fake, *conv, fake, 0, 0, 0, None) == 1
        assert fn(jp, fake, *conv, fake, 0, 0, 0, None) == 7
    assert L.fscnn_conv2d_sparse_filter_v(None, fake, *conv, fake, 0, None) == 1
    assert L.fscnn_conv2d_sparse_filter_v(jp, fake, *conv, fake, 0, None) == 7
    assert L.fscnn_conv2d_sparse_filter_emit_into(None, fake, *conv, None, None, jp) == 1
    assert L.fscnn_conv2d_sparse_filter_emit_into(jp, fake, *conv, None, None, None) == 1
    assert L.fscnn_conv2d_sparse_filter_emit_into(jp, fake, *conv, None, None, jp) == 7
    assert L.fscnn_filter_export(None, fake, fake, fake) == 1 and L.fscnn_filter_export(jp, fake, fake, fake) == 7
    assert L.fscnn_input_export(None, fake, fake, fake) == 1 and L.fscnn_input_export(jp, fake, fake, fake) == 7
    assert L.fscnn_filter_prepare(None, 1, 4, 4, 1, 1, 0, 0, 0, None) == 1
    assert L.fscnn_filter_prepare(jp, 1, 4, 4, 1, 1, 0, 0, 0, None) == 7
    assert L.fscnn_filter_prepare_ex(None, 1, 4, 4, 1, 1, 0, 0, 0, 0, 0, 0, None) == 1
    assert L.fscnn_filter_prepare_ex(jp, 1, 4, 4, 1, 1, 0, 0, 0, 0, 0, 0, None) == 7
    params = (ctypes.c_int * 16)()
    assert L.fscnn_filter_plan_export(None, 1, 4, 4, 1, 1, 0, 0, 0, params, None, None, None) == 1
    assert L.fscnn_filter_plan_export(jp, 1, 4, 4, 1, 1, 0, 0, 0, None, None, None, None) == 1
    assert L.fscnn_filter_plan_export(jp, 1, 4, 4, 1, 1, 0, 0, 0, params, None, None, None) == 7
    # layout conversion: NCHW <-> N4 only, out of place, N4 side aligned to 16 bytes
    other = ctypes.c_void_p(512)
    assert L.fscnn_layout_convert(None, 1, 1, 2, 2, 0, other, 1, None) == 1
    assert L.fscnn_layout_convert(fake, 0, 1, 2, 2, 0, other, 1, None) == 2
    assert L.fscnn_layout_convert(fake, 1, 1, 2, 2, 0, other, 0, None) == 4      # same layout on both sides
    assert L.fscnn_layout_convert(fake, 1, 1, 2, 2, 0, other, 7, None) == 4      # unknown layout code
    assert L.fscnn_layout_convert(fake, 1, 1, 2, 2, 0, fake, 1, None) == 4       # in place
    assert L.fscnn_layout_convert(fake, 1, 1, 2, 2, 0, odd, 1, None) == 4
    assert L.fscnn_layout_convert(fake, 1 << 15, 1 << 15, 2, 2, 0, other, 1, None) == 4   # 2^31 elements or more
    assert L.fscnn_maxpool2x2_ex(None, 1, 1, 2, 2, fake, 0, None) == 1
    assert L.fscnn_maxpool2x2_ex(fake, 1, 1, 2, 1, other, 0, None) == 2
    assert L.fscnn_maxpool2x2_ex(fake, 1, 1, 2, 2, other, 5, None) == 4
    assert L.fscnn_maxpool2x2_ex(fake, 1, 1, 2, 2, odd, 1, None) == 4
    # the transpose that allocates nothing refuses what its fixed scratch cannot hold
    na = L.fscnn_sparse_transpose_noalloc
    assert na(fake, fake, fake, 0, 2, ll(1), fake, fake, fake, None) == 2
    assert na(None, fake, fake, 2, 2, ll(1), fake, fake, fake, None) == 1
    assert na(fake, fake, fake, 2, 2, ll(-1), fake, fake, fake, None) == 2
    assert na(fake, fake, fake, 2, 2, ll(1 << 31), fake, fake, fake, None) == 2
    assert na(fake, fake, fake, 2, 2, ll((1 << 31) - 1), fake, fake, fake, None) == 4
    assert L.fscnn_sf_variant_count() >= 1
    bands, rows = ctypes.c_int(), ctypes.c_int()
    assert L.fscnn_sf_band_choice(1, 1, 8, 0, 0, None, ctypes.byref(rows)) == 1
    assert L.fscnn_sf_band_choice(1, 0, 8, 0, 0, ctypes.byref(bands), ctypes.byref(rows)) == 2
    assert L.fscnn_sf_band_choice(0, 1, 8, 0, 0, ctypes.byref(bands), ctypes.byref(rows)) == 4


def test_band_choice_is_host_arithmetic():
    from paper_2212_08815_amd import fscnn
    four = [v for v in range(1, fscnn.sf_variant_count() + 1) if fscnn.sf_variant_name(v).startswith("bv4")]
    other = [v for v in range(1, fscnn.sf_variant_count() + 1) if not fscnn.sf_variant_name(v).startswith("bv4")]
    assert four and other
    for v in four:
        assert fscnn.sf_band_choice(v, 1, 56) == (4, 14) and fscnn.sf_band_choice(v, 2, 56) == (2, 28)
        assert fscnn.sf_band_choice(v, 1, 14) == (4, 4) and fscnn.sf_band_choice(v, 1, 28, pool=True) == (4, 8)
        assert fscnn.sf_band_choice(v, 1, 1) == (4, 1) and fscnn.sf_band_choice(v, 2, 7, pool=True) == (2, 4)
        assert fscnn.sf_band_choice(v, 3, 56) == (1, 56) and fscnn.sf_band_choice(v, 32, 56) == (1, 56)
        assert fscnn.sf_band_choice(v, 1, 56, n4=True) == (1, 56)
    for v in other:
        assert fscnn.sf_band_choice(v, 1, 56) == (1, 56)


def test_no_cpu_fallback_without_a_device(L):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    h = ctypes.c_void_p()
    fake = ctypes.c_void_p(256)
    assert L.fscnn_filter_compress(fake, 2, 2, 3, 3, None, ctypes.byref(h)) == 6   # ERR_DEVICE
    assert L.fscnn_input_compress(fake, 1, 2, 3, 3, None, ctypes.byref(h)) == 6
    assert L.fscnn_maxpool2x2(fake, 1, 1, 2, 2, fake, None) == 6


def test_binding_refuses_cpu_tensors():
    import torch
    from paper_2212_08815_amd import fscnn
    with pytest.raises(TypeError):
        fscnn.filter_compress(torch.zeros(2, 2, 3, 3))
    with pytest.raises(TypeError):
        fscnn.input_compress(torch.zeros(1, 2, 3, 3))
