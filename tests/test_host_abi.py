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
    assert L.fscnn_sparse_transpose_workspace(10, 100) == 4 * (2 * 10 * 4 + 10)
    assert L.fscnn_sparse_transpose_workspace(0, 5) == -1 and L.fscnn_sparse_transpose_workspace(1 << 40, 1 << 40) == -1
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


def test_build_refuses_scratch_in_kernels_with_asynchronous_asm_loads():
    """The sparse-input kernel's inline-assembly loads fill registers long after they are issued; a
    register spilled in between would be saved before it is filled, so the build checks the
    compiler's resource report and fails if such a kernel uses scratch."""
    from paper_2212_08815_amd import build
    report = "\n".join([
        "x.hip:1:1: remark: Function Name: _ZN5fscnn17conv_si_kq_kernelINS_7SiKqCfgILi4ELi4ELi4ELi1EEEEEvPKi [-Rpass-analysis=kernel-resource-usage]",
        "x.hip:1:1: remark:     VGPRs: 128 [-Rpass-analysis=kernel-resource-usage]",
        "x.hip:1:1: remark:     ScratchSize [bytes/lane]: 28 [-Rpass-analysis=kernel-resource-usage]",
        "x.hip:2:1: remark: Function Name: _ZN5fscnn20conv_sf_tiled_kernelIS0_EEvPKf [-Rpass-analysis=kernel-resource-usage]",
        "x.hip:2:1: remark:     ScratchSize [bytes/lane]: 64 [-Rpass-analysis=kernel-resource-usage]",
        "x.hip:3:1: remark: Function Name: _ZN5fscnn17conv_si_kq_kernelINS_7SiKqCfgILi2ELi4ELi2ELi1EEEEEvPKi [-Rpass-analysis=kernel-resource-usage]",
        "x.hip:3:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]",
    ])
    bad = build._scratch_users(report)
    assert len(bad) == 1 and "Li4ELi4ELi4ELi1E" in bad[0] and "28 bytes/lane" in bad[0]
