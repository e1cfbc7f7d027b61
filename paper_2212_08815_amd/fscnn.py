"""Thin ctypes binding of libfscnn.so (C ABI in include/fscnn.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  torch is used for device memory (`data_ptr()`) and the current
stream.  There is no CPU fallback: if the library has not been built, or a call
returns an error status, an exception is raised.
"""
import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# FSCNN_LIB names another build of the same library (the host-sanitized one of build.py --sanitize-host)
LIB_PATH = os.environ.get("FSCNN_LIB") or os.path.join(_HERE, "libfscnn.so")
_lib = None

OK = 0
STATUS_NAMES = {0: "OK", 1: "ERR_NULL", 2: "ERR_SHAPE", 3: "ERR_MISMATCH", 4: "ERR_UNSUPPORTED",
                5: "ERR_ALLOC", 6: "ERR_DEVICE", 7: "ERR_HANDLE"}

# every symbol include/fscnn.h declares
EXPORTS = [
    "fscnn_status_string", "fscnn_conv2d_out_shape", "fscnn_filter_compress", "fscnn_filter_info",
    "fscnn_filter_export", "fscnn_filter_prepare", "fscnn_filter_plan_export",
    "fscnn_filter_destroy", "fscnn_sf_variant_count", "fscnn_sf_variant_name", "fscnn_sf_variant_choice",
    "fscnn_conv2d_sparse_filter", "fscnn_conv2d_sparse_filter_v", "fscnn_input_compress",
    "fscnn_conv2d_sparse_filter_emit",
    "fscnn_conv2d_sparse_filter_emit_into",
    "fscnn_input_info", "fscnn_input_export", "fscnn_input_destroy", "fscnn_conv2d_sparse_input",
    "fscnn_maxpool2x2", "fscnn_conv2d_sparse_filter_ex", "fscnn_layout_convert",
    "fscnn_maxpool2x2_ex", "fscnn_conv2d_sparse_filter_pool2x2",
    "fscnn_sparse_transpose", "fscnn_sparse_tensor_transpose", "fscnn_sparse_transpose_workspace",
    "fscnn_dense_filter_prepare", "fscnn_dense_filter_destroy", "fscnn_conv2d_sparse_input_prepared",
    "fscnn_si_variant_count", "fscnn_conv2d_sparse_filter_leaky", "fscnn_sparse_transpose_noalloc",
    "fscnn_filter_prepare_ex", "fscnn_sf_band_choice",
]

NCHW, N4 = 0, 1      # fscnn_layout_t


class FscnnError(RuntimeError):
    def __init__(self, status, what):
        self.status = int(status)
        msg = lib().fscnn_status_string(self.status).decode()
        super().__init__("%s: %s (%s)" % (what, STATUS_NAMES.get(self.status, self.status), msg))


def lib():
    """Loads libfscnn.so; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libfscnn.so is missing: run `python -m paper_2212_08815_amd.build` "
                               "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        L.fscnn_status_string.restype = ctypes.c_char_p
        L.fscnn_status_string.argtypes = [ctypes.c_int]
        L.fscnn_sf_variant_name.restype = ctypes.c_char_p
        L.fscnn_sf_variant_name.argtypes = [ctypes.c_int]
        L.fscnn_sf_variant_count.restype = ctypes.c_int
        L.fscnn_sparse_transpose_workspace.restype = ctypes.c_longlong
        L.fscnn_sparse_transpose_workspace.argtypes = [ctypes.c_longlong, ctypes.c_longlong]
        for name in EXPORTS:
            fn = getattr(L, name)
            if name not in ("fscnn_status_string", "fscnn_sf_variant_name", "fscnn_sf_variant_count",
                            "fscnn_sparse_transpose_workspace"):
                fn.restype = ctypes.c_int
        _lib = L
    return _lib


def _check(status, what):
    if status != OK:
        raise FscnnError(status, what)


def _ptr(t):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev_f32(t, name):
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise TypeError("%s must be a contiguous float32 CUDA tensor" % name)
    return t


def _i(v):
    return ctypes.c_int(int(v))


def conv2d_out_shape(H, W, R, S, stride=(1, 1), pad=(0, 0)):
    ho, wo = ctypes.c_int(), ctypes.c_int()
    _check(lib().fscnn_conv2d_out_shape(_i(H), _i(W), _i(R), _i(S), _i(stride[0]), _i(stride[1]),
                                        _i(pad[0]), _i(pad[1]), ctypes.byref(ho), ctypes.byref(wo)),
           "fscnn_conv2d_out_shape")
    return ho.value, wo.value


def sf_variant_count():
    return int(lib().fscnn_sf_variant_count())


def sf_variant_name(v):
    return lib().fscnn_sf_variant_name(int(v)).decode()


def sf_variant_choice(f, N, H, W, stride=(1, 1), n4=False, pool=False):
    """fscnn_sf_variant_choice -> variant id the automatic choice takes (-1 = direct kernel)."""
    v = ctypes.c_int(0)
    _check(lib().fscnn_sf_variant_choice(f.handle, _i(N), _i(H), _i(W), _i(stride[0]), _i(stride[1]),
                                         _i(1 if n4 else 0), _i(1 if pool else 0), ctypes.byref(v)),
           "fscnn_sf_variant_choice")
    return int(v.value)


def sf_band_choice(variant, N, Ho, n4=False, pool=False):
    """fscnn_sf_band_choice -> (bands per image, output rows per band) of a launch."""
    b, r = ctypes.c_int(0), ctypes.c_int(0)
    _check(lib().fscnn_sf_band_choice(_i(variant), _i(N), _i(Ho), _i(1 if n4 else 0), _i(1 if pool else 0),
                                      ctypes.byref(b), ctypes.byref(r)), "fscnn_sf_band_choice")
    return int(b.value), int(r.value)


class SparseFilter:
    """Owner of a fscnn_filter_t handle."""

    def __init__(self, handle, shape, nnz):
        self._h = handle
        self.shape = shape
        self.nnz = nnz

    def __del__(self):
        try:
            self.destroy()
        except Exception:        # interpreter shutdown: the module's globals may be gone already
            pass

    def destroy(self):
        if getattr(self, "_h", None):
            lib().fscnn_filter_destroy(self._h)
            self._h = None

    @property
    def handle(self):
        if not self._h:
            raise RuntimeError("filter handle already destroyed")
        return self._h


def filter_compress(w):
    """fscnn_filter_compress: dense K x C x R x S float32 CUDA tensor -> SparseFilter."""
    w = _dev_f32(w, "w")
    if w.dim() != 4:
        raise TypeError("w must be K x C x R x S")
    K, C, R, S = w.shape
    h = ctypes.c_void_p()
    _check(lib().fscnn_filter_compress(_ptr(w), _i(K), _i(C), _i(R), _i(S), _stream(), ctypes.byref(h)),
           "fscnn_filter_compress")
    nnz = ctypes.c_longlong()
    _check(lib().fscnn_filter_info(h, None, None, None, None, ctypes.byref(nnz)), "fscnn_filter_info")
    return SparseFilter(h, (K, C, R, S), nnz.value)


def filter_export(f):
    """fscnn_filter_export -> (rowptr int32[K+1], idx uint32[nnz], val float32[nnz]) numpy."""
    K = f.shape[0]
    rowptr = np.empty(K + 1, np.int32)
    idx = np.empty(f.nnz, np.uint32)
    val = np.empty(f.nnz, np.float32)
    _check(lib().fscnn_filter_export(f.handle, rowptr.ctypes.data_as(ctypes.c_void_p),
                                     idx.ctypes.data_as(ctypes.c_void_p),
                                     val.ctypes.data_as(ctypes.c_void_p)), "fscnn_filter_export")
    return rowptr, idx, val


def filter_prepare(f, N, H, W, stride=(1, 1), pad=(0, 0), variant=0, x_layout=NCHW, y_layout=NCHW, pool=False):
    """fscnn_filter_prepare_ex: plan (and, for small problems, the channel-split scratch of the
    current stream) of the convolution call with these arguments."""
    _check(lib().fscnn_filter_prepare_ex(f.handle, _i(N), _i(H), _i(W), _i(stride[0]), _i(stride[1]),
                                         _i(pad[0]), _i(pad[1]), _i(x_layout), _i(y_layout), _i(1 if pool else 0),
                                         _i(variant), _stream()),
           "fscnn_filter_prepare_ex")


def filter_plan_export(f, N, H, W, stride=(1, 1), pad=(0, 0), variant=0):
    """fscnn_filter_plan_export -> dict(params..., segptr, rec_off, rec_val)."""
    params = np.zeros(16, np.int32)
    args = (f.handle, _i(N), _i(H), _i(W), _i(stride[0]), _i(stride[1]), _i(pad[0]), _i(pad[1]),
            _i(variant))
    _check(lib().fscnn_filter_plan_export(*args, params.ctypes.data_as(ctypes.c_void_p), None, None, None),
           "fscnn_filter_plan_export")
    out = dict(variant=int(params[0]), CC=int(params[1]), KG=int(params[2]), NCH=int(params[3]),
               NG=int(params[4]), IN_ROWS=int(params[5]), PITCH=int(params[6]), BV=int(params[7]),
               nrec=int(params[8]), direct=bool(params[9]), SLOTS=int(params[10]),
               WAVES=int(params[11]), DENSE=int(params[12]))
    if out["direct"]:
        return out
    nb = out["NG"] * out["NCH"] * out["KG"]
    segptr = np.empty(nb + 1, np.int32)
    off = np.empty(out["nrec"], np.uint32)
    val = np.empty(out["nrec"], np.float32)
    _check(lib().fscnn_filter_plan_export(*args, params.ctypes.data_as(ctypes.c_void_p),
                                          segptr.ctypes.data_as(ctypes.c_void_p),
                                          off.ctypes.data_as(ctypes.c_void_p),
                                          val.ctypes.data_as(ctypes.c_void_p)),
           "fscnn_filter_plan_export")
    out.update(segptr=segptr, rec_off=off, rec_val=val)
    return out


def n4_shape(N, C, H, W):
    """Shape of the torch tensor that backs an N4 tensor of N images."""
    return ((N + 3) // 4, C, H, W, 4)


def _logical_shape(x, layout, n):
    if layout == NCHW:
        if x.dim() != 4:
            raise TypeError("an NCHW tensor must be N x C x H x W")
        return tuple(x.shape)
    if x.dim() != 5 or x.shape[4] != 4:
        raise TypeError("an N4 tensor must be ceil(N/4) x C x H x W x 4")
    n = x.shape[0] * 4 if n is None else n
    if (n + 3) // 4 != x.shape[0]:
        raise TypeError("n does not match the N4 tensor")
    return (n, x.shape[1], x.shape[2], x.shape[3])


def conv2d_sparse_filter(f, x, stride=(1, 1), pad=(0, 0), bias=None, relu=False, out=None, variant=0,
                         x_layout=NCHW, y_layout=NCHW, n=None, pool=False, leaky=None):
    """fscnn_conv2d_sparse_filter_ex (or, with pool=True, fscnn_conv2d_sparse_filter_pool2x2; or,
    with leaky=slope, fscnn_conv2d_sparse_filter_leaky): x -> y (CUDA float32).  NCHW tensors are
    N x C x H x W; N4 tensors are ceil(N/4) x C x H x W x 4 with `n` the number of real images."""
    x = _dev_f32(x, "x")
    bias = _dev_f32(bias, "bias")
    N, C, H, W = _logical_shape(x, x_layout, n)
    K, _, R, S = f.shape
    Ho, Wo = conv2d_out_shape(H, W, R, S, stride, pad)
    if pool:
        Ho, Wo = Ho // 2, Wo // 2
    oshape = (N, K, Ho, Wo) if y_layout == NCHW else n4_shape(N, K, Ho, Wo)
    if out is None:
        out = torch.empty(oshape, dtype=torch.float32, device=x.device)
    else:
        _dev_f32(out, "out")
        if tuple(out.shape) != oshape:
            raise TypeError("out has the wrong shape")
    if bias is not None and bias.numel() != K:
        raise TypeError("bias must have K entries")
    if leaky is not None:
        if pool or relu:
            raise TypeError("leaky excludes relu and pool")
        _check(lib().fscnn_conv2d_sparse_filter_leaky(
            f.handle, _ptr(x), _i(N), _i(C), _i(H), _i(W), _i(stride[0]), _i(stride[1]), _i(pad[0]), _i(pad[1]),
            _ptr(bias), ctypes.c_float(float(leaky)), _ptr(out), _i(x_layout), _i(y_layout), _i(variant),
            _stream()), "fscnn_conv2d_sparse_filter_leaky")
        return out
    fn = lib().fscnn_conv2d_sparse_filter_pool2x2 if pool else lib().fscnn_conv2d_sparse_filter_ex
    _check(fn(f.handle, _ptr(x), _i(N), _i(C), _i(H), _i(W), _i(stride[0]), _i(stride[1]), _i(pad[0]),
              _i(pad[1]), _ptr(bias), _i(bool(relu)), _ptr(out), _i(x_layout), _i(y_layout), _i(variant),
              _stream()),
           "fscnn_conv2d_sparse_filter_pool2x2" if pool else "fscnn_conv2d_sparse_filter_ex")
    return out


def layout_convert(x, src_layout, n=None):
    """fscnn_layout_convert: NCHW -> N4 or N4 -> NCHW (new tensor)."""
    x = _dev_f32(x, "x")
    N, C, H, W = _logical_shape(x, src_layout, n)
    dst_layout = N4 if src_layout == NCHW else NCHW
    out = torch.empty((N, C, H, W) if dst_layout == NCHW else n4_shape(N, C, H, W),
                      dtype=torch.float32, device=x.device)
    _check(lib().fscnn_layout_convert(_ptr(x), _i(N), _i(C), _i(H), _i(W), _i(src_layout), _ptr(out),
                                      _i(dst_layout), _stream()), "fscnn_layout_convert")
    return out


class SparseInput:
    """Owner of a fscnn_input_t handle.  `nnz` is asked of the library on first use (for a handle
    that a convolution emitted this waits for the pass that fills it)."""

    def __init__(self, handle, shape, nnz=None):
        self._h = handle
        self.shape = shape
        self._nnz = nnz

    @property
    def nnz(self):
        if self._nnz is None:
            n = ctypes.c_longlong()
            _check(lib().fscnn_input_info(self.handle, None, None, None, None, ctypes.byref(n)), "fscnn_input_info")
            self._nnz = n.value
        return self._nnz

    def __del__(self):
        try:
            self.destroy()
        except Exception:        # interpreter shutdown: the module's globals may be gone already
            pass

    def destroy(self):
        if getattr(self, "_h", None):
            lib().fscnn_input_destroy(self._h)
            self._h = None

    @property
    def handle(self):
        if not self._h:
            raise RuntimeError("input handle already destroyed")
        return self._h


def input_compress(x):
    """fscnn_input_compress: dense N x C x H x W float32 CUDA tensor -> SparseInput."""
    x = _dev_f32(x, "x")
    if x.dim() != 4:
        raise TypeError("x must be N x C x H x W")
    N, C, H, W = x.shape
    h = ctypes.c_void_p()
    _check(lib().fscnn_input_compress(_ptr(x), _i(N), _i(C), _i(H), _i(W), _stream(), ctypes.byref(h)),
           "fscnn_input_compress")
    nnz = ctypes.c_longlong()
    _check(lib().fscnn_input_info(h, None, None, None, None, ctypes.byref(nnz)), "fscnn_input_info")
    return SparseInput(h, (N, C, H, W), nnz.value)


def conv2d_sparse_filter_emit(f, x, stride=(1, 1), pad=(0, 0), bias=None, relu=False, dense_out=None,
                              into=None):
    """fscnn_conv2d_sparse_filter_emit: NCHW x -> SparseInput holding the non-zero results of the
    convolution.  dense_out, if given (N x K x Ho x Wo), also receives the dense result.  into, a
    SparseInput that an earlier call returned for the same shapes, is refilled and returned
    (fscnn_conv2d_sparse_filter_emit_into: no allocation)."""
    x = _dev_f32(x, "x")
    bias = _dev_f32(bias, "bias")
    if x.dim() != 4:
        raise TypeError("x must be N x C x H x W")
    N, C, H, W = x.shape
    K, _, R, S = f.shape
    Ho, Wo = conv2d_out_shape(H, W, R, S, stride, pad)
    if dense_out is not None:
        _dev_f32(dense_out, "dense_out")
        if tuple(dense_out.shape) != (N, K, Ho, Wo):
            raise TypeError("dense_out has the wrong shape")
    if bias is not None and bias.numel() != K:
        raise TypeError("bias must have K entries")
    if into is not None:
        _check(lib().fscnn_conv2d_sparse_filter_emit_into(
            f.handle, _ptr(x), _i(N), _i(C), _i(H), _i(W), _i(stride[0]), _i(stride[1]), _i(pad[0]), _i(pad[1]),
            _ptr(bias), _i(bool(relu)), _ptr(dense_out), _stream(), into.handle),
            "fscnn_conv2d_sparse_filter_emit_into")
        into._nnz = None
        return into
    h = ctypes.c_void_p()
    _check(lib().fscnn_conv2d_sparse_filter_emit(
        f.handle, _ptr(x), _i(N), _i(C), _i(H), _i(W), _i(stride[0]), _i(stride[1]), _i(pad[0]), _i(pad[1]),
        _ptr(bias), _i(bool(relu)), _ptr(dense_out), _stream(), ctypes.byref(h)),
        "fscnn_conv2d_sparse_filter_emit")
    return SparseInput(h, (N, K, Ho, Wo))


def input_export(s):
    N, C, H, W = s.shape
    prow = np.empty(N * H * W + 1, np.int32)
    cidx = np.empty(s.nnz, np.uint32)
    val = np.empty(s.nnz, np.float32)
    _check(lib().fscnn_input_export(s.handle, prow.ctypes.data_as(ctypes.c_void_p),
                                    cidx.ctypes.data_as(ctypes.c_void_p),
                                    val.ctypes.data_as(ctypes.c_void_p)), "fscnn_input_export")
    return prow, cidx, val


def conv2d_sparse_input(s, w, stride=(1, 1), pad=(0, 0), bias=None, relu=False, out=None):
    """fscnn_conv2d_sparse_input: compressed x, dense w K x C x R x S -> y N x K x Ho x Wo."""
    w = _dev_f32(w, "w")
    bias = _dev_f32(bias, "bias")
    N, C, H, W = s.shape
    if w.dim() != 4 or w.shape[1] != C:
        raise TypeError("w must be K x C x R x S with C matching the input")
    K, _, R, S = w.shape
    Ho, Wo = conv2d_out_shape(H, W, R, S, stride, pad)
    if out is None:
        out = torch.empty((N, K, Ho, Wo), dtype=torch.float32, device=w.device)
    elif tuple(out.shape) != (N, K, Ho, Wo):
        raise TypeError("out has the wrong shape")
    if bias is not None and bias.numel() != K:
        raise TypeError("bias must have K entries")
    _check(lib().fscnn_conv2d_sparse_input(s.handle, _ptr(w), _i(K), _i(R), _i(S), _i(stride[0]),
                                           _i(stride[1]), _i(pad[0]), _i(pad[1]), _ptr(bias),
                                           _i(bool(relu)), _ptr(_dev_f32(out, "out")), _stream()),
           "fscnn_conv2d_sparse_input")
    return out


class DenseFilter:
    """Owner of a fscnn_dense_t handle (K-contiguous copy of a dense filter bank)."""

    def __init__(self, handle, shape):
        self._h = handle
        self.shape = shape

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def destroy(self):
        if getattr(self, "_h", None):
            lib().fscnn_dense_filter_destroy(self._h)
            self._h = None

    @property
    def handle(self):
        if not self._h:
            raise RuntimeError("dense filter handle already destroyed")
        return self._h


def dense_filter_prepare(w):
    """fscnn_dense_filter_prepare: dense K x C x R x S CUDA tensor -> DenseFilter."""
    w = _dev_f32(w, "w")
    if w.dim() != 4:
        raise TypeError("w must be K x C x R x S")
    K, C, R, S = w.shape
    h = ctypes.c_void_p()
    _check(lib().fscnn_dense_filter_prepare(_ptr(w), _i(K), _i(C), _i(R), _i(S), _stream(), ctypes.byref(h)),
           "fscnn_dense_filter_prepare")
    return DenseFilter(h, (K, C, R, S))


def si_variant_count():
    return int(lib().fscnn_si_variant_count())


def conv2d_sparse_input_prepared(s, d, stride=(1, 1), pad=(0, 0), bias=None, relu=False, out=None, variant=0):
    """fscnn_conv2d_sparse_input_prepared: compressed x, prepared dense filters -> y N x K x Ho x Wo."""
    N, C, H, W = s.shape
    K, C2, R, S = d.shape
    Ho, Wo = conv2d_out_shape(H, W, R, S, stride, pad)
    bias = _dev_f32(bias, "bias")
    if out is None:
        out = torch.empty((N, K, Ho, Wo), dtype=torch.float32, device="cuda")
    _check(lib().fscnn_conv2d_sparse_input_prepared(s.handle, d.handle, _i(stride[0]), _i(stride[1]), _i(pad[0]),
                                                    _i(pad[1]), _ptr(bias), _i(1 if relu else 0), _ptr(out),
                                                    _i(variant), _stream()), "fscnn_conv2d_sparse_input_prepared")
    return out


def maxpool2x2(x, out=None, layout=NCHW, n=None):
    x = _dev_f32(x, "x")
    N, C, H, W = _logical_shape(x, layout, n)
    oshape = (N, C, H // 2, W // 2) if layout == NCHW else n4_shape(N, C, H // 2, W // 2)
    if out is None:
        out = torch.empty(oshape, dtype=torch.float32, device=x.device)
    _check(lib().fscnn_maxpool2x2_ex(_ptr(x), _i(N), _i(C), _i(H), _i(W), _ptr(out), _i(layout),
                                     _stream()), "fscnn_maxpool2x2_ex")
    return out


def _dev_i32(t, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()):
        raise TypeError("%s must be a contiguous int32 CUDA tensor" % name)
    return t


def sparse_transpose_workspace(new_rows, nnz):
    return int(lib().fscnn_sparse_transpose_workspace(int(new_rows), int(nnz)))


def _transpose(entry, rowptr, idx, val, dims, new_rows, workspace):
    rowptr, idx, val = _dev_i32(rowptr, "rowptr"), _dev_i32(idx, "idx"), _dev_f32(val, "val")
    nnz = idx.numel()
    if val.numel() != nnz:
        raise TypeError("idx and val must have one element per stored node")
    need = sparse_transpose_workspace(new_rows, nnz)
    if need < 0:
        raise FscnnError(4, entry)
    if workspace is None:
        workspace = torch.empty((need + 3) // 4, dtype=torch.int32, device=rowptr.device)
    tptr = torch.empty(new_rows + 1, dtype=torch.int32, device=rowptr.device)
    tidx = torch.empty(nnz, dtype=torch.int32, device=rowptr.device)
    tval = torch.empty(nnz, dtype=torch.float32, device=rowptr.device)
    _check(getattr(lib(), entry)(_ptr(rowptr), _ptr(idx), _ptr(val), *[_i(d) for d in dims],
                                 ctypes.c_longlong(nnz), _ptr(tptr), _ptr(tidx), _ptr(tval), _ptr(workspace),
                                 ctypes.c_longlong(workspace.numel() * workspace.element_size()), _stream()), entry)
    return tptr, tidx, tval


def sparse_transpose(rowptr, idx, val, n_rows, n_cols, workspace=None):
    """fscnn_sparse_transpose (Alg. 3).  rowptr/idx are int32 CUDA tensors (idx holds the u32
    column indices), val float32; returns (tptr, tidx, tval) CUDA tensors."""
    if rowptr.numel() != n_rows + 1:
        raise TypeError("rowptr must have n_rows + 1 elements")
    return _transpose("fscnn_sparse_transpose", rowptr, idx, val, (n_rows, n_cols), n_cols, workspace)


def sparse_transpose_noalloc(rowptr, idx, val, n_rows, n_cols, out):
    """fscnn_sparse_transpose_noalloc: as sparse_transpose, into the caller's `out` = (tptr, tidx,
    tval) tensors; the binding allocates nothing either."""
    rowptr, idx, val = _dev_i32(rowptr, "rowptr"), _dev_i32(idx, "idx"), _dev_f32(val, "val")
    tptr, tidx, tval = _dev_i32(out[0], "tptr"), _dev_i32(out[1], "tidx"), _dev_f32(out[2], "tval")
    nnz = idx.numel()
    if rowptr.numel() != n_rows + 1 or val.numel() != nnz:
        raise TypeError("rowptr must have n_rows + 1 elements, idx and val one per stored node")
    if tptr.numel() < n_cols + 1 or tidx.numel() < nnz or tval.numel() < nnz:
        raise TypeError("output tensors too small")
    _check(lib().fscnn_sparse_transpose_noalloc(_ptr(rowptr), _ptr(idx), _ptr(val), _i(n_rows), _i(n_cols),
                                                ctypes.c_longlong(nnz), _ptr(tptr), _ptr(tidx), _ptr(tval),
                                                _stream()), "fscnn_sparse_transpose_noalloc")
    return out


def sparse_tensor_transpose(rowptr, widx, val, W, H, C, workspace=None):
    """fscnn_sparse_tensor_transpose (Alg. 4): order O_whc (row c*H+h lists w) -> order O_chw
    (row w*H+h lists c)."""
    if rowptr.numel() != C * H + 1:
        raise TypeError("rowptr must have C*H + 1 elements")
    return _transpose("fscnn_sparse_tensor_transpose", rowptr, widx, val, (W, H, C), W * H, workspace)
