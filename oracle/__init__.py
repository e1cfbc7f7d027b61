"""ctypes front end of the CPU oracle (oracle/fscnn_oracle.c).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg import this package.  It never imports the HIP
library or its Python binding; it takes and returns numpy arrays only.

Every function below is a thin marshalling layer; the arithmetic lives in the C
file, whose header cites the passages of the paper it follows.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fscnn_oracle.c")
_LIB = os.path.join(_HERE, "libfscnn_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (-O2, OpenMP, no intrinsics).  With FSCNN_ORACLE_SANITIZE=1 in
    the environment a copy instrumented with -fsanitize=address,undefined is built and loaded
    instead (the process then needs gcc's libasan.so preloaded: see tests/README_sanitize.txt)."""
    san = os.environ.get("FSCNN_ORACLE_SANITIZE") == "1"
    lib = _LIB.replace(".so", "_asan.so") if san else _LIB
    if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(_SRC):
        tmp = lib + ".tmp%d" % os.getpid()
        flags = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                 "-fno-sanitize-recover=undefined"] if san else ["-O2"]
        subprocess.check_call(["gcc"] + flags + ["-std=c99", "-fopenmp", "-fPIC", "-shared",
                                                 "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, lib)
    return lib


_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_i32p = ctypes.POINTER(ctypes.c_int32)
_u32p = ctypes.POINTER(ctypes.c_uint32)
_i64p = ctypes.POINTER(ctypes.c_longlong)


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_count_nonzero.restype = ctypes.c_longlong
        _lib.oracle_input_compress.restype = ctypes.c_longlong
        _lib.oracle_out_dim.restype = ctypes.c_int
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _p(a, typ):
    if a is None:
        return None
    return a.ctypes.data_as(typ)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def num_threads():
    return int(_load().oracle_num_threads())


def out_dim(n, f, stride, pad):
    return int(_load().oracle_out_dim(int(n), int(f), int(stride), int(pad)))


def filter_compress(w):
    """dense K x C x R x S -> (rowptr int32[K+1], idx uint32[nnz], val float32[nnz])."""
    w = _f32(w)
    K, C, R, S = w.shape
    lib = _load()
    nnz = int(lib.oracle_count_nonzero(_p(w, _f32p), ctypes.c_longlong(w.size)))
    rowptr = np.zeros(K + 1, np.int32)
    idx = np.zeros(nnz, np.uint32)
    val = np.zeros(nnz, np.float32)
    lib.oracle_filter_compress(_p(w, _f32p), K, C, R, S, _p(rowptr, _i32p), _p(idx, _u32p), _p(val, _f32p))
    return rowptr, idx, val


def filter_decompress(rowptr, idx, val, shape):
    K, C, R, S = shape
    w = np.empty(shape, np.float32)
    _load().oracle_filter_decompress(_p(np.ascontiguousarray(rowptr, np.int32), _i32p),
                                     _p(np.ascontiguousarray(idx, np.uint32), _u32p),
                                     _p(_f32(val), _f32p), K, C, R, S, _p(w, _f32p))
    return w


def _act(relu, leaky):
    """Activation code of the C functions: 0 none, 1 ReLU, 2 LeakyReLU(leaky)."""
    if leaky is None:
        return int(bool(relu))
    assert not relu, "leaky excludes relu"
    _load().oracle_set_leaky_slope(ctypes.c_double(float(np.float32(leaky))))
    return 2


def _out_shape(x, K, R, S, stride, pad):
    N, C, H, W = x.shape
    return (N, K, out_dim(H, R, stride[0], pad[0]), out_dim(W, S, stride[1], pad[1]))


def conv2d_dense(x, w, stride=(1, 1), pad=(0, 0), bias=None, relu=False, want_abs=False, leaky=None):
    x, w = _f32(x), _f32(w)
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    assert C == C2
    bias = None if bias is None else _f32(bias)
    y = np.empty(_out_shape(x, K, R, S, stride, pad), np.float32)
    a = np.empty(y.shape, np.float64) if want_abs else None
    _load().oracle_conv2d_dense(_p(x, _f32p), N, C, H, W, _p(w, _f32p), K, R, S,
                                stride[0], stride[1], pad[0], pad[1],
                                _p(bias, _f32p), _act(relu, leaky), _p(y, _f32p), _p(a, _f64p))
    return (y, a) if want_abs else y


def conv2d_sparse_filter(x, csr, fshape, stride=(1, 1), pad=(0, 0), bias=None, relu=False,
                         want_abs=False, leaky=None):
    """csr = (rowptr, idx, val) as produced by filter_compress; fshape = (K, C, R, S)."""
    x = _f32(x)
    N, C, H, W = x.shape
    K, C2, R, S = fshape
    assert C == C2
    rowptr = np.ascontiguousarray(csr[0], np.int32)
    idx = np.ascontiguousarray(csr[1], np.uint32)
    val = _f32(csr[2])
    bias = None if bias is None else _f32(bias)
    y = np.empty(_out_shape(x, K, R, S, stride, pad), np.float32)
    a = np.empty(y.shape, np.float64) if want_abs else None
    rc = _load().oracle_conv2d_sparse_filter(_p(x, _f32p), N, C, H, W, _p(rowptr, _i32p),
                                             _p(idx, _u32p), _p(val, _f32p), K, R, S,
                                             stride[0], stride[1], pad[0], pad[1],
                                             _p(bias, _f32p), _act(relu, leaky), _p(y, _f32p),
                                             _p(a, _f64p))
    assert rc == 0
    return (y, a) if want_abs else y


def conv2d_points(x, w, flat, stride=(1, 1), pad=(0, 0), bias=None, relu=False, want_abs=False, leaky=None):
    """The dense definition at the flat output indices `flat` (into N x K x Ho x Wo)."""
    x, w = _f32(x), _f32(w)
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    assert C == C2
    flat = np.ascontiguousarray(flat, np.int64)
    bias = None if bias is None else _f32(bias)
    out = np.empty(flat.size, np.float32)
    a = np.empty(flat.size, np.float64) if want_abs else None
    _load().oracle_conv2d_points(_p(x, _f32p), N, C, H, W, _p(w, _f32p), K, R, S,
                                 stride[0], stride[1], pad[0], pad[1],
                                 _p(bias, _f32p), _act(relu, leaky),
                                 _p(flat, _i64p), ctypes.c_longlong(flat.size), _p(out, _f32p),
                                 _p(a, _f64p))
    return (out, a) if want_abs else out


def input_compress(x):
    """dense N x C x H x W -> (prow int32[N*H*W+1], cidx uint32[nnz], xval float32[nnz])."""
    x = _f32(x)
    N, C, H, W = x.shape
    lib = _load()
    prow = np.zeros(N * H * W + 1, np.int32)
    nnz = int(lib.oracle_input_compress(_p(x, _f32p), N, C, H, W, _p(prow, _i32p), None, None))
    cidx = np.zeros(nnz, np.uint32)
    xval = np.zeros(nnz, np.float32)
    lib.oracle_input_compress(_p(x, _f32p), N, C, H, W, _p(prow, _i32p), _p(cidx, _u32p), _p(xval, _f32p))
    return prow, cidx, xval


def input_decompress(prow, cidx, xval, shape):
    N, C, H, W = shape
    x = np.empty(shape, np.float32)
    _load().oracle_input_decompress(_p(np.ascontiguousarray(prow, np.int32), _i32p),
                                    _p(np.ascontiguousarray(cidx, np.uint32), _u32p),
                                    _p(_f32(xval), _f32p), N, C, H, W, _p(x, _f32p))
    return x


def conv2d_sparse_input(csr_x, xshape, w, stride=(1, 1), pad=(0, 0), bias=None, relu=False,
                        want_abs=False):
    N, C, H, W = xshape
    w = _f32(w)
    K, C2, R, S = w.shape
    assert C == C2
    prow = np.ascontiguousarray(csr_x[0], np.int32)
    cidx = np.ascontiguousarray(csr_x[1], np.uint32)
    xval = _f32(csr_x[2])
    bias = None if bias is None else _f32(bias)
    y = np.empty((N, K, out_dim(H, R, stride[0], pad[0]), out_dim(W, S, stride[1], pad[1])), np.float32)
    a = np.empty(y.shape, np.float64) if want_abs else None
    rc = _load().oracle_conv2d_sparse_input(_p(prow, _i32p), _p(cidx, _u32p), _p(xval, _f32p),
                                            N, C, H, W, _p(w, _f32p), K, R, S,
                                            stride[0], stride[1], pad[0], pad[1],
                                            _p(bias, _f32p), int(bool(relu)), _p(y, _f32p),
                                            _p(a, _f64p))
    assert rc == 0
    return (y, a) if want_abs else y


def maxpool2x2(x):
    x = _f32(x)
    N, C, H, W = x.shape
    y = np.empty((N, C, H // 2, W // 2), np.float32)
    _load().oracle_maxpool2x2(_p(x, _f32p), N, C, H, W, _p(y, _f32p))
    return y


def sparse_transpose(rowptr, idx, val, n_rows, n_cols):
    """Alg. 3: rows -> columns.  Returns (tptr int32[n_cols+1], tidx uint32[nnz], tval float32[nnz])."""
    rowptr = np.ascontiguousarray(rowptr, np.int32)
    idx = np.ascontiguousarray(idx, np.uint32)
    val = _f32(val)
    assert rowptr.shape == (n_rows + 1,) and idx.shape == val.shape == (int(rowptr[-1]),)
    nnz = int(rowptr[-1])
    tptr = np.zeros(n_cols + 1, np.int32)
    tidx = np.zeros(nnz, np.uint32)
    tval = np.zeros(nnz, np.float32)
    _load().oracle_sparse_transpose(_p(rowptr, _i32p), _p(idx, _u32p), _p(val, _f32p), n_rows, n_cols,
                                    _p(tptr, _i32p), _p(tidx, _u32p), _p(tval, _f32p))
    return tptr, tidx, tval


def sparse_tensor_transpose(rowptr, widx, val, W, H, C):
    """Alg. 4: order O_whc (row c*H+h lists w) -> order O_chw (row w*H+h lists c)."""
    rowptr = np.ascontiguousarray(rowptr, np.int32)
    widx = np.ascontiguousarray(widx, np.uint32)
    val = _f32(val)
    assert rowptr.shape == (C * H + 1,) and widx.shape == val.shape == (int(rowptr[-1]),)
    nnz = int(rowptr[-1])
    tptr = np.zeros(W * H + 1, np.int32)
    cidx = np.zeros(nnz, np.uint32)
    tval = np.zeros(nnz, np.float32)
    _load().oracle_sparse_tensor_transpose(_p(rowptr, _i32p), _p(widx, _u32p), _p(val, _f32p), W, H, C,
                                           _p(tptr, _i32p), _p(cidx, _u32p), _p(tval, _f32p))
    return tptr, cidx, tval
