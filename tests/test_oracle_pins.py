"""Pins of the CPU oracle against things other than itself (no GPU needed).

Each test fixes the oracle to something the paper or the mathematics determines:
brute force in a second formulation, impulse responses (orientation and index
packing), integer-exact data, special cases that reduce to a matrix product or a
dense library convolution, closed forms, numpy's nonzero() for the compressed
indices.  A dropped term, a flipped kernel, a swapped stride/pad axis or a
transposed index in oracle/fscnn_oracle.c fails at least one of them.
"""
import itertools

import numpy as np
import pytest
import torch

import oracle
from paper_2212_08815_amd import inputs


# --------------------------------------------------------------------------- sizes
def test_output_size_formula():
    # Alg. 1 step 3 / Alg. 6 step 3: (H_I - H_F)/S + 1 without padding
    assert oracle.out_dim(7, 3, 1, 0) == 5
    assert oracle.out_dim(7, 3, 2, 0) == 3
    assert oracle.out_dim(8, 3, 2, 0) == 3          # floor
    assert oracle.out_dim(5, 5, 1, 0) == 1
    # Sec. 5 "Other layers": padded 3x3 stride-1 output has the input's shape
    for n in (1, 2, 14, 224):
        assert oracle.out_dim(n, 3, 1, 1) == n
    assert oracle.out_dim(2, 3, 1, 0) == 0          # filter does not fit
    assert oracle.out_dim(224, 7, 2, 3) == 112


# --------------------------------------------------------------------------- brute force
def _brute(x, w, stride, pad, bias, relu):
    """Second formulation: explicit zero-padded copy, then a valid convolution."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    sh, sw = stride
    ph, pw = pad
    xp = [[[[0.0] * (W + 2 * pw) for _ in range(H + 2 * ph)] for _ in range(C)] for _ in range(N)]
    for n, c, i, j in itertools.product(range(N), range(C), range(H), range(W)):
        xp[n][c][i + ph][j + pw] = float(x[n, c, i, j])
    Ho = (H + 2 * ph - R) // sh + 1
    Wo = (W + 2 * pw - S) // sw + 1
    y = np.zeros((N, K, Ho, Wo), np.float32)
    for n, k, i, j in itertools.product(range(N), range(K), range(Ho), range(Wo)):
        a = 0.0
        for c in range(C):
            for r in range(R):
                for s in range(S):
                    a += float(w[k, c, r, s]) * xp[n][c][i * sh + r][j * sw + s]
        if bias is not None:
            a += float(bias[k])
        if relu:
            a = max(a, 0.0)
        y[n, k, i, j] = np.float32(a)
    return y


@pytest.mark.parametrize("stride", [(1, 1), (2, 2), (1, 2)])
@pytest.mark.parametrize("pad", [(0, 0), (1, 1), (2, 1)])
def test_brute_force_tiny(stride, pad):
    seed = stride[0] * 100 + stride[1] * 10 + pad[0] * 3 + pad[1]
    x, w, b = inputs.random_layer(seed, 2, 3, 3, 6, 5, 3, 2, keep=0.5)
    want = _brute(x, w, stride, pad, b, True)
    got = oracle.conv2d_dense(x, w, stride, pad, b, True)
    assert got.shape == want.shape
    # zero terms added in the same c,r,s order -> identical doubles -> identical floats
    assert np.array_equal(got, want)
    got2 = oracle.conv2d_sparse_filter(x, oracle.filter_compress(w), w.shape, stride, pad, b, True)
    assert np.array_equal(got2, want)


# --------------------------------------------------------------------------- impulses
def test_filter_impulse_copies_shifted_input():
    # w = single 1.0 at (k0,c0,r0,s0)  =>  y[n,k0,oy,ox] = x[n,c0,oy*s-p+r0,ox*s-p+s0]
    rng = np.random.default_rng(5)
    x = rng.standard_normal((2, 3, 7, 9)).astype(np.float32)
    for (k0, c0, r0, s0), (st, p) in itertools.product([(0, 0, 0, 0), (1, 2, 2, 1), (3, 1, 0, 2)],
                                                       [(1, 1), (2, 1), (1, 0)]):
        w = np.zeros((4, 3, 3, 3), np.float32)
        w[k0, c0, r0, s0] = 1.0
        y = oracle.conv2d_sparse_filter(x, oracle.filter_compress(w), w.shape, (st, st), (p, p))
        N, K, Ho, Wo = y.shape
        for oy in range(Ho):
            for ox in range(Wo):
                iy, ix = oy * st - p + r0, ox * st - p + s0
                want = x[:, c0, iy, ix] if (0 <= iy < 7 and 0 <= ix < 9) else np.zeros(2, np.float32)
                assert np.array_equal(y[:, k0, oy, ox], want)
        others = [k for k in range(4) if k != k0]
        assert not y[:, others].any()


def test_input_impulse_gives_unflipped_filter():
    # x = single 1.0 at (c0,y0,x0), stride 1: y[k,oy,ox] = w[k,c0,y0+p-oy,x0+p-ox]
    rng = np.random.default_rng(6)
    w = rng.standard_normal((3, 2, 3, 3)).astype(np.float32)
    x = np.zeros((1, 2, 8, 8), np.float32)
    c0, y0, x0, p = 1, 4, 3, 1
    x[0, c0, y0, x0] = 1.0
    y = oracle.conv2d_dense(x, w, (1, 1), (p, p))
    for k in range(3):
        for oy in range(8):
            for ox in range(8):
                r, s = y0 + p - oy, x0 + p - ox
                want = w[k, c0, r, s] if (0 <= r < 3 and 0 <= s < 3) else np.float32(0)
                assert y[0, k, oy, ox] == want
    # reading the patch around the impulse in raster order shows the filter reversed:
    # the operation is a cross-correlation, as Alg. 1's index pairing states
    patch = y[0, 0, y0 - 1:y0 + 2, x0 - 1:x0 + 2]
    assert np.array_equal(patch, w[0, c0, ::-1, ::-1])


# --------------------------------------------------------------------------- library / closed form
def _torch_conv(x, w, stride, pad, bias, relu):
    y = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                   None if bias is None else torch.from_numpy(bias).double(),
                                   stride=stride, padding=pad)
    if relu:
        y = torch.relu(y)
    return y.float().numpy()


@pytest.mark.parametrize("case", [
    dict(n=2, c=5, k=7, h=11, w_=13, r=3, s=3, stride=(1, 1), pad=(1, 1)),
    dict(n=1, c=4, k=3, h=12, w_=9, r=5, s=3, stride=(2, 1), pad=(2, 0)),
    dict(n=3, c=2, k=2, h=9, w_=9, r=1, s=1, stride=(2, 2), pad=(0, 0)),
    dict(n=1, c=8, k=8, h=10, w_=17, r=3, s=3, stride=(2, 2), pad=(1, 1)),
    dict(n=1, c=3, k=4, h=8, w_=8, r=2, s=4, stride=(1, 3), pad=(0, 2)),
])
def test_integer_data_equals_library_convolution_exactly(case):
    # small integers: every partial sum is an exact integer, so any summation order
    # (the library's included) gives the same float
    c = dict(case)
    stride, pad = c.pop("stride"), c.pop("pad")
    x, w, b = inputs.random_layer(7, keep=0.4, integer=True, **c)
    want = _torch_conv(x, w, stride, pad, b, True)
    got = oracle.conv2d_sparse_filter(x, oracle.filter_compress(w), w.shape, stride, pad, b, True)
    assert np.array_equal(got, want)


def test_real_data_close_to_library_convolution():
    x, w, b = inputs.random_layer(8, 2, 16, 8, 14, 14, 3, 3, keep=0.3)
    want = _torch_conv(x, w, (1, 1), (1, 1), b, False)
    got = oracle.conv2d_dense(x, w, (1, 1), (1, 1), b, False)
    # both round one fp64 sum to fp32; the sums differ by fp64 reassociation only
    assert np.max(np.abs(got - want)) <= 2e-7 * np.max(np.abs(want))


def test_one_by_one_is_matrix_product():
    x, w, _ = inputs.random_layer(9, 2, 6, 5, 4, 7, 1, 1, keep=0.5, integer=True, bias=False)
    got = oracle.conv2d_sparse_filter(x, oracle.filter_compress(w), w.shape)
    want = np.einsum("kc,ncp->nkp", w[:, :, 0, 0].astype(np.float64),
                     x.reshape(2, 6, -1).astype(np.float64)).reshape(2, 5, 4, 7)
    assert np.array_equal(got, want.astype(np.float32))


def test_all_ones_closed_form():
    # x = 1, w = 1: y = C * (#taps inside the image); interior 9C, edge 6C, corner 4C
    C = 5
    x = np.ones((1, C, 6, 7), np.float32)
    w = np.ones((2, C, 3, 3), np.float32)
    y = oracle.conv2d_dense(x, w, (1, 1), (1, 1))
    assert np.all(y[0, :, 1:-1, 1:-1] == 9 * C)
    assert np.all(y[0, :, 0, 1:-1] == 6 * C) and np.all(y[0, :, 1:-1, -1] == 6 * C)
    assert y[0, 0, 0, 0] == 4 * C and y[0, 1, -1, -1] == 4 * C
    # ramp input x[.,.,i,j] = j, filter = 1 at the right-hand tap only: y = j+1 (0 past the edge)
    xr = np.broadcast_to(np.arange(7, dtype=np.float32), (1, 1, 6, 7)).copy()
    wr = np.zeros((1, 1, 3, 3), np.float32)
    wr[0, 0, 1, 2] = 1
    yr = oracle.conv2d_dense(xr, wr, (1, 1), (1, 1))
    assert np.array_equal(yr[0, 0, 3], np.array([1, 2, 3, 4, 5, 6, 0], np.float32))


def test_zero_filter_bias_relu_and_linearity():
    x, w, b = inputs.random_layer(10, 1, 4, 6, 8, 8, 3, 3, keep=0.5, integer=True)
    z = np.zeros_like(w)
    y = oracle.conv2d_sparse_filter(x, oracle.filter_compress(z), z.shape, (1, 1), (1, 1), b, True)
    assert np.array_equal(y, np.broadcast_to(np.maximum(b, 0)[None, :, None, None], y.shape))
    # split the support into two disjoint halves: conv(w1) + conv(w2) == conv(w1 + w2)
    m = np.random.default_rng(3).random(w.shape) < 0.5
    y1 = oracle.conv2d_dense(x, np.where(m, w, 0), (1, 1), (1, 1))
    y2 = oracle.conv2d_dense(x, np.where(m, 0, w), (1, 1), (1, 1))
    assert np.array_equal(y1 + y2, oracle.conv2d_dense(x, w, (1, 1), (1, 1)))
    # bias is added before the ReLU, not after
    xb = np.zeros((1, 1, 3, 3), np.float32)
    wb = np.zeros((2, 1, 1, 1), np.float32)
    yb = oracle.conv2d_dense(xb, wb, bias=np.array([-2.0, 3.0], np.float32), relu=True)
    assert np.all(yb[0, 0] == 0) and np.all(yb[0, 1] == 3)


def test_leaky_relu_closed_form_and_against_the_pre_activation():
    """Sec. 5 "Other layers": the activation is element-wise on the output.  All-ones input and
    all-minus-one 3x3 filters: the pre-activation is -(taps inside the image) * C + bias, LeakyReLU
    multiplies the negative ones by the slope; positive outputs (large bias) pass unchanged."""
    C, H, W = 3, 5, 6
    x = np.ones((1, C, H, W), np.float32)
    w = -np.ones((2, C, 3, 3), np.float32)
    b = np.array([0.5, 100.0], np.float32)
    slope = 0.25                                       # exact in binary: no rounding in the product
    y = oracle.conv2d_dense(x, w, (1, 1), (1, 1), b, leaky=slope)
    ty = np.array([2] + [3] * (H - 2) + [2])
    tx = np.array([2] + [3] * (W - 2) + [2])
    pre = -(ty[:, None] * tx[None, :] * C).astype(np.float64)
    assert np.array_equal(y[0, 0], ((pre + 0.5) * slope).astype(np.float32))      # all negative
    assert np.array_equal(y[0, 1], (pre + 100.0).astype(np.float32))              # all positive
    # generic data: equal to the formula applied to the un-activated oracle output, within the
    # one extra rounding that route takes
    rng = np.random.default_rng(17)
    x = rng.standard_normal((2, 4, 7, 6)).astype(np.float32)
    w = rng.standard_normal((3, 4, 3, 3)).astype(np.float32)
    b = rng.standard_normal(3).astype(np.float32)
    pre = oracle.conv2d_dense(x, w, (1, 1), (1, 1), b)
    got = oracle.conv2d_dense(x, w, (1, 1), (1, 1), b, leaky=0.1)
    want = np.where(pre > 0, pre, pre.astype(np.float64) * float(np.float32(0.1)))
    assert np.all(np.abs(got - want) <= 2.0 ** -23 * np.abs(want)) and (got < 0).any() and (got > 0).any()
    assert np.array_equal(got > 0, pre > 0)
    flat = np.arange(0, got.size, 7)
    assert np.array_equal(oracle.conv2d_points(x, w, flat, (1, 1), (1, 1), b, leaky=0.1), got.ravel()[flat])
    assert np.array_equal(oracle.conv2d_dense(x, w, (1, 1), (1, 1), b, leaky=0.0), np.maximum(pre, 0))


def test_abs_sum_and_points_agree_with_full():
    x, w, b = inputs.random_layer(11, 2, 5, 4, 9, 8, 3, 3, keep=0.5)
    y, a = oracle.conv2d_dense(x, w, (2, 1), (1, 1), b, True, want_abs=True)
    aw = _torch_conv(np.abs(x), np.abs(w), (2, 1), (1, 1), np.abs(b), False)
    assert np.allclose(a, aw, rtol=1e-6)
    flat = np.random.default_rng(0).choice(y.size, 50, replace=False)
    yp, ap = oracle.conv2d_points(x, w, flat, (2, 1), (1, 1), b, True, want_abs=True)
    assert np.array_equal(yp, y.ravel()[flat]) and np.array_equal(ap, a.ravel()[flat])


# --------------------------------------------------------------------------- compressed forms
def test_filter_compress_is_csr_of_k_by_crs_matrix():
    c = inputs.config1()
    w = c["w"]
    rowptr, idx, val = oracle.filter_compress(w)
    K = w.shape[0]
    m = w.reshape(K, -1)
    rows, cols = np.nonzero(m)                      # row-major order = ascending flat index
    assert rowptr[0] == 0 and rowptr[-1] == rows.size == np.count_nonzero(w)
    assert np.array_equal(np.diff(rowptr), np.bincount(rows, minlength=K))
    assert np.array_equal(idx, cols.astype(np.uint32))
    assert np.array_equal(val.view(np.uint32), m[rows, cols].view(np.uint32))
    for k in range(K):
        seg = idx[rowptr[k]:rowptr[k + 1]].astype(np.int64)
        assert np.all(np.diff(seg) > 0)
    # flat index decodes as (c*R + r)*S + s
    k0 = int(rows[7])
    f = int(cols[7])
    cc, rr, ss = f // 9, (f // 3) % 3, f % 3
    assert w[k0, cc, rr, ss] == val[7]
    assert np.array_equal(oracle.filter_decompress(rowptr, idx, val, w.shape), w)


def test_filter_compress_special_values():
    w = np.zeros((2, 2, 1, 3), np.float32)
    w[0, 0, 0, 1] = -0.0
    w[0, 1, 0, 0] = np.nan
    w[1, 0, 0, 2] = np.float32(1e-42)               # denormal
    w[1, 1, 0, 1] = -3.5
    rowptr, idx, val = oracle.filter_compress(w)
    assert list(rowptr) == [0, 1, 3]
    assert list(idx) == [3, 2, 4]
    assert np.isnan(val[0]) and val[1] == np.float32(1e-42) and val[2] == -3.5
    back = oracle.filter_decompress(rowptr, idx, val, w.shape)
    assert not np.signbit(back[0, 0, 0, 1])         # -0.0 is not stored, comes back as +0.0
    # empty rows and an all-zero bank
    rp, ix, vl = oracle.filter_compress(np.zeros((3, 2, 3, 3), np.float32))
    assert list(rp) == [0, 0, 0, 0] and ix.size == 0 and vl.size == 0


def test_input_compress_is_per_pixel_channel_list():
    x, _, _ = inputs.random_layer(12, 2, 7, 1, 5, 6, 1, 1, keep=1.0, x_zero_frac=0.7)
    prow, cidx, xval = oracle.input_compress(x)
    m = np.transpose(x, (0, 2, 3, 1)).reshape(-1, 7)       # rows = pixels in (n,iy,ix) order
    rows, cols = np.nonzero(m)
    assert prow[0] == 0 and prow[-1] == rows.size
    assert np.array_equal(np.diff(prow), np.bincount(rows, minlength=m.shape[0]))
    assert np.array_equal(cidx, cols.astype(np.uint32))
    assert np.array_equal(xval, m[rows, cols])
    assert np.array_equal(oracle.input_decompress(prow, cidx, xval, x.shape), x)


def test_three_way_agreement_sparse_filter_sparse_input_dense():
    x, w, b = inputs.random_layer(13, 2, 6, 5, 7, 7, 3, 3, keep=0.3, x_zero_frac=0.6)
    d = oracle.conv2d_dense(x, w, (1, 1), (1, 1), b, True)
    sf = oracle.conv2d_sparse_filter(x, oracle.filter_compress(w), w.shape, (1, 1), (1, 1), b, True)
    si = oracle.conv2d_sparse_input(oracle.input_compress(x), x.shape, w, (1, 1), (1, 1), b, True)
    assert np.array_equal(d, sf) and np.array_equal(d, si)


def test_maxpool_helper():
    x = np.random.default_rng(1).standard_normal((2, 3, 7, 6)).astype(np.float32)
    y = oracle.maxpool2x2(x)
    want = x[:, :, :6, :6].reshape(2, 3, 3, 2, 3, 2).max(axis=(3, 5))
    assert y.shape == (2, 3, 3, 3) and np.array_equal(y, want)


# --------------------------------------------------------------------------- stored values
def test_golden_fixture_still_reproduced():
    """tests/golden/config1_oracle.txt is written by tests/golden/make_golden.py, which
    calls only oracle/; it guards the oracle (and the input generator) against drift."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "config1_oracle.txt")
    vals = {}
    with open(path) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, v = line.split("=")
            vals[key.strip()] = v.strip()
    c = inputs.config1()
    rowptr, idx, val = oracle.filter_compress(c["w"])
    y = oracle.conv2d_sparse_filter(c["x"], (rowptr, idx, val), c["w"].shape, c["stride"], c["pad"])
    assert int(vals["nnz"]) == rowptr[-1]
    assert int(vals["idx_sum"]) == int(idx.astype(np.int64).sum())
    assert vals["rowptr_head"] == " ".join(str(v) for v in rowptr[:8])
    probe = [float(v) for v in vals["y_probe"].split()]
    pos = [int(v) for v in vals["y_probe_flat"].split()]
    assert np.array_equal(np.array(probe, np.float32), y.ravel()[pos])


# ------------------------------------------------------------------ sparse transposes (Alg. 3, Alg. 4)
def _csr_of(dense2d):
    """Row-major compressed form of a 2-D array, built with numpy only (nonzero() walks row-major)."""
    r, c = np.nonzero(dense2d)
    ptr = np.zeros(dense2d.shape[0] + 1, np.int32)
    np.add.at(ptr, r + 1, 1)
    return np.cumsum(ptr).astype(np.int32), c.astype(np.uint32), dense2d[r, c].astype(np.float32)


@pytest.mark.parametrize("shape,keep,seed", [((1, 1), 1.0, 0), ((5, 7), 0.4, 1), ((64, 33), 0.1, 2),
                                             ((9, 200), 0.03, 3), ((40, 40), 1.0, 4), ((6, 6), 0.0, 5)])
def test_matrix_transpose_is_the_library_csc_conversion(shape, keep, seed):
    import scipy.sparse as sp
    rng = np.random.default_rng(seed)
    m = (rng.standard_normal(shape) * (rng.random(shape) < keep)).astype(np.float32)
    ptr, idx, val = _csr_of(m)
    tptr, tidx, tval = oracle.sparse_transpose(ptr, idx, val, *shape)
    # pin 1: a library's CSR -> CSC conversion (CSC of M = the rows of M^T), indices sorted
    lib = sp.csr_matrix((val, idx.astype(np.int32), ptr), shape=shape).tocsc()
    lib.sort_indices()
    assert np.array_equal(tptr, lib.indptr) and np.array_equal(tidx, lib.indices.astype(np.uint32))
    assert np.array_equal(tval.view(np.uint32), lib.data.astype(np.float32).view(np.uint32))
    # pin 2: the compressed form of the dense transpose, built with numpy only
    p2, i2, v2 = _csr_of(np.ascontiguousarray(m.T))
    assert np.array_equal(tptr, p2) and np.array_equal(tidx, i2) and np.array_equal(tval, v2)
    # pin 3: transposing twice gives the matrix back
    bptr, bidx, bval = oracle.sparse_transpose(tptr, tidx, tval, shape[1], shape[0])
    assert np.array_equal(bptr, ptr) and np.array_equal(bidx, idx) and np.array_equal(bval, val)


def test_matrix_transpose_keeps_stored_values_bit_for_bit():
    # stored entries are whatever the caller stored: NaN, -0.0 and denormals travel unchanged
    ptr = np.array([0, 2, 2, 4], np.int32)
    idx = np.array([0, 3, 1, 3], np.uint32)
    val = np.array([np.nan, -0.0, 1e-42, np.inf], np.float32)
    tptr, tidx, tval = oracle.sparse_transpose(ptr, idx, val, 3, 4)
    assert tptr.tolist() == [0, 1, 2, 2, 4] and tidx.tolist() == [0, 2, 0, 2]
    assert tval.view(np.uint32).tolist() == val[[0, 2, 1, 3]].view(np.uint32).tolist()


@pytest.mark.parametrize("W,H,C,keep,seed", [(1, 1, 1, 1.0, 0), (4, 3, 5, 0.5, 1), (14, 14, 40, 0.3, 2),
                                             (7, 9, 3, 1.0, 3), (6, 5, 8, 0.0, 4), (33, 2, 17, 0.1, 5)])
def test_tensor_transpose_whc_to_chw(W, H, C, keep, seed):
    rng = np.random.default_rng(seed)
    t = (rng.standard_normal((C, H, W)) * (rng.random((C, H, W)) < keep)).astype(np.float32)   # t[c, h, w]
    # order O_whc: w runs innermost, then h, then c = the rows (c, h) of the C x H x W array
    ptr, widx, val = _csr_of(t.reshape(C * H, W))
    tptr, cidx, tval = oracle.sparse_tensor_transpose(ptr, widx, val, W, H, C)
    # pin 1: order O_chw = rows (w, h) listing c: the compressed form of the array permuted to [w, h, c]
    p2, i2, v2 = _csr_of(np.ascontiguousarray(t.transpose(2, 1, 0)).reshape(W * H, C))
    assert np.array_equal(tptr, p2) and np.array_equal(cidx, i2) and np.array_equal(tval, v2)
    # pin 2: brute force in Python, visiting (w, h, c) in the target order
    want = [(w * H + h, c, t[c, h, w]) for w in range(W) for h in range(H) for c in range(C) if t[c, h, w] != 0]
    rows = np.repeat(np.arange(W * H), np.diff(tptr))
    assert [(int(r), int(c), v) for r, c, v in zip(rows, cidx, tval)] == want
    # pin 3: a single Alg. 3 transpose of the (c*H + h) x w matrix has the same entries per column w
    mptr, midx, mval = oracle.sparse_transpose(ptr, widx, val, C * H, W)
    assert int(mptr[-1]) == int(tptr[-1])
    for w in range(W):
        a = sorted((int(r) % H, int(r) // H) for r in midx[mptr[w]:mptr[w + 1]])        # (h, c) pairs
        b = sorted((h, int(c)) for h in range(H) for c in cidx[tptr[w * H + h]:tptr[w * H + h + 1]])
        assert a == b
