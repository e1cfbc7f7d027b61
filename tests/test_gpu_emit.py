"""GPU parity for the sparse-filter convolution that returns its result compressed (Sec. 4,
sparse outputs: only non-zero results become nodes).  The stored structure is integer work and
must match bit for bit once both sides decide "non-zero" on the same fp32 numbers; the values
follow the fp32 rule of tests/parity.py."""
import numpy as np
import pytest
import torch

import oracle
from paper_2212_08815_amd import inputs
from parity import assert_parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def F():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2212_08815_amd import fscnn
    fscnn.lib()
    return fscnn


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def bits(a):
    return np.ascontiguousarray(a, np.float32).view(np.uint32)


def densify(prow, cidx, val, shape):
    """Pixel rows of (channel, value) pairs -> dense N x K x H x W (zeros elsewhere)."""
    n, k, h, w = shape
    y = np.zeros((n, h, w, k), np.float32)
    flat = y.reshape(n * h * w, k)
    rows = np.repeat(np.arange(n * h * w), np.diff(prow))
    flat[rows, cidx] = val
    return np.ascontiguousarray(y.transpose(0, 3, 1, 2))


CASES = [
    (2, 19, 37, 11, 23, 3, 3, (1, 1), (1, 1)),      # ragged everything
    (1, 40, 70, 28, 28, 3, 3, (1, 1), (1, 1)),      # several tiles
    (5, 16, 64, 14, 14, 3, 3, (1, 1), (1, 1)),      # batch with a ragged group of four
    (2, 24, 16, 17, 15, 3, 3, (2, 2), (1, 1)),      # stride 2
    (1, 33, 20, 9, 12, 1, 1, (1, 1), (0, 0)),       # 1x1 filters
    (1, 7, 66, 10, 9, 5, 2, (1, 2), (2, 0)),        # direct kernel
    (16, 72, 96, 56, 56, 3, 3, (1, 1), (1, 1)),     # many chunks and enough work-groups not to split: epilogue counts
    (1, 128, 40, 14, 14, 3, 3, (1, 1), (1, 1)),     # small and deep: channel-split mode, counted in a separate pass
]


@pytest.mark.parametrize("case", CASES)
def test_emit_integer_data_bit_exact(F, case):
    n, c, k, h, w_, r, s_, stride, pad = case
    x, w, b = inputs.random_layer(300 + c + k, n, c, k, h, w_, r, s_, keep=0.4, integer=True)
    want = oracle.conv2d_dense(x, w, stride, pad, b, True)          # exact in fp32
    op, oc, ov = oracle.input_compress(want)
    s = F.conv2d_sparse_filter_emit(F.filter_compress(dev(w)), dev(x), stride, pad, dev(b), True)
    assert s.shape == want.shape and s.nnz == op[-1]
    prow, cidx, val = F.input_export(s)
    assert np.array_equal(prow, op) and np.array_equal(cidx, oc) and np.array_equal(bits(val), bits(ov))


@pytest.mark.parametrize("case", CASES)
def test_emit_random_data_matches_oracle(F, case):
    n, c, k, h, w_, r, s_, stride, pad = case
    x, w, b = inputs.random_layer(400 + c + k, n, c, k, h, w_, r, s_, keep=0.3)
    o, a = oracle.conv2d_dense(x, w, stride, pad, b, True, want_abs=True)
    f = F.filter_compress(dev(w))
    yd = torch.empty(o.shape, dtype=torch.float32, device="cuda")
    s = F.conv2d_sparse_filter_emit(f, dev(x), stride, pad, dev(b), True, dense_out=yd)
    prow, cidx, val = F.input_export(s)
    yd = host(yd)
    # values: the dense result and the compressed one, both against the oracle
    assert_parity(yd, o, a, c * r * s_, "emit dense %r" % (case,))
    assert_parity(densify(prow, cidx, val, o.shape), o, a, c * r * s_, "emit compressed %r" % (case,))
    # structure: which results count as non-zero is decided on the kernel's fp32 numbers, so the
    # oracle compresses those; the answer is unique
    op, oc, ov = oracle.input_compress(yd)
    assert np.array_equal(prow, op) and np.array_equal(cidx, oc) and np.array_equal(bits(val), bits(ov))
    # ... and wherever the exact result is clear of zero by more than the rounding bound, the
    # decision agrees with the oracle's own
    pre, pa = oracle.conv2d_dense(x, w, stride, pad, b, False, want_abs=True)
    clear = np.abs(pre) > (c * r * s_ + 2) * 2.0 ** -22 * pa
    assert clear.mean() > 0.9
    assert np.array_equal((yd != 0)[clear], (pre > 0)[clear])
    # without the dense copy: the same handle contents, bit for bit (one writer per output element)
    s2 = F.conv2d_sparse_filter_emit(f, dev(x), stride, pad, dev(b), True)
    p2, c2, v2 = F.input_export(s2)
    assert np.array_equal(p2, prow) and np.array_equal(c2, cidx) and np.array_equal(bits(v2), bits(val))


def test_emit_chains_into_the_sparse_input_convolution(F):
    x, w1, b1 = inputs.random_layer(501, 3, 24, 40, 28, 28, 3, 3, keep=0.2)
    _, w2, b2 = inputs.random_layer(502, 3, 40, 72, 28, 28, 3, 3, keep=1.0)
    mid = F.conv2d_sparse_filter_emit(F.filter_compress(dev(w1)), dev(x), (1, 1), (1, 1), dev(b1), True)
    d = F.dense_filter_prepare(dev(w2))
    g = host(F.conv2d_sparse_input_prepared(mid, d, (1, 1), (1, 1), dev(b2), True))
    o1 = oracle.conv2d_dense(x, w1, (1, 1), (1, 1), b1, True)
    cs = oracle.input_compress(o1)
    o2, a2 = oracle.conv2d_sparse_input(cs, o1.shape, w2, (1, 1), (1, 1), b2, True, want_abs=True)
    # two layers: the first layer's rounding enters the second as an input perturbation
    assert_parity(g, o2, a2, 24 * 9 + 40 * 9, "emit -> sparse input chain")
    # and against the oracle fed the first layer's result as the GPU computed it
    m = densify(*F.input_export(mid), o1.shape)
    o3, a3 = oracle.conv2d_dense(m, w2, (1, 1), (1, 1), b2, True, want_abs=True)
    assert_parity(g, o3, a3, 40 * 9, "sparse input on the emitted tensor")


def test_emit_into_refills_a_handle_without_allocating(F):
    n, c, k, h, w_ = 5, 24, 37, 19, 21
    x1, w, b = inputs.random_layer(520, n, c, k, h, w_, 3, 3, keep=0.3)
    x2 = inputs.random_layer(521, n, c, k, h, w_, 3, 3, keep=0.3)[0]
    f = F.filter_compress(dev(w))
    s = F.conv2d_sparse_filter_emit(f, dev(x1), (1, 1), (1, 1), dev(b), True)
    first = F.input_export(s)
    for x in (x2, x1):                       # other contents (another count of non-zeros), then back
        fresh = F.input_export(F.conv2d_sparse_filter_emit(f, dev(x), (1, 1), (1, 1), dev(b), True))
        free0 = torch.cuda.mem_get_info()[0]
        again = F.conv2d_sparse_filter_emit(f, dev(x), (1, 1), (1, 1), dev(b), True, into=s)
        assert again is s and torch.cuda.mem_get_info()[0] == free0
        got = F.input_export(s)
        assert s.nnz == fresh[0][-1]
        assert all(np.array_equal(bits(g) if g.dtype == np.float32 else g,
                                  bits(e) if e.dtype == np.float32 else e) for g, e in zip(got, fresh))
    assert all(np.array_equal(g, e) for g, e in zip(got, first))
    yd = torch.empty((n, k, h, w_), dtype=torch.float32, device="cuda")
    F.conv2d_sparse_filter_emit(f, dev(x2), (1, 1), (1, 1), dev(b), True, dense_out=yd, into=s)
    op, oc, ov = oracle.input_compress(host(yd))
    prow, cidx, val = F.input_export(s)
    assert np.array_equal(prow, op) and np.array_equal(cidx, oc) and np.array_equal(bits(val), bits(ov))
    # a handle of another shape or origin is refused; one made with a dense_out has no room for y
    with pytest.raises(F.FscnnError) as e:
        F.conv2d_sparse_filter_emit(f, dev(x1[:4]), (1, 1), (1, 1), dev(b), True, into=s)
    assert e.value.status == 3
    with pytest.raises(F.FscnnError) as e:
        F.conv2d_sparse_filter_emit(f, dev(x1), (1, 1), (1, 1), dev(b), True, into=F.input_compress(yd))
    assert e.value.status == 4
    s3 = F.conv2d_sparse_filter_emit(f, dev(x1), (1, 1), (1, 1), dev(b), True, dense_out=yd)
    with pytest.raises(F.FscnnError) as e:
        F.conv2d_sparse_filter_emit(f, dev(x1), (1, 1), (1, 1), dev(b), True, into=s3)
    assert e.value.status == 1


def test_emit_nothing_and_everything(F):
    x, w, _ = inputs.random_layer(510, 2, 8, 12, 9, 7, 3, 3, keep=0.5)
    f = F.filter_compress(dev(w))
    low = np.full(12, -1e6, np.float32)
    s = F.conv2d_sparse_filter_emit(f, dev(x), (1, 1), (1, 1), dev(low), True)       # ReLU clips all
    prow, cidx, val = F.input_export(s)
    assert s.nnz == 0 and not prow.any() and cidx.size == 0 and val.size == 0
    high = np.full(12, 1e3, np.float32)
    s = F.conv2d_sparse_filter_emit(f, dev(x), (1, 1), (1, 1), dev(high), False)     # all kept
    prow, cidx, val = F.input_export(s)
    assert s.nnz == 2 * 12 * 9 * 7
    assert np.array_equal(prow, 12 * np.arange(2 * 9 * 7 + 1))
    assert np.array_equal(cidx.reshape(-1, 12), np.tile(np.arange(12, dtype=np.uint32), (2 * 9 * 7, 1)))
    o, a = oracle.conv2d_dense(x, w, (1, 1), (1, 1), high, False, want_abs=True)
    assert_parity(densify(prow, cidx, val, o.shape), o, a, 8 * 9, "emit, everything kept")


def test_emit_rejects_bad_arguments(F):
    x, w, b = inputs.random_layer(511, 1, 6, 6, 8, 8, 3, 3, keep=0.5)
    f = F.filter_compress(dev(w))
    with pytest.raises(F.FscnnError) as e:
        F.conv2d_sparse_filter_emit(f, dev(x[:, :5]), (1, 1), (1, 1))        # C differs from the handle's
    assert e.value.status == 3
    with pytest.raises(F.FscnnError) as e:
        F.conv2d_sparse_filter_emit(f, dev(x), (1, 1), (-1, 0))
    assert e.value.status == 2
    xd = dev(x)
    with pytest.raises(F.FscnnError) as e:
        F.conv2d_sparse_filter_emit(f, xd, (1, 1), (1, 1), dense_out=xd)     # dense copy on top of x
    assert e.value.status == 4
