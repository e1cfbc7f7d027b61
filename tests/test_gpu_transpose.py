"""GPU parity of the sparse transposes (Alg. 3, Alg. 4) against the oracle, through the C ABI.
Integer and copy work only: every array must match bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2212_08815_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def F():
    from paper_2212_08815_amd import fscnn
    fscnn.lib()
    assert torch.cuda.is_available()
    return fscnn


def csr_of(dense2d):
    r, c = np.nonzero(dense2d)
    ptr = np.zeros(dense2d.shape[0] + 1, np.int64)
    np.add.at(ptr, r + 1, 1)
    return np.cumsum(ptr).astype(np.int32), c.astype(np.uint32), dense2d[r, c].astype(np.float32)


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int32) if a.dtype == np.uint32 else np.ascontiguousarray(a, np.int32)).cuda()


def same(got, want):
    tptr, tidx, tval = (t.cpu().numpy() for t in got)
    assert np.array_equal(tptr, want[0])
    assert np.array_equal(tidx.view(np.uint32), want[1])
    assert np.array_equal(tval.view(np.uint32), want[2].view(np.uint32))


@pytest.mark.parametrize("shape,keep,seed", [((1, 1), 1.0, 0), ((5, 7), 0.4, 1), ((64, 33), 0.1, 2), ((9, 2000), 0.03, 3),
                                             ((300, 300), 1.0, 4), ((6, 6), 0.0, 5), ((1, 4097), 0.5, 6),
                                             ((4097, 1), 0.5, 7), ((1000, 70), 0.002, 8), ((7, 40000), 0.01, 9)])
def test_matrix_transpose_matches_oracle(F, shape, keep, seed):
    rng = np.random.default_rng(seed)
    m = (rng.standard_normal(shape) * (rng.random(shape) < keep)).astype(np.float32)
    ptr, idx, val = csr_of(m)
    want = oracle.sparse_transpose(ptr, idx, val, *shape)
    got = F.sparse_transpose(dev_i32(ptr), dev_i32(idx), torch.from_numpy(val).cuda(), *shape)
    torch.cuda.synchronize()
    same(got, want)
    back = F.sparse_transpose(got[0], got[1], got[2], shape[1], shape[0])       # twice = identity
    same(back, (ptr, idx, val))


def test_matrix_transpose_of_a_compressed_filter_bank_and_special_values(F):
    # the K x (C*R*S) matrix of a 95 % sparse 512x512x3x3 filter bank, as the library compresses it
    _, w, _ = inputs.random_layer(3, 1, 512, 512, 4, 4, 3, 3, keep=0.05)
    f = F.filter_compress(torch.from_numpy(w).cuda())
    ptr, idx, val = F.filter_export(f)
    want = oracle.sparse_transpose(ptr, idx, val, 512, 512 * 9)
    same(F.sparse_transpose(dev_i32(ptr), dev_i32(idx), torch.from_numpy(val).cuda(), 512, 512 * 9), want)
    # NaN, -0.0, denormal, Inf travel unchanged; a workspace the caller brings is accepted
    ptr = np.array([0, 2, 2, 4], np.int32)
    idx = np.array([0, 3, 1, 3], np.uint32)
    val = np.array([np.nan, -0.0, 1e-42, np.inf], np.float32)
    ws = torch.empty(F.sparse_transpose_workspace(4, 4) // 4 + 1, dtype=torch.int32, device="cuda")
    same(F.sparse_transpose(dev_i32(ptr), dev_i32(idx), torch.from_numpy(val).cuda(), 3, 4, workspace=ws),
         oracle.sparse_transpose(ptr, idx, val, 3, 4))
    small = torch.empty(2, dtype=torch.int32, device="cuda")
    with pytest.raises(F.FscnnError) as e:
        F.sparse_transpose(dev_i32(ptr), dev_i32(idx), torch.from_numpy(val).cuda(), 3, 4, workspace=small)
    assert e.value.status == 4


@pytest.mark.parametrize("W,H,C,keep,seed", [(1, 1, 1, 1.0, 0), (4, 3, 5, 0.5, 1), (14, 14, 40, 0.3, 2), (7, 9, 3, 1.0, 3),
                                             (6, 5, 8, 0.0, 4), (33, 2, 17, 0.1, 5), (28, 28, 512, 0.31, 6),
                                             (56, 56, 70, 0.05, 7), (150, 131, 9, 0.2, 8)])  # 19 650 new rows: tiled scan
def test_tensor_transpose_matches_oracle(F, W, H, C, keep, seed):
    rng = np.random.default_rng(seed)
    t = (rng.standard_normal((C, H, W)) * (rng.random((C, H, W)) < keep)).astype(np.float32)
    ptr, widx, val = csr_of(t.reshape(C * H, W))
    want = oracle.sparse_tensor_transpose(ptr, widx, val, W, H, C)
    got = F.sparse_tensor_transpose(dev_i32(ptr), dev_i32(widx), torch.from_numpy(val).cuda(), W, H, C)
    torch.cuda.synchronize()
    same(got, want)


def test_tensor_transpose_chains_with_the_activation_compressor(F):
    # O_chw of x[c, h, w] read with the roles of h and w swapped is the per-pixel channel list in
    # raster order, i.e. what fscnn_input_compress produces for the same image
    rng = np.random.default_rng(11)
    C, H, W = 48, 12, 20
    x = np.maximum(rng.standard_normal((1, C, H, W)) - 0.5, 0).astype(np.float32)
    prow, cidx, xval = F.input_export(F.input_compress(torch.from_numpy(x).cuda()))
    xt = np.ascontiguousarray(x[0].transpose(0, 2, 1))                   # [c, w, h]: "height" := w, "width" := h
    ptr, hidx, val = csr_of(xt.reshape(C * W, H))
    got = F.sparse_tensor_transpose(dev_i32(ptr), dev_i32(hidx), torch.from_numpy(val).cuda(), H, W, C)
    same(got, (prow, cidx, xval))


def test_large_sparse_matrix_needs_scratch_in_proportion_to_its_nodes(F):
    """200 000 x 300 000 with about a million stored nodes: the scratch is a few bytes per node and
    per new row (a rows x columns bit matrix would be gigabytes)."""
    rng = np.random.default_rng(12)
    n_rows, n_cols, per_row = 200_000, 300_000, 5
    cols = np.sort(rng.integers(0, n_cols, (n_rows, per_row)), axis=1)
    keep = np.ones_like(cols, bool)
    keep[:, 1:] = cols[:, 1:] != cols[:, :-1]                      # indices strictly ascending inside a row
    ptr = np.concatenate([[0], np.cumsum(keep.sum(1))]).astype(np.int32)
    idx = cols[keep].astype(np.uint32)
    val = rng.standard_normal(idx.size).astype(np.float32)
    need = F.sparse_transpose_workspace(n_cols, idx.size)
    assert need < 16 << 20
    want = oracle.sparse_transpose(ptr, idx, val, n_rows, n_cols)
    got = F.sparse_transpose(dev_i32(ptr), dev_i32(idx), torch.from_numpy(val).cuda(), n_rows, n_cols)
    torch.cuda.synchronize()
    same(got, want)


def test_a_node_with_an_index_out_of_range_is_dropped(F):
    ptr = np.array([0, 3, 5], np.int32)
    idx = np.array([0, 2, 9, 1, 2], np.uint32)                     # 9 >= n_cols = 3
    val = np.arange(1, 6, dtype=np.float32)
    tptr, tidx, tval = (t.cpu().numpy() for t in F.sparse_transpose(dev_i32(ptr), dev_i32(idx),
                                                                    torch.from_numpy(val).cuda(), 2, 3))
    assert list(tptr) == [0, 1, 2, 4]
    assert list(tidx[:4]) == [0, 1, 0, 1] and list(tval[:4]) == [1.0, 4.0, 2.0, 5.0]
