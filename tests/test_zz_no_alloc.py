"""The entry point that allocates nothing (fscnn_sparse_transpose_noalloc: scratch in a static
device array of the library) against the entry point it is a variant of (fscnn_sparse_transpose,
scratch brought by the caller), through the C ABI: two calls in a row, the second with a smaller
input, every output array bit for bit (integer and copy work)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def F():
    from paper_2212_08815_amd import fscnn
    fscnn.lib()
    assert torch.cuda.is_available()
    return fscnn


def _csr(rng, n_rows, n_cols, keep):
    m = (rng.standard_normal((n_rows, n_cols)) * (rng.random((n_rows, n_cols)) < keep)).astype(np.float32)
    r, c = np.nonzero(m)
    ptr = np.zeros(n_rows + 1, np.int64)
    np.add.at(ptr, r + 1, 1)
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, np.int32)).cuda()
    return i32(np.cumsum(ptr)), i32(c), torch.from_numpy(m[r, c]).cuda()


def test_noalloc_transpose_equals_the_workspace_form_twice_in_a_row(F):
    rng = np.random.default_rng(2212)
    # the outputs are allocated once, for the larger case, and poisoned before each call
    cases = [(512, 4608, 0.05), (37, 300, 0.2)]          # second call: smaller rows, columns and nnz
    big = _csr(rng, *cases[0])
    out = (torch.empty(cases[0][1] + 1, dtype=torch.int32, device="cuda"),
           torch.empty(big[1].numel(), dtype=torch.int32, device="cuda"),
           torch.empty(big[1].numel(), dtype=torch.float32, device="cuda"))
    for (n_rows, n_cols, keep), ops in zip(cases, [big, _csr(rng, *cases[1])]):
        ptr, idx, val = ops
        nnz = idx.numel()
        assert 0 < F.sparse_transpose_workspace(n_cols, nnz) <= 8 << 20
        want = F.sparse_transpose(ptr, idx, val, n_rows, n_cols)
        for t in out:
            t.fill_(-7)
        before = torch.cuda.memory_allocated()
        F.sparse_transpose_noalloc(ptr, idx, val, n_rows, n_cols, out)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        assert torch.equal(out[0][:n_cols + 1], want[0])
        assert torch.equal(out[1][:nnz], want[1])
        assert torch.equal(out[2][:nnz].view(torch.int32), want[2].view(torch.int32))
        # nothing was written past the result
        assert bool((out[0][n_cols + 1:] == -7).all()) and bool((out[1][nnz:] == -7).all())


def test_noalloc_transpose_rejects_sizes_beyond_its_static_scratch(F):
    import ctypes
    L = F.lib()
    fake = ctypes.c_void_p(256)
    ll = ctypes.c_longlong
    assert F.sparse_transpose_workspace(3_000_000, 10) > 8 << 20
    assert L.fscnn_sparse_transpose_noalloc(fake, fake, fake, 5, 3_000_000, ll(10), fake, fake, fake, None) == 4
    assert L.fscnn_sparse_transpose_noalloc(fake, fake, fake, 5, 10, ll(2_000_000), fake, fake, fake, None) == 4
    assert L.fscnn_sparse_transpose_noalloc(None, fake, fake, 5, 10, ll(1), fake, fake, fake, None) == 1
    assert L.fscnn_sparse_transpose_noalloc(fake, fake, fake, 0, 10, ll(1), fake, fake, fake, None) == 2
