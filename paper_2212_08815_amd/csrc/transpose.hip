// Sparse matrix transpose (Alg. 3) and sparse 3-D tensor transpose O_whc -> O_chw (Alg. 4).
//
// Both reorder stored nodes: every node moves to a new row (its "bucket") and the nodes of a
// new row are ordered by a "key" that is unique inside the row:
//   matrix, rows -> columns:   bucket = column of the node,  key = its old row;
//   tensor, O_whc -> O_chw:    old row = c*H + h lists w;  bucket = w*H + h,  key = c.
// The paper does this with a sequential walk that advances one cursor per new row (the vector
// v of Alg. 3) - a stable counting sort.  The same result is computed here without any
// order-dependent step: a bit matrix marks which (bucket, key) pairs exist, the population
// counts of a bucket's words give the bucket sizes and, accumulated, the rank of every key
// inside its bucket, so each node knows its final position on its own.  Integer work only;
// values are copied bit for bit.
#include "internal.h"

namespace fscnn {

namespace {

constexpr int kBlock = 256;

__global__ void __launch_bounds__(kBlock) reorder_clear_kernel(uint32_t *__restrict__ p, long long n)
{
    const long long i = (long long)blockIdx.x * kBlock + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// Row of entry e: the last r with rowptr[r] <= e (rows may be empty).
__device__ inline int row_of(const int *__restrict__ rowptr, int n_rows, long long e)
{
    int lo = 0, hi = n_rows;  // invariant: rowptr[lo] <= e < rowptr[hi]
    while (hi - lo > 1) {
        const int mid = lo + (hi - lo) / 2;
        if (rowptr[mid] <= e) lo = mid; else hi = mid;
    }
    return lo;
}

struct Dest {
    long long bucket;
    int key;
    bool ok;
};

// TENSOR = false: n_cols columns;  TENSOR = true: n_cols = W, H rows per channel.
template <bool TENSOR>
__device__ inline Dest dest_of(int row, uint32_t col, int n_cols, int H)
{
    Dest d;
    d.ok = col < (uint32_t)n_cols;  // a corrupt index is dropped, never followed
    if (TENSOR) {
        const int c = row / H, h = row - c * H;
        d.bucket = (long long)col * H + h;
        d.key = c;
    } else {
        d.bucket = col;
        d.key = row;
    }
    return d;
}

template <bool TENSOR>
__global__ void __launch_bounds__(kBlock) reorder_mark_kernel(const int *__restrict__ rowptr,
                                                              const uint32_t *__restrict__ idx,
                                                              int n_rows, int n_cols, int H,
                                                              long long nnz, int nw,
                                                              uint32_t *__restrict__ bits)
{
    const long long e = (long long)blockIdx.x * kBlock + threadIdx.x;
    if (e >= nnz) return;
    const Dest d = dest_of<TENSOR>(row_of(rowptr, n_rows, e), idx[e], n_cols, H);
    if (d.ok) atomicOr(&bits[d.bucket * nw + (d.key >> 5)], 1u << (d.key & 31));
}

// Per bucket: exclusive running population count over its words, and the total.
__global__ void __launch_bounds__(kBlock) reorder_count_kernel(const uint32_t *__restrict__ bits,
                                                               long long n_buckets, int nw,
                                                               int *__restrict__ before,
                                                               int *__restrict__ cnt)
{
    const long long b = (long long)blockIdx.x * kBlock + threadIdx.x;
    if (b >= n_buckets) return;
    int run = 0;
    for (int w = 0; w < nw; ++w) {
        before[b * nw + w] = run;
        run += __popc(bits[b * nw + w]);
    }
    cnt[b] = run;
}

template <bool TENSOR>
__global__ void __launch_bounds__(kBlock) reorder_scatter_kernel(
    const int *__restrict__ rowptr, const uint32_t *__restrict__ idx, const float *__restrict__ val,
    int n_rows, int n_cols, int H, long long nnz, int nw, const uint32_t *__restrict__ bits,
    const int *__restrict__ before, const int *__restrict__ tptr, uint32_t *__restrict__ tidx,
    float *__restrict__ tval)
{
    const long long e = (long long)blockIdx.x * kBlock + threadIdx.x;
    if (e >= nnz) return;
    const Dest d = dest_of<TENSOR>(row_of(rowptr, n_rows, e), idx[e], n_cols, H);
    if (!d.ok) return;
    const long long wd = d.bucket * nw + (d.key >> 5);
    const int rank = before[wd] + __popc(bits[wd] & ((1u << (d.key & 31)) - 1u));
    const long long dst = (long long)tptr[d.bucket] + rank;
    if (dst < nnz) {  // holds for every well-formed input (strictly ascending indices per row)
        tidx[dst] = (uint32_t)d.key;
        tval[dst] = val[e];
    }
}

inline unsigned blocks_for(long long n) { return (unsigned)((n + kBlock - 1) / kBlock); }

}  // namespace

long long reorder_workspace_bytes(long long n_buckets, long long n_keys)
{
    if (n_buckets <= 0 || n_keys <= 0) return -1;
    const long long nw = (n_keys + 31) / 32;
    const long long words = n_buckets * nw;
    if (nw > 0x7fffffffLL || words / nw != n_buckets || words > (1LL << 33)) return -1;
    return 4 * (2 * words + n_buckets + scan_tmp_elems(n_buckets));
}

hipError_t launch_reorder(bool tensor, const int *rowptr, const uint32_t *idx, const float *val,
                          int n_rows, int n_cols, int H, long long n_buckets, int n_keys,
                          long long nnz, int *tptr, uint32_t *tidx, float *tval, void *workspace,
                          hipStream_t st)
{
    const int nw = (n_keys + 31) / 32;
    const long long words = n_buckets * nw;
    uint32_t *bits = static_cast<uint32_t *>(workspace);
    int *before = reinterpret_cast<int *>(bits + words);
    int *cnt = before + words;
    hipLaunchKernelGGL(reorder_clear_kernel, dim3(blocks_for(words)), dim3(kBlock), 0, st, bits, words);
    if (nnz > 0) {
        if (tensor)
            hipLaunchKernelGGL(reorder_mark_kernel<true>, dim3(blocks_for(nnz)), dim3(kBlock), 0, st,
                               rowptr, idx, n_rows, n_cols, H, nnz, nw, bits);
        else
            hipLaunchKernelGGL(reorder_mark_kernel<false>, dim3(blocks_for(nnz)), dim3(kBlock), 0, st,
                               rowptr, idx, n_rows, n_cols, H, nnz, nw, bits);
    }
    hipLaunchKernelGGL(reorder_count_kernel, dim3(blocks_for(n_buckets)), dim3(kBlock), 0, st, bits,
                       n_buckets, nw, before, cnt);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = launch_exclusive_scan(cnt, tptr, n_buckets, cnt + n_buckets, st);
    if (e != hipSuccess) return e;
    if (nnz > 0) {
        if (tensor)
            hipLaunchKernelGGL(reorder_scatter_kernel<true>, dim3(blocks_for(nnz)), dim3(kBlock), 0, st,
                               rowptr, idx, val, n_rows, n_cols, H, nnz, nw, bits, before, tptr, tidx,
                               tval);
        else
            hipLaunchKernelGGL(reorder_scatter_kernel<false>, dim3(blocks_for(nnz)), dim3(kBlock), 0, st,
                               rowptr, idx, val, n_rows, n_cols, H, nnz, nw, bits, before, tptr, tidx,
                               tval);
    }
    return hipGetLastError();
}

}  // namespace fscnn
