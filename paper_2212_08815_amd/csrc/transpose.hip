// Sparse matrix transpose (Alg. 3) and sparse 3-D tensor transpose O_whc -> O_chw (Alg. 4).
//
// Both reorder stored nodes: every node moves to a new row (its "bucket") and the nodes of a
// new row are ordered by a "key" that is unique inside the row:
//   matrix, rows -> columns:   bucket = column of the node,  key = its old row;
//   tensor, O_whc -> O_chw:    old row = c*H + h lists w;  bucket = w*H + h,  key = c.
// The paper does this with a sequential walk that advances one cursor per new row (the vector
// v of Alg. 3) - a stable counting sort.  The same result is computed here in passes whose
// outcome does not depend on thread order, with scratch of O(nodes + new rows):
//   1. count the nodes of every bucket (integer atomic adds: the sums are order-independent);
//   2. exclusive scan of the counts = the new pointer array;
//   3. drop every node into its bucket's segment of a scratch copy, at a position handed out by
//      an atomic cursor - the segment then holds the right nodes in an arbitrary order;
//   4. every node of the scratch copy counts the nodes of its segment with a smaller key - its
//      rank, since keys are unique inside a bucket - and lands at pointer[bucket] + rank.
// The arbitrary order of step 3 never reaches the result.  Step 4 costs the sum of the squared
// bucket sizes (a bucket is a column of the matrix / a pixel's channel list: tens to hundreds
// of nodes).  Integer work only; values are copied bit for bit.
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
__global__ void __launch_bounds__(kBlock) reorder_count_kernel(const int *__restrict__ rowptr,
                                                               const uint32_t *__restrict__ idx,
                                                               int n_rows, int n_cols, int H,
                                                               long long nnz, int *__restrict__ cnt)
{
    const long long e = (long long)blockIdx.x * kBlock + threadIdx.x;
    if (e >= nnz) return;
    const Dest d = dest_of<TENSOR>(row_of(rowptr, n_rows, e), idx[e], n_cols, H);
    if (d.ok) atomicAdd(&cnt[d.bucket], 1);
}

// cursor[b] = tptr[b]: where the next node of bucket b is dropped
__global__ void __launch_bounds__(kBlock) reorder_cursor_kernel(const int *__restrict__ tptr,
                                                                long long n_buckets, int *__restrict__ cursor)
{
    const long long b = (long long)blockIdx.x * kBlock + threadIdx.x;
    if (b < n_buckets) cursor[b] = tptr[b];
}

template <bool TENSOR>
__global__ void __launch_bounds__(kBlock) reorder_drop_kernel(
    const int *__restrict__ rowptr, const uint32_t *__restrict__ idx, const float *__restrict__ val,
    int n_rows, int n_cols, int H, long long nnz, int *__restrict__ cursor,
    uint32_t *__restrict__ skey, float *__restrict__ sval)
{
    const long long e = (long long)blockIdx.x * kBlock + threadIdx.x;
    if (e >= nnz) return;
    const Dest d = dest_of<TENSOR>(row_of(rowptr, n_rows, e), idx[e], n_cols, H);
    if (!d.ok) return;
    const int p = atomicAdd(&cursor[d.bucket], 1);
    if (p < nnz) {
        skey[p] = (uint32_t)d.key;
        sval[p] = val[e];
    }
}

// One thread per position of the scratch copy: its bucket is the segment of tptr that holds the
// position; its rank is the number of smaller keys in that segment.
__global__ void __launch_bounds__(kBlock) reorder_place_kernel(const int *__restrict__ tptr,
                                                               long long n_buckets, long long total,
                                                               const uint32_t *__restrict__ skey,
                                                               const float *__restrict__ sval,
                                                               uint32_t *__restrict__ tidx,
                                                               float *__restrict__ tval)
{
    const long long p = (long long)blockIdx.x * kBlock + threadIdx.x;
    if (p >= total || p >= tptr[n_buckets]) return;   // past the last node that was kept
    // last b with tptr[b] <= p (buckets may be empty)
    long long lo = 0, hi = n_buckets;
    while (hi - lo > 1) {
        const long long mid = lo + (hi - lo) / 2;
        if (tptr[mid] <= p) lo = mid; else hi = mid;
    }
    const int a = tptr[lo], b = tptr[lo + 1];
    const uint32_t key = skey[p];
    int rank = 0;
    for (int q = a; q < b; ++q) rank += skey[q] < key ? 1 : 0;
    tidx[a + rank] = key;
    tval[a + rank] = sval[p];
}

inline unsigned blocks_for(long long n) { return (unsigned)((n + kBlock - 1) / kBlock); }

// scratch layout (32-bit words): cnt[n_buckets] | scan scratch | cursor[n_buckets] | skey[nnz] | sval[nnz]
struct Layout {
    long long cnt, scan, cursor, skey, sval, words;
};
inline Layout layout_of(long long n_buckets, long long nnz)
{
    Layout l;
    l.cnt = 0;
    l.scan = n_buckets;
    l.cursor = l.scan + scan_tmp_elems(n_buckets);
    l.skey = l.cursor + n_buckets;
    l.sval = l.skey + nnz;
    l.words = l.sval + nnz;
    return l;
}

// Scratch of the entry point that allocates nothing: one copy per GPU, held until the process
// ends.  Host code never passes this name to a kernel: it is a host-side stand-in, the device
// address comes from hipGetSymbolAddress (static_scratch below).
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex scratch_mu;
void *scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, once looked up

}  // namespace

hipError_t static_scratch(void **ptr)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (!scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // with `dev` current: this GPU's copy
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        scratch_ptr[dev] = p;
    }
    *ptr = scratch_ptr[dev];
    return hipSuccess;
}

long long reorder_workspace_bytes(long long n_buckets, long long nnz)
{
    if (n_buckets <= 0 || nnz < 0 || n_buckets >= (1LL << 31) || nnz >= (1LL << 31)) return -1;
    return 4 * layout_of(n_buckets, nnz).words;
}

hipError_t launch_reorder(bool tensor, const int *rowptr, const uint32_t *idx, const float *val,
                          int n_rows, int n_cols, int H, long long n_buckets, long long nnz,
                          int *tptr, uint32_t *tidx, float *tval, void *workspace, hipStream_t st)
{
    const Layout l = layout_of(n_buckets, nnz);
    int *ws = static_cast<int *>(workspace);
    int *cnt = ws + l.cnt, *cursor = ws + l.cursor;
    uint32_t *skey = reinterpret_cast<uint32_t *>(ws + l.skey);
    float *sval = reinterpret_cast<float *>(ws + l.sval);
    hipLaunchKernelGGL(reorder_clear_kernel, dim3(blocks_for(n_buckets)), dim3(kBlock), 0, st,
                       reinterpret_cast<uint32_t *>(cnt), n_buckets);
    if (nnz > 0) {
        if (tensor)
            hipLaunchKernelGGL(reorder_count_kernel<true>, dim3(blocks_for(nnz)), dim3(kBlock), 0, st,
                               rowptr, idx, n_rows, n_cols, H, nnz, cnt);
        else
            hipLaunchKernelGGL(reorder_count_kernel<false>, dim3(blocks_for(nnz)), dim3(kBlock), 0, st,
                               rowptr, idx, n_rows, n_cols, H, nnz, cnt);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = launch_exclusive_scan(cnt, tptr, n_buckets, ws + l.scan, st);
    if (e != hipSuccess || nnz == 0) return e;
    hipLaunchKernelGGL(reorder_cursor_kernel, dim3(blocks_for(n_buckets)), dim3(kBlock), 0, st, tptr,
                       n_buckets, cursor);
    if (tensor)
        hipLaunchKernelGGL(reorder_drop_kernel<true>, dim3(blocks_for(nnz)), dim3(kBlock), 0, st, rowptr,
                           idx, val, n_rows, n_cols, H, nnz, cursor, skey, sval);
    else
        hipLaunchKernelGGL(reorder_drop_kernel<false>, dim3(blocks_for(nnz)), dim3(kBlock), 0, st, rowptr,
                           idx, val, n_rows, n_cols, H, nnz, cursor, skey, sval);
    // nodes with a corrupt index were skipped: the kernel reads the number of kept nodes from the
    // pointer array's last element and places no position beyond it
    hipLaunchKernelGGL(reorder_place_kernel, dim3(blocks_for(nnz)), dim3(kBlock), 0, st, tptr, n_buckets,
                       nnz, skey, sval, tidx, tval);
    return hipGetLastError();
}

}  // namespace fscnn
