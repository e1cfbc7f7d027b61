// Compression kernels: dense filter bank -> CSR(C) (count, scan, ordered pack), the
// regrouping of the nonzeros into the (group, chunk, channel) stream the convolution
// kernel reads, dense activation -> per-pixel channel lists, and the helper max-pool.
//
// The paper (Sec. 3) fixes the format only: values, column indices and cumulative row
// counts that start with 0, one row per filter.  The construction used here is
// count -> exclusive scan -> order-preserving compaction, which makes the result unique
// (ascending flat index inside each row) and independent of thread scheduling.
#include "internal.h"

namespace fscnn {

namespace {

constexpr int kBlock = 256;

__device__ inline int lane_id() { return threadIdx.x & 63; }

// Exclusive prefix of `flag` over the work-group in thread order, plus the group total.
// Uses one ballot per wave and a small LDS array for the wave totals.
__device__ inline int block_exclusive_count(bool flag, int *wave_tot /* LDS, >= blockDim/64 */,
                                            int *total)
{
    const unsigned long long m = __ballot(flag);
    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int nw = blockDim.x >> 6;
    const int within = __popcll(m & ((1ull << lane) - 1ull));
    if (lane == 0) wave_tot[wave] = __popcll(m);
    __syncthreads();
    int before = 0, tot = 0;
    for (int i = 0; i < nw; ++i) {
        const int t = wave_tot[i];
        if (i < wave) before += t;
        tot += t;
    }
    __syncthreads();  // wave_tot may be reused by the caller's next round
    *total = tot;
    return before + within;
}

// ---- A1: per output channel, the number of entries with w != 0 ------------------------
__global__ void __launch_bounds__(kBlock) filter_count_kernel(const float *__restrict__ w,
                                                              long long row, int *__restrict__ cnt)
{
    __shared__ int part[kBlock / 64];
    const float *wk = w + (long long)blockIdx.x * row;
    int c = 0;
    for (long long f = threadIdx.x; f < row; f += kBlock) c += (wk[f] != 0.0f) ? 1 : 0;
    for (int o = 32; o > 0; o >>= 1) c += __shfl_down(c, o, 64);
    if (lane_id() == 0) part[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
        for (int i = 0; i < kBlock / 64; ++i) t += part[i];
        cnt[blockIdx.x] = t;
    }
}

// ---- exclusive scan of n ints into out[0..n] (out[n] = total); one work-group ---------
constexpr int kScanThreads = 1024;
__global__ void __launch_bounds__(kScanThreads) exclusive_scan_kernel(const int *__restrict__ in,
                                                                      int *__restrict__ out,
                                                                      long long n)
{
    __shared__ int sums[kScanThreads];
    const long long per = (n + kScanThreads - 1) / kScanThreads;
    const long long lo = (long long)threadIdx.x * per;
    const long long hi = lo + per < n ? lo + per : n;
    int s = 0;
    for (long long i = lo; i < hi; ++i) s += in[i];
    sums[threadIdx.x] = s;
    __syncthreads();
    // Hillis-Steele inclusive scan over the 1024 partial sums
    for (int o = 1; o < kScanThreads; o <<= 1) {
        int v = (int)threadIdx.x >= o ? sums[threadIdx.x - o] : 0;
        __syncthreads();
        sums[threadIdx.x] += v;
        __syncthreads();
    }
    int run = threadIdx.x == 0 ? 0 : sums[threadIdx.x - 1];
    for (long long i = lo; i < hi; ++i) {
        const int v = in[i];
        out[i] = run;
        run += v;
    }
    if (threadIdx.x == kScanThreads - 1) out[n] = sums[kScanThreads - 1];
}

// ---- the same for large n, three passes over tiles of kTile elements -------------------
// (1) every work-group adds up its tile; (2) the tile sums are scanned by the single-group
// kernel above; (3) every work-group scans its tile starting from its tile's offset.  Tiles go
// through LDS so that global loads and stores are contiguous while each thread scans a
// contiguous run.
constexpr int kTileThreads = 256, kTilePer = 16, kTile = kTileThreads * kTilePer;

__global__ void __launch_bounds__(kTileThreads) scan_tile_sum_kernel(const int *__restrict__ in,
                                                                     long long n, int *__restrict__ tsum)
{
    __shared__ int part[kTileThreads / 64];
    const long long base = (long long)blockIdx.x * kTile;
    int s = 0;
#pragma unroll
    for (int k = 0; k < kTilePer; ++k) {
        const long long i = base + k * kTileThreads + threadIdx.x;
        if (i < n) s += in[i];
    }
    for (int o = 32; o > 0; o >>= 1) s += __shfl_down(s, o, 64);
    if (lane_id() == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
        for (int i = 0; i < kTileThreads / 64; ++i) t += part[i];
        tsum[blockIdx.x] = t;
    }
}

__global__ void __launch_bounds__(kTileThreads) scan_tile_kernel(const int *__restrict__ in, long long n,
                                                                 const int *__restrict__ toff,
                                                                 int *__restrict__ out)
{
    __shared__ int tile[kTile + kTile / 32];     // padded: a thread's run of 16 starts in its own bank group
    __shared__ int tsum[kTileThreads];
    const long long base = (long long)blockIdx.x * kTile;
    auto at = [](int e) { return e + e / 32; };
#pragma unroll
    for (int k = 0; k < kTilePer; ++k) {
        const int e = k * kTileThreads + threadIdx.x;
        tile[at(e)] = base + e < n ? in[base + e] : 0;
    }
    __syncthreads();
    int s = 0;
#pragma unroll
    for (int k = 0; k < kTilePer; ++k) s += tile[at(threadIdx.x * kTilePer + k)];
    tsum[threadIdx.x] = s;
    __syncthreads();
    for (int o = 1; o < kTileThreads; o <<= 1) {
        const int v = (int)threadIdx.x >= o ? tsum[threadIdx.x - o] : 0;
        __syncthreads();
        tsum[threadIdx.x] += v;
        __syncthreads();
    }
    int run = toff[blockIdx.x] + (threadIdx.x == 0 ? 0 : tsum[threadIdx.x - 1]);
#pragma unroll
    for (int k = 0; k < kTilePer; ++k) {
        const int idx = at(threadIdx.x * kTilePer + k);
        const int v = tile[idx];
        tile[idx] = run;
        run += v;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kTilePer; ++k) {
        const int e = k * kTileThreads + threadIdx.x;
        if (base + e < n) out[base + e] = tile[at(e)];
    }
    // the grand total goes to out[n]
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == kTileThreads - 1) out[n] = toff[gridDim.x];
}

// ---- A2: ordered pack of row k into idx/val at rowptr[k] ------------------------------
__global__ void __launch_bounds__(kBlock) filter_pack_kernel(const float *__restrict__ w,
                                                             long long row,
                                                             const int *__restrict__ rowptr,
                                                             uint32_t *__restrict__ idx,
                                                             float *__restrict__ val)
{
    __shared__ int wave_tot[kBlock / 64];
    const int k = blockIdx.x;
    const float *wk = w + (long long)k * row;
    long long base = rowptr[k];
    for (long long f0 = 0; f0 < row; f0 += kBlock) {
        const long long f = f0 + threadIdx.x;
        float v = 0.0f;
        if (f < row) v = wk[f];
        const bool nz = (f < row) && (v != 0.0f);
        int tot;
        const int pos = block_exclusive_count(nz, wave_tot, &tot);
        if (nz) {
            idx[base + pos] = (uint32_t)f;
            val[base + pos] = v;
        }
        base += tot;
    }
}

// ---- A3: regroup into (group g, chunk ci, channel-in-group kk) buckets -----------------
// Rows are ascending in the flat index, hence ascending in c: the entries of chunk ci are the
// contiguous run with ci*CC*R*S <= flat < (ci+1)*CC*R*S, found by binary search.
__device__ inline int lower_bound_u32(const uint32_t *a, int lo, int hi, uint32_t key)
{
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid] < key) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// Bucket b <-> (group g, wave w, chunk ci, slot j), slot fastest: the records of one wave form
// one contiguous stream ordered by (chunk, slot); its output channel is k = g*KG + w*SLOTS + j.
struct Bucket {
    int k, ci;
};
__device__ inline Bucket decode_bucket(long long b, int SLOTS, int WAVES, int NCH)
{
    Bucket r;
    const int j = (int)(b % SLOTS);
    r.ci = (int)((b / SLOTS) % NCH);
    const int w = (int)((b / ((long long)SLOTS * NCH)) % WAVES);
    const int g = (int)(b / ((long long)SLOTS * NCH * WAVES));
    r.k = (g * WAVES + w) * SLOTS + j;
    return r;
}

__global__ void plan_count_kernel(const int *__restrict__ rowptr, const uint32_t *__restrict__ idx,
                                  int K, int RS, int CC, int SLOTS, int WAVES, int NCH, int NG,
                                  int *__restrict__ cnt)
{
    const long long b = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long nb = (long long)NG * NCH * SLOTS * WAVES;
    if (b >= nb) return;
    const Bucket q = decode_bucket(b, SLOTS, WAVES, NCH);
    int c = 0;
    if (q.k < K) {
        const int lo = rowptr[q.k], hi = rowptr[q.k + 1];
        const int a = lower_bound_u32(idx, lo, hi, (uint32_t)q.ci * CC * RS);
        const int e = lower_bound_u32(idx, lo, hi, (uint32_t)(q.ci + 1) * CC * RS);
        c = e - a;
    }
    cnt[b] = c;
}

__global__ void plan_fill_kernel(const int *__restrict__ rowptr, const uint32_t *__restrict__ idx,
                                 const float *__restrict__ val, int K, int R, int S, int CC,
                                 int SLOTS, int WAVES, int NCH, int NG, int IN_ROWS, int PITCH,
                                 int BV, int STRIDE, const int *__restrict__ segptr,
                                 Rec *__restrict__ recs)
{
    const long long b = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long nb = (long long)NG * NCH * SLOTS * WAVES;
    if (b < kPlanSpare) {  // spare records a prefetching reader may touch past the end
        const int last = segptr[nb];
        Rec z;
        z.off = 0u;
        z.val = 0.0f;
        recs[last + b] = z;
    }
    if (b >= nb) return;
    const Bucket q = decode_bucket(b, SLOTS, WAVES, NCH);
    if (q.k >= K) return;
    const int RS = R * S;
    const int lo = rowptr[q.k], hi = rowptr[q.k + 1];
    const int a = lower_bound_u32(idx, lo, hi, (uint32_t)q.ci * CC * RS);
    const int e = lower_bound_u32(idx, lo, hi, (uint32_t)(q.ci + 1) * CC * RS);
    int o = segptr[b];
    for (int i = a; i < e; ++i, ++o) {
        const uint32_t f = idx[i];
        const int c = (int)(f / RS) - q.ci * CC;
        const int rs = (int)(f % RS);
        const int r = rs / S, s = rs % S;
        Rec rec;
        // stride 2: tap (r, s) lies in plane (r mod 2, s mod 2) of the channel at (r/2, s/2)
        const int plane = (r % STRIDE) * STRIDE + (s % STRIDE);
        rec.off = (uint32_t)(((((c * STRIDE * STRIDE + plane) * IN_ROWS) + r / STRIDE) * PITCH + s / STRIDE) * BV * 4);
        rec.val = val[i];
        recs[o] = rec;
    }
}

// The plan of the taps-outer form: for every (group, wave, chunk), CC*R*S groups of SLOTS records
// {LDS byte offset of tap (c mod CC, r, s), weight of output channel (group*WAVES + wave)*SLOTS + j
// at that tap}, a zero weight where the row stores nothing there (or k, c lie past the bank).
__global__ void plan_fill_dense_kernel(const int *__restrict__ rowptr, const uint32_t *__restrict__ idx,
                                       const float *__restrict__ val, int K, int C, int R, int S, int CC,
                                       int SLOTS, int WAVES, int NCH, int NG, int IN_ROWS, int PITCH,
                                       int BV, long long nrec, Rec *__restrict__ recs)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < kPlanSpare) {
        Rec z;
        z.off = 0u;
        z.val = 0.0f;
        recs[nrec + i] = z;
    }
    if (i >= nrec) return;
    const int RS = R * S, T = CC * RS;
    const int j = (int)(i % SLOTS);
    const int t = (int)((i / SLOTS) % T);
    const int ci = (int)((i / ((long long)SLOTS * T)) % NCH);
    const long long gw = i / ((long long)SLOTS * T * NCH);   // group * WAVES + wave
    const int k = (int)(gw * SLOTS + j);
    const int cl = t / RS, rs = t % RS;
    const int c = ci * CC + cl;
    Rec rec;
    rec.off = (uint32_t)((((cl * IN_ROWS) + rs / S) * PITCH + rs % S) * BV * 4);
    rec.val = 0.0f;
    if (k < K && c < C) {
        const uint32_t flat = (uint32_t)(c * RS + rs);
        const int lo = rowptr[k], hi = rowptr[k + 1];
        const int at = lower_bound_u32(idx, lo, hi, flat);
        if (at < hi && idx[at] == flat) rec.val = val[at];
    }
    recs[i] = rec;
}

// ---- A7: compressed activation, rows = pixels, columns = channels ----------------------
// One thread per (pixel, step of CC channels): threads of a work-group take consecutive pixels
// of one step, so the reads of a channel plane are contiguous.  The exclusive scan of the counts
// in (pixel, step) order is at once the position of every step's first entry (the chunk pointers
// the convolution kernels read) and, at step 0, the start of the pixel's row.
__global__ void __launch_bounds__(kBlock) input_count_kernel(const float *__restrict__ x, int C,
                                                             long long HW, long long npix, int CC,
                                                             int NCH, int *__restrict__ cnt)
{
    const long long p = (long long)blockIdx.x * kBlock + threadIdx.x;
    const int j = blockIdx.y;
    if (p >= npix) return;
    const long long n = p / HW, q = p % HW;
    const float *xp = x + n * C * HW + q;
    const int c1 = (j + 1) * CC < C ? (j + 1) * CC : C;
    int c = 0;
    for (int ch = j * CC; ch < c1; ++ch) c += (xp[(long long)ch * HW] != 0.0f) ? 1 : 0;
    cnt[p * NCH + j] = c;
}

// A work-group packs the lists of PX consecutive pixels (PX a power of two, at most 32): thread
// (pixel px, step lane sj) walks the steps sj, sj + 256/PX, ... of its pixel, so the reads of a
// channel plane cover PX adjacent floats, and drops its (channel, value) pairs into an LDS image
// of the group's output range -- the lists of consecutive pixels are adjacent in memory -- which
// is then copied out with fully coalesced stores.
__global__ void __launch_bounds__(kBlock) input_fill_kernel(const float *__restrict__ x, int C,
                                                            long long HW, long long npix, int CC,
                                                            int NCH, int PX,
                                                            const int *__restrict__ cptr,
                                                            uint32_t *__restrict__ cidx,
                                                            float *__restrict__ xval, int spare)
{
    extern __shared__ uint32_t stage[];   // [cap] channel indices, then [cap] value bit patterns
    const int cap = PX * NCH * CC;
    // the entries past the last stored one (readers fetch a few positions ahead); the number of
    // stored entries is the pointer array's last element
    if (blockIdx.x == 0 && (int)threadIdx.x < spare) {
        const long long total = cptr[npix * NCH];
        cidx[total + threadIdx.x] = 0u;
        xval[total + threadIdx.x] = 0.0f;
    }
    const long long p0 = (long long)blockIdx.x * PX;
    const long long p1 = p0 + PX < npix ? p0 + PX : npix;
    const int base = cptr[p0 * NCH];
    const int count = cptr[p1 * NCH] - base;      // <= cap: at most C entries per pixel
    const int px = threadIdx.x % PX, sj = threadIdx.x / PX;
    const long long p = p0 + px;
    if (p < npix) {
        const long long n = p / HW, q = p % HW;
        const float *xp = x + n * C * HW + q;
        for (int j = sj; j < NCH; j += kBlock / PX) {
            const int c1 = (j + 1) * CC < C ? (j + 1) * CC : C;
            int o = cptr[p * NCH + j] - base;
            for (int ch = j * CC; ch < c1; ++ch) {
                const float v = xp[(long long)ch * HW];
                if (v != 0.0f) {
                    stage[o] = (uint32_t)ch;
                    stage[cap + o] = __float_as_uint(v);
                    ++o;
                }
            }
        }
    }
    __syncthreads();
    for (int t = threadIdx.x; t < count; t += kBlock) {
        cidx[base + t] = stage[t];
        xval[base + t] = __uint_as_float(stage[cap + t]);
    }
}

// ---- helper: 2x2 / stride-2 max pooling ------------------------------------------------
__global__ void __launch_bounds__(kBlock) maxpool2x2_kernel(const float *__restrict__ x,
                                                            long long NC, int H, int W, int Ho,
                                                            int Wo, float *__restrict__ y)
{
    const long long o = (long long)blockIdx.x * kBlock + threadIdx.x;
    if (o >= NC * Ho * Wo) return;
    const int ox = (int)(o % Wo);
    const int oy = (int)((o / Wo) % Ho);
    const long long nc = o / ((long long)Wo * Ho);
    const float *p = x + (nc * H + 2 * oy) * W + 2 * ox;
    float m = p[0];
    m = p[1] > m ? p[1] : m;
    m = p[W] > m ? p[W] : m;
    m = p[W + 1] > m ? p[W + 1] : m;
    y[o] = m;
}

// same pooling on a batch-interleaved (N4) tensor: one thread per output pixel of one image
// group, all four images at once
__global__ void __launch_bounds__(kBlock) maxpool2x2_n4_kernel(const float4 *__restrict__ x,
                                                               long long GC, int H, int W, int Ho,
                                                               int Wo, float4 *__restrict__ y)
{
    const long long o = (long long)blockIdx.x * kBlock + threadIdx.x;
    if (o >= GC * Ho * Wo) return;
    const int ox = (int)(o % Wo);
    const int oy = (int)((o / Wo) % Ho);
    const long long gc = o / ((long long)Wo * Ho);
    const float4 *p = x + (gc * H + 2 * oy) * W + 2 * ox;
    const float4 a = p[0], b = p[1], c = p[W], d = p[W + 1];
    auto mx4 = [](float p0, float p1, float p2, float p3) {  // same compare order as the NCHW kernel
        float m = p0;
        m = p1 > m ? p1 : m;
        m = p2 > m ? p2 : m;
        m = p3 > m ? p3 : m;
        return m;
    };
    y[o] = make_float4(mx4(a.x, b.x, c.x, d.x), mx4(a.y, b.y, c.y, d.y), mx4(a.z, b.z, c.z, d.z),
                       mx4(a.w, b.w, c.w, d.w));
}

// NCHW <-> N4 ([ceil(N/4)][C][H][W][4]); images past N read as / are written as nothing (N4 pad
// lanes are filled with 0)
__global__ void __launch_bounds__(kBlock) layout_convert_kernel(const float *__restrict__ src,
                                                                int N, long long CHW, int src_n4,
                                                                float *__restrict__ dst)
{
    const long long t = (long long)blockIdx.x * kBlock + threadIdx.x;
    const long long groups = (N + 3) / 4;
    if (t >= groups * CHW) return;
    const long long g = t / CHW, q = t % CHW;
    if (src_n4) {
        const float4 v = reinterpret_cast<const float4 *>(src)[t];
        const float e[4] = {v.x, v.y, v.z, v.w};
        for (int b = 0; b < 4; ++b)
            if (g * 4 + b < N) dst[(g * 4 + b) * CHW + q] = e[b];
    } else {
        float e[4];
        for (int b = 0; b < 4; ++b) e[b] = g * 4 + b < N ? src[(g * 4 + b) * CHW + q] : 0.0f;
        reinterpret_cast<float4 *>(dst)[t] = make_float4(e[0], e[1], e[2], e[3]);
    }
}

inline unsigned blocks_for(long long n, int per) { return (unsigned)((n + per - 1) / per); }

}  // namespace

hipError_t launch_filter_count(const float *w, int K, long long row, int *cnt, hipStream_t st)
{
    hipLaunchKernelGGL(filter_count_kernel, dim3(K), dim3(kBlock), 0, st, w, row, cnt);
    return hipGetLastError();
}

long long scan_tmp_elems(long long n)
{
    return n <= 4 * kTile ? 0 : 2 * ((n + kTile - 1) / kTile) + 2;
}

hipError_t launch_exclusive_scan(const int *in, int *out, long long n, int *tmp, hipStream_t st)
{
    if (n <= 4 * kTile) {
        hipLaunchKernelGGL(exclusive_scan_kernel, dim3(1), dim3(kScanThreads), 0, st, in, out, n);
        return hipGetLastError();
    }
    const long long nt = (n + kTile - 1) / kTile;
    int *tsum = tmp, *toff = tmp + nt;   // toff has nt + 1 entries
    hipLaunchKernelGGL(scan_tile_sum_kernel, dim3((unsigned)nt), dim3(kTileThreads), 0, st, in, n, tsum);
    hipLaunchKernelGGL(exclusive_scan_kernel, dim3(1), dim3(kScanThreads), 0, st, tsum, toff, nt);
    hipLaunchKernelGGL(scan_tile_kernel, dim3((unsigned)nt), dim3(kTileThreads), 0, st, in, n, toff, out);
    return hipGetLastError();
}

hipError_t launch_filter_pack(const float *w, int K, long long row, const int *rowptr,
                              uint32_t *idx, float *val, hipStream_t st)
{
    hipLaunchKernelGGL(filter_pack_kernel, dim3(K), dim3(kBlock), 0, st, w, row, rowptr, idx, val);
    return hipGetLastError();
}

hipError_t launch_plan_count(const int *rowptr, const uint32_t *idx, int K, int RS, const SfGeom &g,
                             int NCH, int NG, int *cnt, hipStream_t st)
{
    const long long nb = (long long)NG * NCH * g.KG;
    hipLaunchKernelGGL(plan_count_kernel, dim3(blocks_for(nb, kBlock)), dim3(kBlock), 0, st, rowptr,
                       idx, K, RS, g.CC, g.SLOTS, g.WAVES, NCH, NG, cnt);
    return hipGetLastError();
}

hipError_t launch_plan_fill(const int *rowptr, const uint32_t *idx, const float *val, int K, int R,
                            int S, const SfGeom &g, int NCH, int NG, const int *segptr, Rec *recs,
                            hipStream_t st)
{
    const long long nb = (long long)NG * NCH * g.KG;
    hipLaunchKernelGGL(plan_fill_kernel, dim3(blocks_for(nb, kBlock)), dim3(kBlock), 0, st, rowptr,
                       idx, val, K, R, S, g.CC, g.SLOTS, g.WAVES, NCH, NG, g.IN_ROWS, g.PITCH, g.BV, g.STRIDE,
                       segptr, recs);
    return hipGetLastError();
}

hipError_t launch_plan_fill_dense(const int *rowptr, const uint32_t *idx, const float *val, int K, int C,
                                  int R, int S, const SfGeom &g, int NCH, int NG, long long nrec, Rec *recs,
                                  hipStream_t st)
{
    const long long n = nrec > kPlanSpare ? nrec : kPlanSpare;
    hipLaunchKernelGGL(plan_fill_dense_kernel, dim3(blocks_for(n, kBlock)), dim3(kBlock), 0, st, rowptr, idx,
                       val, K, C, R, S, g.CC, g.SLOTS, g.WAVES, NCH, NG, g.IN_ROWS, g.PITCH, g.BV, nrec, recs);
    return hipGetLastError();
}

hipError_t launch_input_count(const float *x, int N, int C, int H, int W, int CC, int NCH, int *cnt,
                              hipStream_t st)
{
    const long long HW = (long long)H * W, npix = (long long)N * HW;
    hipLaunchKernelGGL(input_count_kernel, dim3(blocks_for(npix, kBlock), NCH), dim3(kBlock), 0, st, x, C,
                       HW, npix, CC, NCH, cnt);
    return hipGetLastError();
}

hipError_t launch_input_fill(const float *x, int N, int C, int H, int W, int CC, int NCH,
                             const int *cptr, uint32_t *cidx, float *xval, int spare, hipStream_t st)
{
    const long long HW = (long long)H * W, npix = (long long)N * HW;
    if (spare > kBlock) return hipErrorInvalidValue;
    // pixels per work-group: as many (up to 32) as keep the LDS image of their lists, 8 bytes per
    // possible entry, within 64 KB
    int PX = 32;
    while (PX > 1 && (long long)PX * NCH * CC * 8 > 65536) PX /= 2;
    const long long lds = (long long)PX * NCH * CC * 8;
    if (lds > 65536) return hipErrorInvalidValue;   // more than 8192 channels: not served
    hipLaunchKernelGGL(input_fill_kernel, dim3(blocks_for(npix, PX)), dim3(kBlock), (size_t)lds, st, x, C,
                       HW, npix, CC, NCH, PX, cptr, cidx, xval, spare);
    return hipGetLastError();
}

hipError_t launch_layout_convert(const float *src, int N, int C, int H, int W, int src_n4, float *dst,
                                 hipStream_t st)
{
    const long long CHW = (long long)C * H * W;
    const long long n = (long long)((N + 3) / 4) * CHW;
    hipLaunchKernelGGL(layout_convert_kernel, dim3(blocks_for(n, kBlock)), dim3(kBlock), 0, st, src, N,
                       CHW, src_n4, dst);
    return hipGetLastError();
}

hipError_t launch_maxpool2x2(const float *x, int N, int C, int H, int W, float *y, int n4,
                             hipStream_t st)
{
    const int Ho = H / 2, Wo = W / 2;
    if (n4) {
        const long long GC = (long long)((N + 3) / 4) * C;
        const long long m = GC * Ho * Wo;
        if (m == 0) return hipSuccess;
        hipLaunchKernelGGL(maxpool2x2_n4_kernel, dim3(blocks_for(m, kBlock)), dim3(kBlock), 0, st,
                           reinterpret_cast<const float4 *>(x), GC, H, W, Ho, Wo,
                           reinterpret_cast<float4 *>(y));
        return hipGetLastError();
    }
    const long long n = (long long)N * C * Ho * Wo;
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(maxpool2x2_kernel, dim3(blocks_for(n, kBlock)), dim3(kBlock), 0, st, x,
                       (long long)N * C, H, W, Ho, Wo, y);
    return hipGetLastError();
}

}  // namespace fscnn
