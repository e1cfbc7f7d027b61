/*
 * FSCNN oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct CPU statement of what the sparse-filter /
 * sparse-input convolution path computes.  Only the tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it.  It shares no code, header,
 * table or helper with the HIP library and never touches a GPU.
 *
 * What it follows (FSCNN, arXiv 2212.08815):
 *   - Sec. 3 ("Sparse Data Structure"): the CSR(C) description -- values B_v,
 *     column indices B_i, cumulative per-row counts B_c that start with 0 --
 *     applied to the K x (C*R*S) matrix of a filter bank (a sparse 4-D tensor
 *     is a list of sparse 3-D tensors with one pointer per tensor).
 *   - Sec. 4, Alg. 1 (single-filter sparse convolution) and Alg. 2 (sparse .
 *     dense inner product): the result is the ordinary un-flipped convolution
 *     sum in which only the terms with a nonzero weight are visited; output
 *     size (H_I - H_F)/S + 1.
 *   - Sec. 5, Alg. 6 (direct forward pass over all filters, C_O = number of
 *     filters) and "Other layers" (padding = same-shape output with shifted
 *     input index; activation = element-wise function on the output).
 *   - Sec. 4, last paragraph of the convolution item: the sparse-input case
 *     uses the same loops with the roles of sparse and dense operand swapped.
 *
 * The paper claims an exact convolution (Sec. 1, second contribution), so the
 * oracle is the definition written out: decompress, then seven nested loops.
 * Accumulation is in double with a single rounding to float at the end; the
 * paper's arithmetic type is 32-bit float (Sec. 6), any summation order of
 * which lies within fp32 accumulation error of this value.
 *
 * Readings of points the paper leaves open (each is listed again in the
 * repository's design notes):
 *   - cross-correlation (no kernel flip): Alg. 1 pairs T_I[l+jS][k+iS] with
 *     T_F[l][k];
 *   - floor division in the output-size formula; symmetric zero padding;
 *   - an entry is "nonzero" iff (value != 0.0f): -0.0 is dropped, NaN and
 *     denormals are kept, kept values are copied bit for bit;
 *   - node order inside a filter row is ascending flat index (c*R + r)*S + s;
 *   - bias (never mentioned in the paper) is added after the sum, before ReLU.
 *
 * Parity pins (tests/test_oracle_pins.py): pure-Python brute force with an
 * explicitly zero-padded copy of the input, impulse responses, integer-exact
 * data, 1x1 convolution == matrix product, a dense library convolution in
 * fp64, closed forms for all-ones data, linearity, numpy's nonzero() for the
 * compressed indices; for the two transposes a library CSR->CSC conversion,
 * numpy's nonzero() on the dense tensor in the target order, brute force and
 * the involution property.  No function here is "parity unpinned".
 *
 *   - Sec. 4, "Sparse Matrix Transpose" (Alg. 3) and "Sparse 3-D Tensor
 *     Transpose" (Alg. 4): what they compute is a re-ordering of the stored
 *     nodes with a plain definition -- the same (position, value) triples,
 *     listed in the target storage order -- so the oracle is that definition:
 *     gather the triples, sort them by the target order (positions are unique,
 *     so the order is total), count the nodes of each new row.  Ending nodes
 *     (index -1) are replaced by pointer arrays throughout, as for the filters.
 *   - Sec. 5 "Other layers" / Sec. 6.2: LeakyReLU is one of the element-wise
 *     activations applied to the output; act = 2 applies y > 0 ? y : slope * y
 *     to the double sum before the single rounding.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Output extent of one spatial axis: Alg. 1 step 3 / Alg. 6 step 3, extended
 * by symmetric padding p (Sec. 5 "Other layers"): floor((in + 2p - f)/s) + 1,
 * or 0 when the filter does not fit. */
int oracle_out_dim(int in, int f, int stride, int pad)
{
    int span = in + 2 * pad - f;
    if (in <= 0 || f <= 0 || stride <= 0 || pad < 0 || span < 0) return 0;
    return span / stride + 1;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Number of entries of w[0..n) that count as nonzero. */
long long oracle_count_nonzero(const float *w, long long n)
{
    long long cnt = 0;
    for (long long i = 0; i < n; ++i)
        if (w[i] != 0.0f) ++cnt;
    return cnt;
}

/* CSR(C) of the K x (C*R*S) filter matrix (Sec. 3): rowptr = B_c (K+1 entries,
 * starts with 0), idx = B_i (flat (c*R+r)*S+s, ascending inside a row),
 * val = B_v (bit copies).  idx/val must hold oracle_count_nonzero() entries. */
void oracle_filter_compress(const float *w, int K, int C, int R, int S,
                            int32_t *rowptr, uint32_t *idx, float *val)
{
    const long long row = (long long)C * R * S;
    long long n = 0;
    rowptr[0] = 0;
    for (int k = 0; k < K; ++k) {
        for (long long f = 0; f < row; ++f) {
            float v = w[(long long)k * row + f];
            if (v != 0.0f) {
                idx[n] = (uint32_t)f;
                memcpy(&val[n], &v, sizeof v);
                ++n;
            }
        }
        rowptr[k + 1] = (int32_t)n;
    }
}

/* Inverse of the above: scatter the stored values into a zeroed dense bank. */
void oracle_filter_decompress(const int32_t *rowptr, const uint32_t *idx, const float *val,
                              int K, int C, int R, int S, float *w)
{
    const long long row = (long long)C * R * S;
    memset(w, 0, sizeof(float) * (size_t)(K * row));
    for (int k = 0; k < K; ++k)
        for (int32_t i = rowptr[k]; i < rowptr[k + 1]; ++i)
            w[(long long)k * row + idx[i]] = val[i];
}

/* One output element of the convolution definition (Alg. 1 steps 5-12 with the
 * channel inner product of Alg. 2 written out densely).  Returns the double
 * sum; *abs_sum (optional) receives sum |w||x| (+|bias|) for error bounds. */
static double conv_point(const float *x, int C, int H, int W, const float *wk, int R, int S,
                         int sh, int sw, int ph, int pw, int oy, int ox, double *abs_sum)
{
    double a = 0.0, m = 0.0;
    for (int c = 0; c < C; ++c)
        for (int r = 0; r < R; ++r)
            for (int s = 0; s < S; ++s) {
                int iy = oy * sh - ph + r;
                int ix = ox * sw - pw + s;
                if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
                double t = (double)wk[((long long)c * R + r) * S + s] *
                           (double)x[((long long)c * H + iy) * W + ix];
                a += t;
                m += fabs(t);
            }
    if (abs_sum) *abs_sum = m;
    return a;
}

/* Bias, then the element-wise activation (Sec. 5 "Other layers"): relu = 0 none, 1 ReLU,
 * 2 LeakyReLU with the slope set by oracle_set_leaky_slope(). */
static double leaky_slope = 0.0;
void oracle_set_leaky_slope(double s) { leaky_slope = s; }

static float finish(double a, const float *bias, int k, int relu)
{
    if (bias) a += (double)bias[k];
    if (relu == 1) a = a > 0.0 ? a : 0.0;
    if (relu == 2) a = a > 0.0 ? a : a * leaky_slope;
    return (float)a;
}

/* Dense definition: y[n,k,oy,ox] = sum_{c,r,s} w[k,c,r,s] * x[n,c,oy*sh-ph+r,ox*sw-pw+s]
 * (+ bias[k]) (ReLU).  x: N x C x H x W, w: K x C x R x S, y: N x K x Ho x Wo, all
 * contiguous.  abs_sum may be NULL; otherwise same shape as y, holds
 * sum|w||x| + |bias| per element (double). */
void oracle_conv2d_dense(const float *x, int N, int C, int H, int W,
                         const float *w, int K, int R, int S,
                         int sh, int sw, int ph, int pw,
                         const float *bias, int relu, float *y, double *abs_sum)
{
    const int Ho = oracle_out_dim(H, R, sh, ph), Wo = oracle_out_dim(W, S, sw, pw);
    const long long xs = (long long)C * H * W, ws = (long long)C * R * S;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int oy = 0; oy < Ho; ++oy)
                for (int ox = 0; ox < Wo; ++ox) {
                    double m;
                    double a = conv_point(x + n * xs, C, H, W, w + k * ws, R, S,
                                          sh, sw, ph, pw, oy, ox, &m);
                    long long o = (((long long)n * K + k) * Ho + oy) * Wo + ox;
                    y[o] = finish(a, bias, k, relu);
                    if (abs_sum) abs_sum[o] = m + (bias ? fabs((double)bias[k]) : 0.0);
                }
}

/* Sparse-filter convolution (Alg. 6 over all filters): decompress the CSR(C)
 * bank, then apply the dense definition. */
int oracle_conv2d_sparse_filter(const float *x, int N, int C, int H, int W,
                                const int32_t *rowptr, const uint32_t *idx, const float *val,
                                int K, int R, int S, int sh, int sw, int ph, int pw,
                                const float *bias, int relu, float *y, double *abs_sum)
{
    float *w = (float *)malloc(sizeof(float) * (size_t)K * C * R * S);
    if (!w) return 1;
    oracle_filter_decompress(rowptr, idx, val, K, C, R, S, w);
    oracle_conv2d_dense(x, N, C, H, W, w, K, R, S, sh, sw, ph, pw, bias, relu, y, abs_sum);
    free(w);
    return 0;
}

/* The same definition at selected output elements only (flat indices into
 * y[N,K,Ho,Wo]); used to check full-size workloads the whole oracle cannot
 * finish in reasonable time. */
void oracle_conv2d_points(const float *x, int N, int C, int H, int W,
                          const float *w, int K, int R, int S,
                          int sh, int sw, int ph, int pw,
                          const float *bias, int relu,
                          const long long *flat, long long npts, float *out, double *abs_sum)
{
    const int Ho = oracle_out_dim(H, R, sh, ph), Wo = oracle_out_dim(W, S, sw, pw);
    const long long xs = (long long)C * H * W, ws = (long long)C * R * S;
    (void)N;
#pragma omp parallel for schedule(static)
    for (long long i = 0; i < npts; ++i) {
        long long o = flat[i];
        int ox = (int)(o % Wo); o /= Wo;
        int oy = (int)(o % Ho); o /= Ho;
        int k = (int)(o % K);
        int n = (int)(o / K);
        double m;
        double a = conv_point(x + n * xs, C, H, W, w + k * ws, R, S, sh, sw, ph, pw, oy, ox, &m);
        out[i] = finish(a, bias, k, relu);
        if (abs_sum) abs_sum[i] = m + (bias ? fabs((double)bias[k]) : 0.0);
    }
}

/* Compressed activation (sparse 3-D tensor in the paper's O_chw order, Sec. 3:
 * the channel run is innermost): one row per pixel in (n, iy, ix) raster order,
 * columns = channel indices ascending, entry kept iff x != 0.0f. */
long long oracle_input_compress(const float *x, int N, int C, int H, int W,
                                int32_t *prow, uint32_t *cidx, float *xval)
{
    long long n = 0, p = 0;
    prow[0] = 0;
    for (int b = 0; b < N; ++b)
        for (int iy = 0; iy < H; ++iy)
            for (int ix = 0; ix < W; ++ix) {
                for (int c = 0; c < C; ++c) {
                    float v = x[(((long long)b * C + c) * H + iy) * W + ix];
                    if (v != 0.0f) {
                        if (cidx) {
                            cidx[n] = (uint32_t)c;
                            memcpy(&xval[n], &v, sizeof v);
                        }
                        ++n;
                    }
                }
                prow[++p] = (int32_t)n;
            }
    return n;
}

void oracle_input_decompress(const int32_t *prow, const uint32_t *cidx, const float *xval,
                             int N, int C, int H, int W, float *x)
{
    memset(x, 0, sizeof(float) * (size_t)N * C * H * W);
    long long p = 0;
    for (int b = 0; b < N; ++b)
        for (int iy = 0; iy < H; ++iy)
            for (int ix = 0; ix < W; ++ix, ++p)
                for (int32_t i = prow[p]; i < prow[p + 1]; ++i)
                    x[(((long long)b * C + cidx[i]) * H + iy) * W + ix] = xval[i];
}

/* Sparse-input convolution (Sec. 4: sparse T_I, dense T_F): decompress the
 * activation, then the dense definition; the output is dense here. */
int oracle_conv2d_sparse_input(const int32_t *prow, const uint32_t *cidx, const float *xval,
                               int N, int C, int H, int W,
                               const float *w, int K, int R, int S,
                               int sh, int sw, int ph, int pw,
                               const float *bias, int relu, float *y, double *abs_sum)
{
    float *x = (float *)malloc(sizeof(float) * (size_t)N * C * H * W);
    if (!x) return 1;
    oracle_input_decompress(prow, cidx, xval, N, C, H, W, x);
    oracle_conv2d_dense(x, N, C, H, W, w, K, R, S, sh, sw, ph, pw, bias, relu, y, abs_sum);
    free(x);
    return 0;
}

/* Stand-alone 2x2 / stride-2 max pooling (Sec. 5 "Pooling Layers": pooling
 * applied directly to the previous layer's output; pooled size = floor(n/2),
 * Alg. 7 step 4).  Helper used only to chain VGG16-shaped layers. */
void oracle_maxpool2x2(const float *x, int N, int C, int H, int W, float *y)
{
    const int Ho = H / 2, Wo = W / 2;
#pragma omp parallel for schedule(static)
    for (long long nc = 0; nc < (long long)N * C; ++nc)
        for (int oy = 0; oy < Ho; ++oy)
            for (int ox = 0; ox < Wo; ++ox) {
                const float *p = x + (nc * H + 2 * oy) * W + 2 * ox;
                float m = p[0];
                if (p[1] > m) m = p[1];
                if (p[W] > m) m = p[W];
                if (p[W + 1] > m) m = p[W + 1];
                y[(nc * Ho + oy) * Wo + ox] = m;
            }
}

/* A stored node with its position in the target order: (major, minor) = (new row, index inside
 * the new row). */
typedef struct {
    long long major;
    uint32_t minor;
    float val;
} oracle_node;

static int node_cmp(const void *pa, const void *pb)
{
    const oracle_node *a = (const oracle_node *)pa, *b = (const oracle_node *)pb;
    if (a->major != b->major) return a->major < b->major ? -1 : 1;
    if (a->minor != b->minor) return a->minor < b->minor ? -1 : 1;
    return 0;
}

/* Lists nodes[0..nnz) in target order: sorted by (major, minor); tptr[r] = number of nodes
 * with major < r. */
static void emit_in_target_order(oracle_node *nodes, long long nnz, long long n_major,
                                 int32_t *tptr, uint32_t *tidx, float *tval)
{
    qsort(nodes, (size_t)nnz, sizeof(oracle_node), node_cmp);
    for (long long r = 0; r <= n_major; ++r) tptr[r] = 0;
    for (long long e = 0; e < nnz; ++e) {
        tptr[nodes[e].major + 1] += 1;
        tidx[e] = nodes[e].minor;
        memcpy(&tval[e], &nodes[e].val, sizeof(float));
    }
    for (long long r = 0; r < n_major; ++r) tptr[r + 1] += tptr[r];
}

/* Sparse matrix transpose (what Alg. 3 computes).  M has n_rows rows and n_cols columns and is
 * stored by rows: row i holds the nodes idx[rowptr[i] .. rowptr[i+1]) = column of each stored
 * entry, ascending, with its value.  The result stores the same entries by columns: new row j
 * (= old column) lists the old rows of its entries, ascending, with their values. */
void oracle_sparse_transpose(const int32_t *rowptr, const uint32_t *idx, const float *val,
                             int n_rows, int n_cols,
                             int32_t *tptr, uint32_t *tidx, float *tval)
{
    const long long nnz = rowptr[n_rows];
    oracle_node *nodes = (oracle_node *)malloc(sizeof(oracle_node) * (size_t)(nnz > 0 ? nnz : 1));
    for (int i = 0; i < n_rows; ++i)
        for (int32_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
            nodes[e].major = idx[e];          /* entry (i, j) becomes entry (j, i) */
            nodes[e].minor = (uint32_t)i;
            nodes[e].val = val[e];
        }
    emit_in_target_order(nodes, nnz, n_cols, tptr, tidx, tval);
    free(nodes);
}

/* Sparse 3-D tensor transpose from order O_whc to order O_chw (what Alg. 4 computes).
 * Input: C matrices stacked, matrix c stored in order O_wh, i.e. row (c*H + h) lists the w of
 * the stored entries of channel c at height h, ascending.  Output: order O_chw (channel runs
 * innermost, then height, then width): row (w*H + h) lists the c of the stored entries at that
 * pixel, ascending. */
void oracle_sparse_tensor_transpose(const int32_t *rowptr, const uint32_t *widx, const float *val,
                                    int W, int H, int C,
                                    int32_t *tptr, uint32_t *cidx, float *tval)
{
    const long long nnz = rowptr[(long long)C * H];
    oracle_node *nodes = (oracle_node *)malloc(sizeof(oracle_node) * (size_t)(nnz > 0 ? nnz : 1));
    for (int c = 0; c < C; ++c)
        for (int h = 0; h < H; ++h)
            for (int32_t e = rowptr[(long long)c * H + h]; e < rowptr[(long long)c * H + h + 1]; ++e) {
                nodes[e].major = (long long)widx[e] * H + h;   /* entry (w, h, c) goes to row w*H + h */
                nodes[e].minor = (uint32_t)c;
                nodes[e].val = val[e];
            }
    emit_in_target_order(nodes, nnz, (long long)W * H, tptr, cidx, tval);
    free(nodes);
}
