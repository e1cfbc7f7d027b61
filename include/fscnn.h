/*
 * fscnn.h -- C ABI of the MI355X (gfx950) sparse-filter / sparse-input 2-D
 * convolution library: the hot path of FSCNN (arXiv 2212.08815).
 *
 * Notation (paper -> here): input T_I (C_I x H_I x W_I) -> x[N,C,H,W], dense
 * NCHW fp32; filters T_F1..T_FN (C_F x H_F x W_F, C_F = C_I, C_O = N of the
 * paper's Sec. 5) -> w[K,C,R,S]; stride S of Alg. 1 -> (stride_h, stride_w);
 * output T_O -> y[N,K,Ho,Wo] with Ho = floor((H + 2*pad_h - R)/stride_h) + 1.
 *
 * Conventions for every entry point
 *   - "_dev" pointers are DEVICE pointers (HIP global memory on the current
 *     device), contiguous, 4-byte aligned, caller-owned; "_host" pointers are
 *     ordinary host memory.  Nothing is freed or retained by the library except
 *     the opaque handles it creates.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Every call returns a status and never throws or aborts.  All argument
 *     checks happen before any kernel is launched.
 *   - Handles are created and destroyed only by the library.  A handle may be
 *     used from several streams at once for convolution calls once the plan for
 *     the geometry exists (see fscnn_filter_prepare).
 *   - No entry point uses a CPU fallback: without a HIP device every compute
 *     call fails with FSCNN_ERR_DEVICE.
 */
#ifndef FSCNN_H
#define FSCNN_H

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fscnn_filter fscnn_filter_t; /* compressed filter bank (device buffers inside)   */
typedef struct fscnn_input fscnn_input_t;   /* compressed activation tensor (device buffers)    */

/* Status codes and layout codes travel as plain int, so that a caller's out-of-range value is an
 * ordinary integer the library can refuse rather than an invalid enumerator. */
typedef int fscnn_status_t;
enum {
    FSCNN_OK = 0,
    FSCNN_ERR_NULL = 1,        /* a required pointer is NULL                                   */
    FSCNN_ERR_SHAPE = 2,       /* non-positive size, negative pad, empty output, size overflow */
    FSCNN_ERR_MISMATCH = 3,    /* x / w dimensions, or the current device, disagree with the handle */
    FSCNN_ERR_UNSUPPORTED = 4, /* valid request outside what the kernels cover                 */
    FSCNN_ERR_ALLOC = 5,       /* device or host allocation failed                             */
    FSCNN_ERR_DEVICE = 6,      /* HIP runtime error (no device, launch failure, ...)           */
    FSCNN_ERR_HANDLE = 7       /* not a live handle (bad magic word / already destroyed)       */
};

const char *fscnn_status_string(fscnn_status_t s);

/* Memory layout of a 4-D activation tensor of N images.
 *   FSCNN_LAYOUT_NCHW: element (n,c,h,w) at ((n*C + c)*H + h)*W + w.
 *   FSCNN_LAYOUT_N4:   batch-interleaved by four: element (n,c,h,w) at
 *                      ((((n/4)*C + c)*H + h)*W + w)*4 + n%4; the buffer holds 4*ceil(N/4)
 *                      images and must be 16-byte aligned; the contents of the images past N are
 *                      unspecified on output and ignored on input.  This is the layout the
 *                      convolution kernel keeps in LDS (one 16-byte read feeds four images), so
 *                      chained layers that pass N4 tensors stage their input with contiguous
 *                      16-byte loads and store their output with 16-byte stores. */
typedef int fscnn_layout_t;
enum { FSCNN_LAYOUT_NCHW = 0, FSCNN_LAYOUT_N4 = 1 };

/* Output extent of a convolution (host only).  Alg. 1 step 3 and Alg. 6 step 3 give
 * (H_I - H_F)/S + 1; with the symmetric zero padding of Sec. 5 ("Other layers") this is
 * floor((H + 2*pad - R)/stride) + 1.  FSCNN_ERR_SHAPE if any size is non-positive, a pad
 * is negative or the filter does not fit. */
fscnn_status_t fscnn_conv2d_out_shape(int H, int W, int R, int S, int stride_h, int stride_w,
                                      int pad_h, int pad_w, int *Ho, int *Wo);

/* ------------------------------------------------------------------ sparse filters
 * Filter compression (Sec. 3: CSR(C) values / column indices / cumulative row counts, a
 * sparse 4-D tensor being one sparse 3-D tensor per filter with a pointer per filter).
 * w_dev: dense K x C x R x S fp32.  The handle holds, per output channel k, the entries
 * with w != 0.0f (-0.0 dropped, NaN/denormals kept, values copied bit for bit) in ascending
 * flat index (c*R + r)*S + s, i.e. sorted by input channel first.  Runs its kernels on
 * `stream` and synchronises it once (the nonzero count sizes the buffers).
 * K*C*R*S must be < 2^31.  *out is set only on FSCNN_OK. */
fscnn_status_t fscnn_filter_compress(const float *w_dev, int K, int C, int R, int S,
                                     void *stream, fscnn_filter_t **out);

/* Shape and nonzero count of a handle (any output pointer may be NULL). */
fscnn_status_t fscnn_filter_info(const fscnn_filter_t *f, int *K, int *C, int *R, int *S,
                                 long long *nnz);

/* Canonical CSR(C) view copied to HOST buffers: rowptr_host[K+1] (int32, starts with 0),
 * idx_host[nnz] (uint32 flat (c*R+r)*S+s), val_host[nnz] (fp32).  Synchronous. */
fscnn_status_t fscnn_filter_export(const fscnn_filter_t *f, int *rowptr_host,
                                   unsigned *idx_host, float *val_host);

/* Builds (once) the device-side plan the convolution kernel streams for this geometry:
 * the nonzeros regrouped by (output-channel group, wave, input-channel chunk, channel slot)
 * with each (c,r,s) packed into the byte offset of that tap inside the LDS input tile.
 * Allocates device memory, launches on `stream` and synchronises it once.  Optional:
 * fscnn_conv2d_sparse_filter builds the plan on first use; after that (or after this
 * call) convolution calls served by the same kernel configuration allocate nothing and do
 * not synchronise.  `variant` selects a kernel configuration (0 = automatic choice; see
 * fscnn_sf_variant_count).  The automatic choice depends on the tensor layouts and on the merged
 * pool: this call prepares for NCHW tensors without pooling, fscnn_filter_prepare_ex for the call
 * it is told about. */
fscnn_status_t fscnn_filter_prepare(fscnn_filter_t *f, int N, int H, int W, int stride_h,
                                    int stride_w, int pad_h, int pad_w, int variant,
                                    void *stream);

/* The same for a convolution call with these layouts and this pool flag (the arguments of
 * fscnn_conv2d_sparse_filter_ex / _pool2x2 / _leaky), to be issued on `stream`: builds the plan
 * of the configuration that call will resolve to and, when the call is small enough to run in
 * the channel-split mode (input channels divided over several work-groups, each storing its
 * partial sums into a scratch copy of the output that a finishing pass adds up in a fixed
 * order), that mode's scratch for `stream`.  Afterwards such calls on `stream` allocate nothing
 * and do not synchronise, which is what a caller that captures them into a HIP graph needs.
 * Without this call the first split-mode call of a handle on a stream allocates its scratch. */
fscnn_status_t fscnn_filter_prepare_ex(fscnn_filter_t *f, int N, int H, int W, int stride_h,
                                       int stride_w, int pad_h, int pad_w, fscnn_layout_t x_layout,
                                       fscnn_layout_t y_layout, int pool, int variant, void *stream);

/* Debug / test view of the plan chosen for a geometry (builds it if needed, synchronous; variant
 * 0 resolves as for NCHW tensors without pooling).  Writes the plan parameters into params_host[16]:
 *   [0] variant id  [1] CC channels per chunk  [2] KG output channels per group
 *   [3] number of chunks  [4] number of groups  [5] tile rows per channel
 *   [6] pitch (vectors per tile row)  [7] BV floats per vector (images interleaved)
 *   [8] records (= nonzeros)  [9] 1 if the direct (untiled) kernel serves this geometry
 *   [10] SLOTS channels per wave  [11] WAVES per group (KG = SLOTS*WAVES)
 *   [12] 1 for the taps-outer form (banks without zeros, few input channels); rest 0.
 * Bucket b = ((group*WAVES + wave)*chunks + chunk)*SLOTS + slot holds the entries of output
 * channel group*KG + wave*SLOTS + slot whose input channel lies in the chunk; a record's
 * byte offset is (((c mod CC)*rows + r)*pitch + s)*BV*4.  Where [12] is set the records are
 * laid out differently -- per (group, wave, chunk), CC*R*S groups of SLOTS records, one group
 * per tap (c mod CC, r, s) in ascending order, record j of a group = {the tap's byte offset,
 * the weight of channel group*KG + wave*SLOTS + j there, 0.0f where none is stored} -- [8] is
 * their number, and segptr still describes the stored entries as above.
 * If segptr_host / rec_off_host / rec_val_host are non-NULL they receive
 * segptr[groups*chunks*KG + 1], and per record the LDS byte offset and the weight.
 * Pass NULL pointers first to learn the sizes. */
fscnn_status_t fscnn_filter_plan_export(fscnn_filter_t *f, int N, int H, int W, int stride_h,
                                        int stride_w, int pad_h, int pad_w, int variant,
                                        int *params_host, int *segptr_host,
                                        unsigned *rec_off_host, float *rec_val_host);

fscnn_status_t fscnn_filter_destroy(fscnn_filter_t *f);

/* Number of selectable kernel configurations of the sparse-filter convolution and a short
 * description of each (variant ids are 1..count; 0 = automatic). */
int fscnn_sf_variant_count(void);
const char *fscnn_sf_variant_name(int variant);

/* Which kernel configuration the automatic choice (variant 0) takes for this filter and
 * geometry: *variant_out receives its id (1..count), or -1 when the untiled direct kernel
 * serves the geometry.  `n4` is nonzero if the input or the output tensor is in the N4
 * layout, `pool` if the merged 2x2 max-pool epilogue is asked for.  Host-only: launches
 * nothing and needs no device. */
fscnn_status_t fscnn_sf_variant_choice(const fscnn_filter_t *f, int N, int H, int W,
                                       int stride_h, int stride_w, int n4, int pool,
                                       int *variant_out);

/* How a launch of configuration `variant` (1..count) lays one or two images over the four image
 * slots of a lane: with NCHW tensors on both sides (`n4` zero) and N <= 2, a four-image
 * configuration gives the slots to *bands_out = 4 / N horizontal bands of *band_rows_out output
 * rows of each image (even where `pool` is nonzero), so that no slot computes on an image that is
 * not there; a band's halo rows are its neighbours' rows, and every output is still the sum over
 * its filter's stored entries in the order of the plan.  Otherwise *bands_out = 1 and
 * *band_rows_out = Ho.  Host-only. */
fscnn_status_t fscnn_sf_band_choice(int variant, int N, int Ho, int n4, int pool, int *bands_out,
                                    int *band_rows_out);

/* Sparse-filter convolution (Alg. 6: every output element, all filters; inner product of
 * Alg. 2 over the stored nonzeros only; no kernel flip; padding as index shift):
 *   y[n,k,oy,ox] = sum over stored (c,r,s,v) of filter k of
 *                  v * x[n,c,oy*stride_h - pad_h + r, ox*stride_w - pad_w + s]   (0 outside)
 *                  (+ bias_dev[k] if bias_dev != NULL) (then max(.,0) if relu != 0).
 * x_dev: N x C x H x W, y_dev: N x K x Ho x Wo (must not alias x), bias_dev: K or NULL.
 * fp32 accumulation in an order fixed by the plan: results are run-to-run identical.  For small
 * problems (at most 128 work-groups with the automatic configuration) the input-channel range is
 * split over several work-groups; each stores its partial sums into a copy of its own (scratch
 * that belongs to the handle's plan, one buffer per stream) and a finishing pass adds the copies
 * in the order of the parts, so this mode is reproducible too, but its sums are grouped
 * differently from those of an explicitly selected configuration (fscnn_conv2d_sparse_filter_v /
 * _ex with variant > 0), which never splits.
 * The batch may be of any size that N, and the number of work-groups, hold as an int: images are
 * addressed with 64-bit offsets.  One image is bounded: C*H*W and K*Ho*Wo must be below 2^31,
 * and beyond C*H*W*16 < 2^31 bytes the untiled direct kernel serves the call.
 * Asynchronous on `stream`.  FSCNN_ERR_MISMATCH if C differs from the handle's. */
fscnn_status_t fscnn_conv2d_sparse_filter(fscnn_filter_t *f, const float *x_dev, int N, int C,
                                          int H, int W, int stride_h, int stride_w, int pad_h,
                                          int pad_w, const float *bias_dev, int relu,
                                          float *y_dev, void *stream);

/* Same, with an explicit kernel configuration (benchmarks and parity tests walk all of
 * them).  FSCNN_ERR_UNSUPPORTED if that configuration cannot serve the geometry. */
fscnn_status_t fscnn_conv2d_sparse_filter_v(fscnn_filter_t *f, const float *x_dev, int N,
                                            int C, int H, int W, int stride_h, int stride_w,
                                            int pad_h, int pad_w, const float *bias_dev,
                                            int relu, float *y_dev, int variant, void *stream);

/* Same operation with explicit tensor layouts for x and y (see fscnn_layout_t) and an explicit
 * kernel configuration (0 = automatic).  N4 tensors need a configuration that keeps four
 * images per lane (the automatic choice does when N >= 4); FSCNN_ERR_UNSUPPORTED otherwise,
 * for strides other than (1,1) and, with 3x3 filters, (2,2), or if an N4 pointer is not 16-byte
 * aligned. */
fscnn_status_t fscnn_conv2d_sparse_filter_ex(fscnn_filter_t *f, const float *x_dev, int N,
                                             int C, int H, int W, int stride_h, int stride_w,
                                             int pad_h, int pad_w, const float *bias_dev,
                                             int relu, float *y_dev, fscnn_layout_t x_layout,
                                             fscnn_layout_t y_layout, int variant, void *stream);

/* The same convolution followed by LeakyReLU instead of ReLU (Sec. 5 "Other layers": an
 * element-wise activation applied to the output; the YOLO networks of Sec. 6 use this one):
 *   y = a > 0 ? a : negative_slope * a,   a = sum (+ bias).
 * negative_slope in [0, 1] (0 is ReLU, 1 the identity); FSCNN_ERR_SHAPE otherwise.  Batch-norm
 * layers fold into the weights and the bias beforehand and need no kernel support.  Other
 * arguments as fscnn_conv2d_sparse_filter_ex. */
fscnn_status_t fscnn_conv2d_sparse_filter_leaky(fscnn_filter_t *f, const float *x_dev, int N, int C,
                                                int H, int W, int stride_h, int stride_w,
                                                int pad_h, int pad_w, const float *bias_dev,
                                                float negative_slope, float *y_dev,
                                                fscnn_layout_t x_layout, fscnn_layout_t y_layout,
                                                int variant, void *stream);

/* Merged convolution + 2x2 / stride-2 max-pooling (Alg. 7: the convolution's elements update
 * a running maximum per pooling region and only the pooled values are stored; pooled extent
 * floor(Ho/2) x floor(Wo/2) as in its step 4).  Same arguments as
 * fscnn_conv2d_sparse_filter_ex, but y_dev is N x K x floor(Ho/2) x floor(Wo/2) in y_layout
 * and equals max-pooling applied to that call's output (bias and ReLU before the maximum).
 * FSCNN_ERR_SHAPE if Ho or Wo < 2; FSCNN_ERR_UNSUPPORTED where only the direct kernel applies
 * (strides other than 1, filters other than 3x3) or the configuration has no pooled form. */
fscnn_status_t fscnn_conv2d_sparse_filter_pool2x2(fscnn_filter_t *f, const float *x_dev, int N,
                                                  int C, int H, int W, int stride_h,
                                                  int stride_w, int pad_h, int pad_w,
                                                  const float *bias_dev, int relu, float *y_dev,
                                                  fscnn_layout_t x_layout,
                                                  fscnn_layout_t y_layout, int variant,
                                                  void *stream);

/* Layout conversion of an N x C x H x W tensor (src_layout != dst_layout, no aliasing).
 * Asynchronous on `stream`. */
fscnn_status_t fscnn_layout_convert(const float *src_dev, int N, int C, int H, int W,
                                    fscnn_layout_t src_layout, float *dst_dev,
                                    fscnn_layout_t dst_layout, void *stream);

/* ------------------------------------------------------------------ sparse inputs
 * Activation compression (Sec. 3, sparse 3-D tensor in order O_chw: the channel run is the
 * innermost list): one row per pixel in (n, iy, ix) raster order holding the (channel,
 * value) pairs with x != 0.0f, channel ascending.  C up to 8192 (beyond:
 * FSCNN_ERR_UNSUPPORTED).  Allocates the handle's buffers and
 * synchronises `stream` once (the number of stored values sizes them).  The pass that writes
 * the pairs is still queued on `stream` when the call returns: x_dev must stay valid until
 * the work queued on `stream` so far has run (stream order suffices), and the library
 * orders every later use of the handle, on any stream, behind that pass. */
fscnn_status_t fscnn_input_compress(const float *x_dev, int N, int C, int H, int W,
                                    void *stream, fscnn_input_t **out);
fscnn_status_t fscnn_input_info(const fscnn_input_t *in, int *N, int *C, int *H, int *W,
                                long long *nnz);
/* prow_host[N*H*W+1] int32, cidx_host[nnz] uint32, val_host[nnz] fp32.  Synchronous. */
fscnn_status_t fscnn_input_export(const fscnn_input_t *in, int *prow_host, unsigned *cidx_host,
                                  float *val_host);
fscnn_status_t fscnn_input_destroy(fscnn_input_t *in);

/* Sparse-filter convolution with sparse output (Sec. 4, the paragraph on sparse outputs of
 * "Sparse Tensor Convolution": only the non-zero results are kept as nodes, so that the
 * next layer can take a sparse input).  Computes y exactly as fscnn_conv2d_sparse_filter
 * does (NCHW x, bias nullable, relu as there) and returns it compressed as
 * fscnn_input_compress would: a handle of shape N x K x Ho x Wo whose pixel rows list the
 * (channel, value) pairs with y != 0.0f.  y_dev may be NULL; if it is not, the dense
 * N x K x Ho x Wo result is left there as well (caller-owned, must not alias x); with
 * y_dev NULL the dense result lives inside the handle's allocation.  The non-zero results are
 * counted in the convolution's own epilogue (per pixel and step of 8 output channels) where
 * the launch allows it -- small problems that run in the channel-split mode, and geometries
 * served by the direct kernel, count in a pass over the dense result instead -- then one scan and
 * one pass that writes the pairs.  The call makes ONE device allocation, sized for the worst
 * case (every result non-zero: 8 bytes per result), and does not wait for the device: it is
 * asynchronous on `stream`, x_dev (and y_dev) must stay valid until the work queued on
 * `stream` has run, and the library orders every later use of the handle, on any stream,
 * behind the pass that fills it.  fscnn_input_info / fscnn_input_export wait for that pass when
 * they are asked for the number of stored values.  *out is owned by the caller
 * (fscnn_input_destroy).  Errors as the two calls it stands for; on error *out is untouched. */
fscnn_status_t fscnn_conv2d_sparse_filter_emit(fscnn_filter_t *f, const float *x_dev, int N, int C,
                                               int H, int W, int stride_h, int stride_w,
                                               int pad_h, int pad_w, const float *bias_dev,
                                               int relu, float *y_dev, void *stream,
                                               fscnn_input_t **out);
/* The same into a handle that an earlier fscnn_conv2d_sparse_filter_emit returned for a result
 * of the same shape N x K x Ho x Wo (else FSCNN_ERR_MISMATCH; a handle of another origin:
 * FSCNN_ERR_UNSUPPORTED; y_dev NULL with a handle made with a y_dev: FSCNN_ERR_NULL): the
 * handle's previous contents are replaced.  Allocates nothing and does not wait for the
 * device -- the form for a loop that runs the same layer again and again.  The caller orders
 * the call behind every use of the handle's previous contents (stream order on one stream
 * suffices); on error the handle's contents are undefined but it can be refilled or destroyed. */
fscnn_status_t fscnn_conv2d_sparse_filter_emit_into(fscnn_filter_t *f, const float *x_dev, int N,
                                                    int C, int H, int W, int stride_h,
                                                    int stride_w, int pad_h, int pad_w,
                                                    const float *bias_dev, int relu, float *y_dev,
                                                    void *stream, fscnn_input_t *into);

/* Sparse-input convolution (Sec. 4, last paragraph of "Sparse Tensor Convolution": the
 * loops of Alg. 1 with a sparse T_I and dense filters; zero activations are skipped):
 * same result definition as above with w_dev the dense K x C x R x S bank.  The output is
 * written dense (N x K x Ho x Wo).  Every output element has one writer (a gather, no
 * atomics).  Asynchronous on `stream`; allocates nothing. */
fscnn_status_t fscnn_conv2d_sparse_input(const fscnn_input_t *in, const float *w_dev, int K,
                                         int R, int S, int stride_h, int stride_w, int pad_h,
                                         int pad_w, const float *bias_dev, int relu,
                                         float *y_dev, void *stream);

/* ------------------------------------------------------------------ helper
 * Stand-alone 2x2 / stride-2 max pooling (Sec. 5 "Pooling Layers": pooling applied directly
 * to the previous layer's output; output size floor(H/2) x floor(W/2) as in Alg. 7 step 4).
 * Only used to chain VGG16-shaped layers; not part of the measured convolution path. */
fscnn_status_t fscnn_maxpool2x2(const float *x_dev, int N, int C, int H, int W, float *y_dev,
                                void *stream);
/* Same on tensors of the given layout (input and output share it). */
fscnn_status_t fscnn_maxpool2x2_ex(const float *x_dev, int N, int C, int H, int W, float *y_dev,
                                   fscnn_layout_t layout, void *stream);

/* Dense filter bank prepared for the sparse-input convolution: a K-contiguous copy
 * wT[c][r][s][k] of w_dev (K x C x R x S, device, contiguous) that the library owns, built by one
 * launch on `stream` (no synchronisation: use the handle on the same stream, or synchronise
 * before using it elsewhere).  w_dev may be released once that launch has run. */
typedef struct fscnn_dense fscnn_dense_t;
fscnn_status_t fscnn_dense_filter_prepare(const float *w_dev, int K, int C, int R, int S, void *stream,
                                          fscnn_dense_t **out);
fscnn_status_t fscnn_dense_filter_destroy(fscnn_dense_t *d);

/* fscnn_conv2d_sparse_input on a prepared filter bank (same result, Sec. 4 as above): lanes
 * own adjacent output channels and read their weights as 8- or 16-byte vectors, weight chunks
 * arrive by direct-to-LDS loads.  3x3 filters at stride 1 only (FSCNN_ERR_UNSUPPORTED otherwise:
 * use fscnn_conv2d_sparse_input).  variant: 0 = automatic, 1..fscnn_si_variant_count() = an
 * explicit kernel configuration (tests and benchmarks walk them).  Allocates nothing,
 * asynchronous on `stream`; y_dev: N x K x Ho x Wo, must not alias the operands. */
fscnn_status_t fscnn_conv2d_sparse_input_prepared(const fscnn_input_t *in, const fscnn_dense_t *d,
                                                  int stride_h, int stride_w, int pad_h, int pad_w,
                                                  const float *bias_dev, int relu, float *y_dev,
                                                  int variant, void *stream);
int fscnn_si_variant_count(void);

/* Sparse matrix transpose (Sec. 4 "Sparse Matrix Transpose", Alg. 3).  M is n_rows x n_cols,
 * stored by rows: rowptr_dev[n_rows+1] (starts with 0, rowptr[n_rows] = nnz), idx_dev[nnz] =
 * column of each stored node, strictly ascending inside a row, val_dev[nnz].  The result stores
 * the same nodes by columns: tptr_dev[n_cols+1], tidx_dev[nnz] = old row of each node, ascending
 * inside a new row, tval_dev[nnz] (bit copies).  Ending nodes of the paper's layout are replaced
 * by the pointer arrays.  All pointers are caller-owned device memory and must not alias;
 * workspace_dev is scratch of at least fscnn_sparse_transpose_workspace(n_cols, nnz) bytes,
 * 4-byte aligned.  Allocates nothing, asynchronous on `stream`.  A node whose index is not below
 * n_cols is dropped (never followed); rows that repeat an index give an unspecified result.
 * ERR_UNSUPPORTED if the workspace is too small or the shape exceeds the scratch format. */
fscnn_status_t fscnn_sparse_transpose(const int *rowptr_dev, const unsigned *idx_dev,
                                      const float *val_dev, int n_rows, int n_cols, long long nnz,
                                      int *tptr_dev, unsigned *tidx_dev, float *tval_dev,
                                      void *workspace_dev, long long workspace_bytes, void *stream);

/* fscnn_sparse_transpose for callers that cannot allocate device memory or bring a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * operands, same result, but the scratch is a static device array inside the library, 8 MiB per
 * GPU, held until the process ends.  ERR_UNSUPPORTED when fscnn_sparse_transpose_workspace(n_cols,
 * nnz) exceeds 8 MiB (about n_cols + nnz <= 1 000 000).  Calls no hipMalloc / hipFree and no
 * allocating library routine, clears its counters with a kernel (no memset node) and does not
 * synchronise.  All calls on one GPU share that GPU's array: two calls that overlap on one GPU
 * (different streams, or threads) race; calls on one stream are ordered and safe. */
fscnn_status_t fscnn_sparse_transpose_noalloc(const int *rowptr_dev, const unsigned *idx_dev,
                                              const float *val_dev, int n_rows, int n_cols,
                                              long long nnz, int *tptr_dev, unsigned *tidx_dev,
                                              float *tval_dev, void *stream);

/* Sparse 3-D tensor transpose from order O_whc to order O_chw (Sec. 4 "Sparse 3-D Tensor
 * Transpose", Alg. 4).  Input: a W x H x C tensor as C stacked matrices in order O_wh: row
 * c*H + h of rowptr_dev[C*H+1] lists in widx_dev the w of its stored nodes, strictly ascending.
 * Output: order O_chw (channel innermost, then height, then width): row w*H + h of
 * tptr_dev[W*H+1] lists in cidx_dev the c of its nodes, ascending; tval_dev are bit copies.
 * Workspace: fscnn_sparse_transpose_workspace(W*H, nnz) bytes.  Otherwise as fscnn_sparse_transpose. */
fscnn_status_t fscnn_sparse_tensor_transpose(const int *rowptr_dev, const unsigned *widx_dev,
                                             const float *val_dev, int W, int H, int C,
                                             long long nnz, int *tptr_dev, unsigned *cidx_dev,
                                             float *tval_dev, void *workspace_dev,
                                             long long workspace_bytes, void *stream);

/* Scratch bytes the two transposes need for a result of `new_rows` rows and `nnz` stored nodes
 * (proportional to new_rows + nnz); -1 if either is not positive / negative or not below 2^31.
 * Host-only. */
long long fscnn_sparse_transpose_workspace(long long new_rows, long long nnz);

#ifdef __cplusplus
}
#endif
#endif /* FSCNN_H */
