// C-ABI entry points of libfscnn.so (declared and documented in include/fscnn.h):
// argument validation, handle management, plan caching, kernel dispatch.  No arithmetic of
// the method happens on the host.
#include <limits.h>

#include <new>

#include "internal.h"

using namespace fscnn;

namespace {

#define FSCNN_HIP(expr)                            \
    do {                                           \
        hipError_t e_ = (expr);                    \
        if (e_ != hipSuccess) {                    \
            (void)hipGetLastError();               \
            return e_ == hipErrorOutOfMemory ? FSCNN_ERR_ALLOC : FSCNN_ERR_DEVICE; \
        }                                          \
    } while (0)

fscnn_status_t out_shape(int H, int W, int R, int S, int sh, int sw, int ph, int pw, int *Ho, int *Wo)
{
    if (H <= 0 || W <= 0 || R <= 0 || S <= 0 || sh <= 0 || sw <= 0 || ph < 0 || pw < 0)
        return FSCNN_ERR_SHAPE;
    const long long spanh = (long long)H + 2LL * ph - R;
    const long long spanw = (long long)W + 2LL * pw - S;
    if (spanh < 0 || spanw < 0) return FSCNN_ERR_SHAPE;
    const long long ho = spanh / sh + 1, wo = spanw / sw + 1;
    if (ho > INT_MAX || wo > INT_MAX) return FSCNN_ERR_SHAPE;
    *Ho = (int)ho;
    *Wo = (int)wo;
    return FSCNN_OK;
}

bool fits_int(long long v) { return v > 0 && v < (1LL << 31); }

fscnn_status_t have_device(int *dev)
{
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || n <= 0) {
        (void)hipGetLastError();
        return FSCNN_ERR_DEVICE;
    }
    if (hipGetDevice(dev) != hipSuccess) {
        (void)hipGetLastError();
        return FSCNN_ERR_DEVICE;
    }
    return FSCNN_OK;
}

bool live(const fscnn_filter_t *f) { return f && f->magic == kFilterMagic; }
bool live(const fscnn_input_t *i) { return i && i->magic == kInputMagic; }
bool live(const fscnn_dense_t *d) { return d && d->magic == kDenseMagic; }

void free_plan(SfPlan *p)
{
    if (!p) return;
    if (p->segptr) (void)hipFree(p->segptr);
    if (p->recs) (void)hipFree(p->recs);
    for (auto &sc : p->split)
        if (sc.buf) (void)hipFree(sc.buf);
    delete p;
}

// Scratch of the channel-split mode for a call on `st`: the buffer this stream used before if it is
// large enough, else a new one (the first such call of a plan on a stream allocates; replacing a
// buffer that is too small waits for the stream's earlier work on it).  One buffer per stream:
// calls that share a handle on different streams never share scratch.
fscnn_status_t split_scratch(fscnn_filter_t *f, SfPlan *p, hipStream_t st, size_t bytes, float **out)
{
    std::lock_guard<std::mutex> lock(f->mu);
    for (auto &sc : p->split)
        if (sc.stream == st) {
            if (sc.bytes < bytes) {
                float *nb = nullptr;
                if (hipMalloc(&nb, bytes) != hipSuccess) {
                    (void)hipGetLastError();
                    return FSCNN_ERR_ALLOC;
                }
                (void)hipStreamSynchronize(st);
                (void)hipFree(sc.buf);
                sc.buf = nb;
                sc.bytes = bytes;
            }
            *out = sc.buf;
            return FSCNN_OK;
        }
    float *nb = nullptr;
    if (hipMalloc(&nb, bytes) != hipSuccess) {
        (void)hipGetLastError();
        return FSCNN_ERR_ALLOC;
    }
    p->split.push_back({st, nb, bytes});
    *out = nb;
    return FSCNN_OK;
}

// Returns the plan of `variant` (>= 1) for this handle, building it on `st` when absent.
// variant == -1 stands for the direct kernel (no device data besides the canonical CSR).
fscnn_status_t get_plan(fscnn_filter_t *f, int variant, hipStream_t st, SfPlan **out)
{
    std::lock_guard<std::mutex> lock(f->mu);
    for (SfPlan *p : f->plans)
        if (p->variant == variant) {
            *out = p;
            return FSCNN_OK;
        }
    SfPlan *p = new (std::nothrow) SfPlan();
    if (!p) return FSCNN_ERR_ALLOC;
    p->variant = variant;
    if (variant == -1) {
        p->direct = true;
        f->plans.push_back(p);
        *out = p;
        return FSCNN_OK;
    }
    // the configuration (validated against the call's stride by resolve_variant) fixes the stride
    if (!sf_variant_geom(variant, f->R, f->S, 1, 1, &p->g) && !sf_variant_geom(variant, f->R, f->S, 2, 2, &p->g)) {
        delete p;
        return FSCNN_ERR_UNSUPPORTED;
    }
    const SfGeom &g = p->g;
    p->NCH = (f->C + g.CC - 1) / g.CC;
    p->NG = (f->K + g.KG - 1) / g.KG;
    const long long nb = (long long)p->NG * p->NCH * g.KG;
    // records: one per stored value; the taps-outer form lists every tap of every chunk instead
    const long long cap = g.DENSE ? (long long)p->NG * g.WAVES * p->NCH * g.CC * f->R * f->S * g.SLOTS : f->nnz;
    if (!fits_int(nb + 1) || cap + kPlanSpare >= (1LL << 31)) {
        delete p;
        return FSCNN_ERR_UNSUPPORTED;
    }
    // the plan is built next to the handle's arrays
    int dev;
    fscnn_status_t ds = have_device(&dev);
    if (ds == FSCNN_OK && dev != f->device) ds = FSCNN_ERR_MISMATCH;
    if (ds != FSCNN_OK) {
        delete p;
        return ds;
    }
    int *cnt = nullptr;
    hipError_t e = hipMalloc(&cnt, sizeof(int) * (size_t)(nb + scan_tmp_elems(nb)));
    if (e == hipSuccess) e = hipMalloc(&p->segptr, sizeof(int) * (size_t)(nb + 1));
    if (e == hipSuccess) e = hipMalloc(&p->recs, sizeof(Rec) * (size_t)(cap + kPlanSpare));
    if (e == hipSuccess)
        e = launch_plan_count(f->rowptr, f->idx, f->K, f->R * f->S, g, p->NCH, p->NG, cnt, st);
    if (e == hipSuccess) e = launch_exclusive_scan(cnt, p->segptr, nb, cnt + nb, st);
    if (e == hipSuccess)
        e = g.DENSE ? launch_plan_fill_dense(f->rowptr, f->idx, f->val, f->K, f->C, f->R, f->S, g, p->NCH,
                                             p->NG, cap, p->recs, st)
                    : launch_plan_fill(f->rowptr, f->idx, f->val, f->K, f->R, f->S, g, p->NCH, p->NG,
                                       p->segptr, p->recs, st);
    // The plan may be used from other streams and `cnt` is released here: wait for the build.
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (cnt) (void)hipFree(cnt);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        free_plan(p);
        return e == hipErrorOutOfMemory ? FSCNN_ERR_ALLOC : FSCNN_ERR_DEVICE;
    }
    p->nrec = cap;
    f->plans.push_back(p);
    *out = p;
    return FSCNN_OK;
}

// Which variant serves this geometry: `variant` > 0 is taken as is (checked), 0 = automatic,
// anything the tiled kernel cannot do goes to the direct kernel (-1).
fscnn_status_t resolve_variant(const fscnn_filter_t *f, int N, int H, int W, int sh, int sw,
                               int variant, int *resolved, bool n4 = false, bool pool = false)
{
    // the tiled kernel serves strides 1 and 2 (equal on both axes) and addresses up to four
    // images' channels with 32-bit byte offsets
    const bool tiled_ok = sh == sw && (sh == 1 || sh == 2) && (long long)f->C * H * W * 16 < 0x7ffffff0LL;
    if (variant < 0 || variant > sf_variant_count()) return FSCNN_ERR_UNSUPPORTED;
    if (variant > 0) {
        SfGeom g;
        if (!tiled_ok || !sf_variant_geom(variant, f->R, f->S, sh, sw, &g)) return FSCNN_ERR_UNSUPPORTED;
        *resolved = variant;
        return FSCNN_OK;
    }
    // N4 tensors need four images per lane whatever the batch size; the choice goes by the
    // output's extent (about the input's divided by the stride)
    const bool no_zeros = f->nnz == (long long)f->K * f->C * f->R * f->S;
    // one or two images through NCHW tensors: the four-image forms, their image slots filled with
    // bands of the image (sf_choose_bands), so the choice sees four slots of a quarter (half) the height
    int slots = n4 && N < 4 ? 4 : N, rows = (H + sh - 1) / sh;
    const bool banded = !n4 && N <= 2;
    if (banded) {
        rows = (rows + 4 / N - 1) / (4 / N);
        slots = 4;
    }
    int v = tiled_ok ? sf_choose_variant(slots, f->C, f->K, rows, (W + sw - 1) / sw, f->R, f->S, sh, pool, n4,
                                         no_zeros, banded)
                     : 0;
    *resolved = v > 0 ? v : -1;
    return FSCNN_OK;
}

// Number of stored values of a compressed activation.  A handle made without a host synchronisation
// (sparse output emission) learns it here: wait for the pass that filled it, read the pointer array's
// last element.  Returns -1 on a runtime error.
long long input_nnz(const fscnn_input_t *in)
{
    if (in->nnz >= 0) return in->nnz;
    int total = 0;
    const size_t last = (size_t)in->N * in->H * in->W * (size_t)in->NCH;
    if (hipEventSynchronize(in->filled) != hipSuccess ||
        hipMemcpy(&total, in->cptr + last, sizeof(int), hipMemcpyDeviceToHost) != hipSuccess) {
        (void)hipGetLastError();
        return -1;
    }
    const_cast<fscnn_input_t *>(in)->nnz = total;   // a cache of what the device holds
    return total;
}

// Orders work on `st` behind the pass that fills a compressed-activation handle (it runs on the
// stream the handle was made on and may still be in flight).
hipError_t after_fill(const fscnn_input_t *in, hipStream_t st)
{
    return st == in->made_on ? hipSuccess : hipStreamWaitEvent(st, in->filled, 0);
}

fscnn_status_t check_conv_args(const fscnn_filter_t *f, const float *x, int N, int C, int H, int W,
                               int sh, int sw, int ph, int pw, const float *y, int *Ho, int *Wo)
{
    if (!f || !x || !y) return FSCNN_ERR_NULL;
    if (!live(f)) return FSCNN_ERR_HANDLE;
    if (N <= 0 || C <= 0) return FSCNN_ERR_SHAPE;
    fscnn_status_t s = out_shape(H, W, f->R, f->S, sh, sw, ph, pw, Ho, Wo);
    if (s != FSCNN_OK) return s;
    if (C != f->C) return FSCNN_ERR_MISMATCH;
    // one image's tensors are indexed with ints; images are addressed with 64-bit offsets, so the
    // batch is bounded only by the number of work-groups a launch can have (checked there)
    if (!fits_int((long long)C * H * W) || !fits_int((long long)f->K * *Ho * *Wo)) return FSCNN_ERR_UNSUPPORTED;
    if (x == y) return FSCNN_ERR_UNSUPPORTED;
    return FSCNN_OK;
}

}  // namespace

extern "C" {

const char *fscnn_status_string(fscnn_status_t s)
{
    switch (s) {
        case FSCNN_OK: return "ok";
        case FSCNN_ERR_NULL: return "null pointer argument";
        case FSCNN_ERR_SHAPE: return "invalid shape (non-positive size, negative pad or empty output)";
        case FSCNN_ERR_MISMATCH: return "tensor dimensions do not match the handle";
        case FSCNN_ERR_UNSUPPORTED: return "request outside what the kernels cover";
        case FSCNN_ERR_ALLOC: return "allocation failed";
        case FSCNN_ERR_DEVICE: return "HIP runtime error or no device";
        case FSCNN_ERR_HANDLE: return "not a live handle";
    }
    return "unknown status";
}

fscnn_status_t fscnn_conv2d_out_shape(int H, int W, int R, int S, int sh, int sw, int ph, int pw,
                                      int *Ho, int *Wo)
{
    if (!Ho || !Wo) return FSCNN_ERR_NULL;
    return out_shape(H, W, R, S, sh, sw, ph, pw, Ho, Wo);
}

fscnn_status_t fscnn_filter_compress(const float *w_dev, int K, int C, int R, int S, void *stream,
                                     fscnn_filter_t **out)
{
    if (!w_dev || !out) return FSCNN_ERR_NULL;
    if (K <= 0 || C <= 0 || R <= 0 || S <= 0) return FSCNN_ERR_SHAPE;
    const long long row = (long long)C * R * S;
    if (!fits_int(row) || !fits_int(row * K)) return FSCNN_ERR_SHAPE;
    int dev;
    fscnn_status_t s = have_device(&dev);
    if (s != FSCNN_OK) return s;
    hipStream_t st = (hipStream_t)stream;

    fscnn_filter_t *f = new (std::nothrow) fscnn_filter();
    if (!f) return FSCNN_ERR_ALLOC;
    f->magic = kFilterMagic;
    f->device = dev;
    f->K = K; f->C = C; f->R = R; f->S = S;
    f->nnz = 0;
    f->rowptr = nullptr; f->idx = nullptr; f->val = nullptr;
    int *cnt = nullptr;
    int total = 0;
    hipError_t e = hipMalloc(&cnt, sizeof(int) * (size_t)(K + scan_tmp_elems(K)));
    if (e == hipSuccess) e = hipMalloc(&f->rowptr, sizeof(int) * (size_t)(K + 1));
    if (e == hipSuccess) e = launch_filter_count(w_dev, K, row, cnt, st);
    if (e == hipSuccess) e = launch_exclusive_scan(cnt, f->rowptr, K, cnt + K, st);
    if (e == hipSuccess)
        e = hipMemcpyAsync(&total, f->rowptr + K, sizeof(int), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e == hipSuccess) {
        f->nnz = total;
        const size_t n = total > 0 ? (size_t)total : 1;
        e = hipMalloc(&f->idx, sizeof(uint32_t) * n);
        if (e == hipSuccess) e = hipMalloc(&f->val, sizeof(float) * n);
    }
    if (e == hipSuccess) e = launch_filter_pack(w_dev, K, row, f->rowptr, f->idx, f->val, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (cnt) (void)hipFree(cnt);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        if (f->rowptr) (void)hipFree(f->rowptr);
        if (f->idx) (void)hipFree(f->idx);
        if (f->val) (void)hipFree(f->val);
        f->magic = 0;
        delete f;
        return e == hipErrorOutOfMemory ? FSCNN_ERR_ALLOC : FSCNN_ERR_DEVICE;
    }
    *out = f;
    return FSCNN_OK;
}

fscnn_status_t fscnn_filter_info(const fscnn_filter_t *f, int *K, int *C, int *R, int *S,
                                 long long *nnz)
{
    if (!f) return FSCNN_ERR_NULL;
    if (!live(f)) return FSCNN_ERR_HANDLE;
    if (K) *K = f->K;
    if (C) *C = f->C;
    if (R) *R = f->R;
    if (S) *S = f->S;
    if (nnz) *nnz = f->nnz;
    return FSCNN_OK;
}

fscnn_status_t fscnn_filter_export(const fscnn_filter_t *f, int *rowptr_host, unsigned *idx_host,
                                   float *val_host)
{
    if (!f || !rowptr_host) return FSCNN_ERR_NULL;
    if (!live(f)) return FSCNN_ERR_HANDLE;
    if (f->nnz > 0 && (!idx_host || !val_host)) return FSCNN_ERR_NULL;
    FSCNN_HIP(hipMemcpy(rowptr_host, f->rowptr, sizeof(int) * (size_t)(f->K + 1), hipMemcpyDeviceToHost));
    if (f->nnz > 0) {
        FSCNN_HIP(hipMemcpy(idx_host, f->idx, sizeof(uint32_t) * (size_t)f->nnz, hipMemcpyDeviceToHost));
        FSCNN_HIP(hipMemcpy(val_host, f->val, sizeof(float) * (size_t)f->nnz, hipMemcpyDeviceToHost));
    }
    return FSCNN_OK;
}

fscnn_status_t fscnn_filter_prepare_ex(fscnn_filter_t *f, int N, int H, int W, int sh, int sw, int ph,
                                       int pw, fscnn_layout_t x_layout, fscnn_layout_t y_layout, int pool,
                                       int variant, void *stream)
{
    if (!f) return FSCNN_ERR_NULL;
    if (!live(f)) return FSCNN_ERR_HANDLE;
    if (N <= 0) return FSCNN_ERR_SHAPE;
    if ((x_layout != FSCNN_LAYOUT_NCHW && x_layout != FSCNN_LAYOUT_N4) ||
        (y_layout != FSCNN_LAYOUT_NCHW && y_layout != FSCNN_LAYOUT_N4))
        return FSCNN_ERR_UNSUPPORTED;
    int Ho, Wo;
    fscnn_status_t s = out_shape(H, W, f->R, f->S, sh, sw, ph, pw, &Ho, &Wo);
    if (s != FSCNN_OK) return s;
    const int in4 = x_layout == FSCNN_LAYOUT_N4, out4 = y_layout == FSCNN_LAYOUT_N4;
    int v;
    s = resolve_variant(f, N, H, W, sh, sw, variant, &v, in4 || out4, pool != 0);
    if (s != FSCNN_OK) return s;
    if ((in4 || out4 || pool) && v < 0) return FSCNN_ERR_UNSUPPORTED;
    if (v > 0 && !sf_variant_has_layout(v, in4, out4, pool)) return FSCNN_ERR_UNSUPPORTED;
    SfPlan *p;
    s = get_plan(f, v, (hipStream_t)stream, &p);
    if (s != FSCNN_OK || p->direct) return s;
    // the same decisions as the convolution call takes
    int band_shift, band_h;
    sf_choose_bands(v, N, Ho, in4 || out4, pool != 0, &band_shift, &band_h);
    const int csplit = variant == 0 ? sf_choose_csplit(v, N << band_shift, f->K, band_h, Wo, p->NCH) : 1;
    if (csplit > 1) {
        float *parts;
        s = split_scratch(f, p, (hipStream_t)stream,
                          sizeof(float) * (size_t)csplit * (size_t)sf_split_elems(N, f->K, Ho, Wo, out4), &parts);
    }
    return s;
}

fscnn_status_t fscnn_filter_prepare(fscnn_filter_t *f, int N, int H, int W, int sh, int sw, int ph,
                                    int pw, int variant, void *stream)
{
    return fscnn_filter_prepare_ex(f, N, H, W, sh, sw, ph, pw, FSCNN_LAYOUT_NCHW, FSCNN_LAYOUT_NCHW, 0, variant,
                                   stream);
}

fscnn_status_t fscnn_filter_plan_export(fscnn_filter_t *f, int N, int H, int W, int sh, int sw,
                                        int ph, int pw, int variant, int *params_host,
                                        int *segptr_host, unsigned *rec_off_host,
                                        float *rec_val_host)
{
    if (!f || !params_host) return FSCNN_ERR_NULL;
    if (!live(f)) return FSCNN_ERR_HANDLE;
    if (N <= 0) return FSCNN_ERR_SHAPE;
    int Ho, Wo;
    fscnn_status_t s = out_shape(H, W, f->R, f->S, sh, sw, ph, pw, &Ho, &Wo);
    if (s != FSCNN_OK) return s;
    int v;
    s = resolve_variant(f, N, H, W, sh, sw, variant, &v);
    if (s != FSCNN_OK) return s;
    SfPlan *p;
    s = get_plan(f, v, nullptr, &p);
    if (s != FSCNN_OK) return s;
    for (int i = 0; i < 16; ++i) params_host[i] = 0;
    params_host[0] = p->variant;
    params_host[9] = p->direct ? 1 : 0;
    if (p->direct) return FSCNN_OK;
    params_host[1] = p->g.CC;
    params_host[2] = p->g.KG;
    params_host[3] = p->NCH;
    params_host[4] = p->NG;
    params_host[5] = p->g.IN_ROWS;
    params_host[6] = p->g.PITCH;
    params_host[7] = p->g.BV;
    params_host[8] = (int)p->nrec;
    params_host[10] = p->g.SLOTS;
    params_host[11] = p->g.WAVES;
    params_host[12] = p->g.DENSE;
    const long long nb = (long long)p->NG * p->NCH * p->g.KG;
    if (segptr_host)
        FSCNN_HIP(hipMemcpy(segptr_host, p->segptr, sizeof(int) * (size_t)(nb + 1), hipMemcpyDeviceToHost));
    if ((rec_off_host || rec_val_host) && p->nrec > 0) {
        if (!rec_off_host || !rec_val_host) return FSCNN_ERR_NULL;
        Rec *tmp = new (std::nothrow) Rec[(size_t)p->nrec];
        if (!tmp) return FSCNN_ERR_ALLOC;
        hipError_t e = hipMemcpy(tmp, p->recs, sizeof(Rec) * (size_t)p->nrec, hipMemcpyDeviceToHost);
        if (e == hipSuccess)
            for (long long i = 0; i < p->nrec; ++i) {
                rec_off_host[i] = tmp[i].off;
                rec_val_host[i] = tmp[i].val;
            }
        delete[] tmp;
        FSCNN_HIP(e);
    }
    return FSCNN_OK;
}

fscnn_status_t fscnn_filter_destroy(fscnn_filter_t *f)
{
    if (!f) return FSCNN_ERR_NULL;
    if (!live(f)) return FSCNN_ERR_HANDLE;
    f->magic = 0;
    for (SfPlan *p : f->plans) free_plan(p);
    f->plans.clear();
    if (f->rowptr) (void)hipFree(f->rowptr);
    if (f->idx) (void)hipFree(f->idx);
    if (f->val) (void)hipFree(f->val);
    delete f;
    return FSCNN_OK;
}

int fscnn_sf_variant_count(void) { return sf_variant_count(); }
const char *fscnn_sf_variant_name(int variant) { return sf_variant_name(variant); }

fscnn_status_t fscnn_sf_variant_choice(const fscnn_filter_t *f, int N, int H, int W, int sh, int sw,
                                       int n4, int pool, int *variant_out)
{
    if (!f || !variant_out) return FSCNN_ERR_NULL;
    if (!live(f)) return FSCNN_ERR_HANDLE;
    if (N <= 0 || H <= 0 || W <= 0 || sh <= 0 || sw <= 0) return FSCNN_ERR_SHAPE;
    return resolve_variant(f, N, H, W, sh, sw, 0, variant_out, n4 != 0, pool != 0);
}

fscnn_status_t fscnn_sf_band_choice(int variant, int N, int Ho, int n4, int pool, int *bands_out,
                                    int *band_rows_out)
{
    if (!bands_out || !band_rows_out) return FSCNN_ERR_NULL;
    if (N <= 0 || Ho <= 0) return FSCNN_ERR_SHAPE;
    if (variant < 1 || variant > sf_variant_count()) return FSCNN_ERR_UNSUPPORTED;
    int shift;
    sf_choose_bands(variant, N, Ho, n4 != 0, pool != 0, &shift, band_rows_out);
    *bands_out = 1 << shift;
    return FSCNN_OK;
}

// emit_cnt / counted: sparse output emission.  When the launch that serves the call can count the
// non-zero results per (pixel, step of 8 channels) in its epilogue it writes them to emit_cnt and
// sets *counted; otherwise the caller counts in a pass of its own.
static fscnn_status_t conv_sf_common(fscnn_filter_t *f, const float *x_dev, int N, int C, int H,
                                     int W, int sh, int sw, int ph, int pw, const float *bias_dev,
                                     int relu, float *y_dev, fscnn_layout_t x_layout,
                                     fscnn_layout_t y_layout, int variant, int pool, void *stream,
                                     int *emit_cnt = nullptr, bool *counted = nullptr)
{
    if (counted) *counted = false;
    int Ho, Wo;
    fscnn_status_t s = check_conv_args(f, x_dev, N, C, H, W, sh, sw, ph, pw, y_dev, &Ho, &Wo);
    if (s != FSCNN_OK) return s;
    if ((x_layout != FSCNN_LAYOUT_NCHW && x_layout != FSCNN_LAYOUT_N4) ||
        (y_layout != FSCNN_LAYOUT_NCHW && y_layout != FSCNN_LAYOUT_N4))
        return FSCNN_ERR_UNSUPPORTED;
    const int in4 = x_layout == FSCNN_LAYOUT_N4, out4 = y_layout == FSCNN_LAYOUT_N4;
    if ((in4 && ((uintptr_t)x_dev & 15)) || (out4 && ((uintptr_t)y_dev & 15))) return FSCNN_ERR_UNSUPPORTED;
    // (a group of four interleaved images is indexed with ints, the groups with 64-bit offsets)
    if ((in4 && !fits_int(4LL * C * H * W)) || (out4 && !fits_int(4LL * f->K * Ho * Wo)))
        return FSCNN_ERR_UNSUPPORTED;
    if (pool && (Ho < 2 || Wo < 2)) return FSCNN_ERR_SHAPE;   // empty pooled output
    int v;
    s = resolve_variant(f, N, H, W, sh, sw, variant, &v, in4 || out4, pool != 0);
    if (s != FSCNN_OK) return s;
    if ((in4 || out4 || pool) && v < 0) return FSCNN_ERR_UNSUPPORTED;   // the direct kernel: NCHW, no pool
    if (v > 0 && !sf_variant_has_layout(v, in4, out4, pool)) return FSCNN_ERR_UNSUPPORTED;
    int dev;
    s = have_device(&dev);
    if (s != FSCNN_OK) return s;
    if (dev != f->device) return FSCNN_ERR_MISMATCH;   // the handle's buffers live on another GPU
    hipStream_t st = (hipStream_t)stream;
    SfPlan *p;
    s = get_plan(f, v, st, &p);
    if (s != FSCNN_OK) return s;
    if (p->direct) {
        FSCNN_HIP(launch_conv_sf_direct(f->rowptr, f->idx, f->val, x_dev, N, C, H, W, f->K, f->R,
                                        f->S, Ho, Wo, sh, sw, ph, pw, bias_dev, relu, y_dev, st));
    } else {
        // automatic choice only: an explicitly selected configuration runs as it is
        int band_shift, band_h;
        sf_choose_bands(v, N, Ho, in4 || out4, pool != 0, &band_shift, &band_h);
        const int csplit = variant == 0 ? sf_choose_csplit(v, N << band_shift, f->K, band_h, Wo, p->NCH) : 1;
        float *parts = nullptr;
        if (csplit > 1) {
            s = split_scratch(f, p, st, sizeof(float) * (size_t)csplit * (size_t)sf_split_elems(N, f->K, Ho, Wo, out4),
                              &parts);
            if (s != FSCNN_OK) return s;
        }
        int *cnt = (emit_cnt && csplit == 1 && !out4 && !pool) ? emit_cnt : nullptr;
        FSCNN_HIP(launch_conv_sf_tiled(*p, x_dev, N, C, H, W, f->K, Ho, Wo, ph, pw, bias_dev, relu,
                                       y_dev, in4, out4, pool, csplit, parts, cnt, band_shift, band_h, st));
        if (counted) *counted = cnt != nullptr;
    }
    return FSCNN_OK;
}

fscnn_status_t fscnn_conv2d_sparse_filter_ex(fscnn_filter_t *f, const float *x_dev, int N, int C,
                                             int H, int W, int sh, int sw, int ph, int pw,
                                             const float *bias_dev, int relu, float *y_dev,
                                             fscnn_layout_t x_layout, fscnn_layout_t y_layout,
                                             int variant, void *stream)
{
    return conv_sf_common(f, x_dev, N, C, H, W, sh, sw, ph, pw, bias_dev, relu, y_dev, x_layout,
                          y_layout, variant, 0, stream);
}

fscnn_status_t fscnn_conv2d_sparse_filter_leaky(fscnn_filter_t *f, const float *x_dev, int N, int C,
                                                int H, int W, int sh, int sw, int ph, int pw,
                                                const float *bias_dev, float negative_slope,
                                                float *y_dev, fscnn_layout_t x_layout,
                                                fscnn_layout_t y_layout, int variant, void *stream)
{
    if (!(negative_slope >= 0.0f && negative_slope <= 1.0f)) return FSCNN_ERR_SHAPE;   // also rejects NaN
    return conv_sf_common(f, x_dev, N, C, H, W, sh, sw, ph, pw, bias_dev, act_code(negative_slope),
                          y_dev, x_layout, y_layout, variant, 0, stream);
}

fscnn_status_t fscnn_conv2d_sparse_filter_pool2x2(fscnn_filter_t *f, const float *x_dev, int N,
                                                  int C, int H, int W, int sh, int sw, int ph,
                                                  int pw, const float *bias_dev, int relu,
                                                  float *y_dev, fscnn_layout_t x_layout,
                                                  fscnn_layout_t y_layout, int variant,
                                                  void *stream)
{
    return conv_sf_common(f, x_dev, N, C, H, W, sh, sw, ph, pw, bias_dev, relu, y_dev, x_layout,
                          y_layout, variant, 1, stream);
}

fscnn_status_t fscnn_conv2d_sparse_filter_v(fscnn_filter_t *f, const float *x_dev, int N, int C,
                                            int H, int W, int sh, int sw, int ph, int pw,
                                            const float *bias_dev, int relu, float *y_dev,
                                            int variant, void *stream)
{
    return fscnn_conv2d_sparse_filter_ex(f, x_dev, N, C, H, W, sh, sw, ph, pw, bias_dev, relu, y_dev,
                                         FSCNN_LAYOUT_NCHW, FSCNN_LAYOUT_NCHW, variant, stream);
}

fscnn_status_t fscnn_layout_convert(const float *src_dev, int N, int C, int H, int W,
                                    fscnn_layout_t src_layout, float *dst_dev,
                                    fscnn_layout_t dst_layout, void *stream)
{
    if (!src_dev || !dst_dev) return FSCNN_ERR_NULL;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return FSCNN_ERR_SHAPE;
    const bool s4 = src_layout == FSCNN_LAYOUT_N4, d4 = dst_layout == FSCNN_LAYOUT_N4;
    if ((!s4 && src_layout != FSCNN_LAYOUT_NCHW) || (!d4 && dst_layout != FSCNN_LAYOUT_NCHW) ||
        s4 == d4 || src_dev == dst_dev)
        return FSCNN_ERR_UNSUPPORTED;
    if (!fits_int(((long long)N + 3) / 4 * 4 * C * H * W)) return FSCNN_ERR_UNSUPPORTED;
    if ((uintptr_t)(s4 ? src_dev : dst_dev) & 15) return FSCNN_ERR_UNSUPPORTED;
    int dev;
    fscnn_status_t s = have_device(&dev);
    if (s != FSCNN_OK) return s;
    FSCNN_HIP(launch_layout_convert(src_dev, N, C, H, W, s4 ? 1 : 0, dst_dev, (hipStream_t)stream));
    return FSCNN_OK;
}

fscnn_status_t fscnn_conv2d_sparse_filter(fscnn_filter_t *f, const float *x_dev, int N, int C, int H,
                                          int W, int sh, int sw, int ph, int pw,
                                          const float *bias_dev, int relu, float *y_dev,
                                          void *stream)
{
    return fscnn_conv2d_sparse_filter_v(f, x_dev, N, C, H, W, sh, sw, ph, pw, bias_dev, relu, y_dev,
                                        0, stream);
}

// Dense N x C x H x W activations -> compressed handle.  Synchronises st once (the number of
// stored values sizes the second buffer); the pass that fills the handle is still running on st
// when this returns, and reads x.
static fscnn_status_t compress_activations(const float *x_dev, int N, int C, int H, int W,
                                           hipStream_t st, fscnn_input_t **out)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return FSCNN_ERR_SHAPE;
    const long long npix = (long long)N * H * W;
    if (!fits_int(npix + 1) || !fits_int(npix * C)) return FSCNN_ERR_SHAPE;
    const int CC = kSiCC, NCH = (C + CC - 1) / CC;
    // the packing pass keeps a pixel's whole list in LDS: up to 8192 channels
    if (!fits_int(npix * NCH + 1) || NCH > 8192 / kSiCC) return FSCNN_ERR_UNSUPPORTED;
    int dev;
    fscnn_status_t s = have_device(&dev);
    if (s != FSCNN_OK) return s;
    fscnn_input_t *in = new (std::nothrow) fscnn_input();
    if (!in) return FSCNN_ERR_ALLOC;
    in->magic = kInputMagic;
    in->device = dev;
    in->N = N; in->C = C; in->H = H; in->W = W;
    in->nnz = 0; in->CC = CC; in->NCH = NCH;
    in->cidx = nullptr; in->xval = nullptr; in->cptr = nullptr;
    in->ptr_block = nullptr; in->node_block = nullptr;
    in->made_on = st; in->filled = nullptr;
    int total = 0;
    const long long nstep = npix * NCH;   // (pixel, channel step) pairs
    // first allocation: the pointer array, then (256-byte aligned) the counts it is scanned from
    // and the scan's scratch; the counts stay with the handle, so nothing is freed here
    const size_t cnt_at = ((size_t)(nstep + 1) * sizeof(int) + 255) / 256 * 256;
    hipError_t e = hipMalloc(&in->ptr_block, cnt_at + sizeof(int) * (size_t)(nstep + scan_tmp_elems(nstep)));
    if (e == hipSuccess) {
        in->cptr = static_cast<int *>(in->ptr_block);
        int *cnt = reinterpret_cast<int *>(static_cast<char *>(in->ptr_block) + cnt_at);
        e = launch_input_count(x_dev, N, C, H, W, CC, NCH, cnt, st);
        if (e == hipSuccess) e = launch_exclusive_scan(cnt, in->cptr, nstep, cnt + nstep, st);
    }
    if (e == hipSuccess)
        e = hipMemcpyAsync(&total, in->cptr + nstep, sizeof(int), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e == hipSuccess) {
        in->nnz = total;
        // second allocation: indices, then (256-byte aligned) values.  Spare entries: the
        // sparse-input kernels fetch the next (channel, value) pairs of a pixel's list ahead, up
        // to kSiSpare positions past the one in use
        const size_t n = (size_t)total + kSiSpare;
        const size_t val_at = (n * sizeof(uint32_t) + 255) / 256 * 256;
        e = hipMalloc(&in->node_block, val_at + n * sizeof(float));
        if (e == hipSuccess) {
            in->cidx = static_cast<uint32_t *>(in->node_block);
            in->xval = reinterpret_cast<float *>(static_cast<char *>(in->node_block) + val_at);
            e = launch_input_fill(x_dev, N, C, H, W, CC, NCH, in->cptr, in->cidx, in->xval, kSiSpare, st);
        }
    }
    if (e == hipSuccess) e = hipEventCreateWithFlags(&in->filled, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventRecord(in->filled, st);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        (void)hipStreamSynchronize(st);   // nothing may still write into what is freed next
        if (in->filled) (void)hipEventDestroy(in->filled);
        if (in->ptr_block) (void)hipFree(in->ptr_block);
        if (in->node_block) (void)hipFree(in->node_block);
        in->magic = 0;
        delete in;
        return e == hipErrorOutOfMemory ? FSCNN_ERR_ALLOC : FSCNN_ERR_DEVICE;
    }
    *out = in;
    return FSCNN_OK;
}

fscnn_status_t fscnn_input_compress(const float *x_dev, int N, int C, int H, int W, void *stream,
                                    fscnn_input_t **out)
{
    if (!x_dev || !out) return FSCNN_ERR_NULL;
    return compress_activations(x_dev, N, C, H, W, (hipStream_t)stream, out);
}

namespace {

// Where the parts of an emitted handle's one allocation start (256-byte aligned parts): pointer
// array | counts + scan scratch | indices | values | the dense result when the caller takes none.
struct EmitLayout {
    long long nstep, dense;
    size_t cnt_at, idx_at, val_at, y_at;
    size_t bytes(bool with_y) const { return y_at + (with_y ? sizeof(float) * (size_t)dense : 0); }
};

EmitLayout emit_layout(long long npix, int K, int NCH)
{
    EmitLayout L;
    L.nstep = npix * NCH;
    L.dense = npix * K;
    auto up = [](size_t v) { return (v + 255) / 256 * 256; };
    L.cnt_at = up((size_t)(L.nstep + 1) * sizeof(int));
    L.idx_at = L.cnt_at + up(sizeof(int) * (size_t)(L.nstep + scan_tmp_elems(L.nstep)));
    L.val_at = L.idx_at + up(sizeof(uint32_t) * (size_t)(L.dense + kSiSpare));
    L.y_at = L.val_at + up(sizeof(float) * (size_t)(L.dense + kSiSpare));
    return L;
}

// Argument checks shared by the two emitting calls; fills the result's shape.
fscnn_status_t emit_check(fscnn_filter_t *f, int N, int C, int H, int W, int sh, int sw, int ph,
                          int pw, int *Ho, int *Wo, int *NCH)
{
    if (!live(f)) return FSCNN_ERR_HANDLE;
    if (N <= 0 || C <= 0) return FSCNN_ERR_SHAPE;
    fscnn_status_t s = out_shape(H, W, f->R, f->S, sh, sw, ph, pw, Ho, Wo);
    if (s != FSCNN_OK) return s;
    const long long npix = (long long)N * *Ho * *Wo, dense = npix * f->K;
    if (!fits_int(dense) || !fits_int(dense + kSiSpare)) return FSCNN_ERR_UNSUPPORTED;
    *NCH = (f->K + kSiCC - 1) / kSiCC;
    if (!fits_int(npix * *NCH + 1) || *NCH > 8192 / kSiCC) return FSCNN_ERR_UNSUPPORTED;
    return FSCNN_OK;
}

// The work of an emitting call on a handle whose allocation is in place: the convolution with its
// bias / activation epilogue (which, where the launch can, counts the non-zero results per pixel
// and step of 8 channels itself), else a count pass, one scan, one pass that writes the pairs.
fscnn_status_t emit_run(fscnn_filter_t *f, const float *x_dev, int N, int C, int H, int W, int sh,
                        int sw, int ph, int pw, const float *bias_dev, int relu, float *y_dev,
                        void *stream, fscnn_input_t *in)
{
    hipStream_t st = (hipStream_t)stream;
    const int K = f->K, Ho = in->H, Wo = in->W;
    const EmitLayout L = emit_layout((long long)N * Ho * Wo, K, in->NCH);
    char *base = static_cast<char *>(in->ptr_block);
    int *cnt = reinterpret_cast<int *>(base + L.cnt_at);
    float *y = y_dev ? y_dev : reinterpret_cast<float *>(base + L.y_at);
    bool counted = false;
    fscnn_status_t s = conv_sf_common(f, x_dev, N, C, H, W, sh, sw, ph, pw, bias_dev, relu, y,
                                      FSCNN_LAYOUT_NCHW, FSCNN_LAYOUT_NCHW, 0, 0, stream, cnt, &counted);
    if (s != FSCNN_OK) return s;
    hipError_t e = hipSuccess;
    if (!counted) e = launch_input_count(y, N, K, Ho, Wo, in->CC, in->NCH, cnt, st);
    if (e == hipSuccess) e = launch_exclusive_scan(cnt, in->cptr, L.nstep, cnt + L.nstep, st);
    if (e == hipSuccess)
        e = launch_input_fill(y, N, K, Ho, Wo, in->CC, in->NCH, in->cptr, in->cidx, in->xval, kSiSpare, st);
    if (e == hipSuccess) e = hipEventRecord(in->filled, st);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return e == hipErrorOutOfMemory ? FSCNN_ERR_ALLOC : FSCNN_ERR_DEVICE;
    }
    in->nnz = -1;
    in->made_on = st;
    return FSCNN_OK;
}

}  // namespace

fscnn_status_t fscnn_conv2d_sparse_filter_emit(fscnn_filter_t *f, const float *x_dev, int N, int C,
                                               int H, int W, int sh, int sw, int ph, int pw,
                                               const float *bias_dev, int relu, float *y_dev,
                                               void *stream, fscnn_input_t **out)
{
    if (!f || !x_dev || !out) return FSCNN_ERR_NULL;
    int Ho, Wo, NCH;
    fscnn_status_t s = emit_check(f, N, C, H, W, sh, sw, ph, pw, &Ho, &Wo, &NCH);
    if (s != FSCNN_OK) return s;
    int dev;
    s = have_device(&dev);
    if (s != FSCNN_OK) return s;
    fscnn_input_t *in = new (std::nothrow) fscnn_input();
    if (!in) return FSCNN_ERR_ALLOC;
    in->magic = kInputMagic;
    in->device = dev;
    in->N = N; in->C = f->K; in->H = Ho; in->W = Wo;
    in->nnz = -1; in->CC = kSiCC; in->NCH = NCH;
    in->ptr_block = nullptr; in->node_block = nullptr;
    in->made_on = (hipStream_t)stream; in->filled = nullptr;
    // ONE allocation, sized for the worst case (every result non-zero), so that nothing here waits
    // for the device
    const EmitLayout L = emit_layout((long long)N * Ho * Wo, f->K, NCH);
    in->emit_bytes = L.bytes(y_dev == nullptr);
    in->emit_has_y = y_dev == nullptr;
    hipError_t e = hipMalloc(&in->ptr_block, in->emit_bytes);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&in->filled, hipEventDisableTiming);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        if (in->ptr_block) (void)hipFree(in->ptr_block);
        delete in;
        return FSCNN_ERR_ALLOC;
    }
    char *base = static_cast<char *>(in->ptr_block);
    in->cptr = reinterpret_cast<int *>(base);
    in->cidx = reinterpret_cast<uint32_t *>(base + L.idx_at);
    in->xval = reinterpret_cast<float *>(base + L.val_at);
    s = emit_run(f, x_dev, N, C, H, W, sh, sw, ph, pw, bias_dev, relu, y_dev, stream, in);
    if (s != FSCNN_OK) {
        (void)hipStreamSynchronize((hipStream_t)stream);   // nothing may still write into what is freed next
        (void)hipEventDestroy(in->filled);
        (void)hipFree(in->ptr_block);
        in->magic = 0;
        delete in;
        return s;
    }
    *out = in;
    return FSCNN_OK;
}

fscnn_status_t fscnn_conv2d_sparse_filter_emit_into(fscnn_filter_t *f, const float *x_dev, int N,
                                                    int C, int H, int W, int sh, int sw, int ph,
                                                    int pw, const float *bias_dev, int relu,
                                                    float *y_dev, void *stream, fscnn_input_t *into)
{
    if (!f || !x_dev || !into) return FSCNN_ERR_NULL;
    if (!live(into)) return FSCNN_ERR_HANDLE;
    int Ho, Wo, NCH;
    fscnn_status_t s = emit_check(f, N, C, H, W, sh, sw, ph, pw, &Ho, &Wo, &NCH);
    if (s != FSCNN_OK) return s;
    int dev;
    s = have_device(&dev);
    if (s != FSCNN_OK) return s;
    if (into->device != dev) return FSCNN_ERR_MISMATCH;
    // only a handle that an emitting call made, for a result of this very shape, has the room
    if (into->emit_bytes == 0) return FSCNN_ERR_UNSUPPORTED;
    if (into->N != N || into->C != f->K || into->H != Ho || into->W != Wo) return FSCNN_ERR_MISMATCH;
    if (!y_dev && !into->emit_has_y) return FSCNN_ERR_NULL;
    return emit_run(f, x_dev, N, C, H, W, sh, sw, ph, pw, bias_dev, relu, y_dev, stream, into);
}

fscnn_status_t fscnn_input_info(const fscnn_input_t *in, int *N, int *C, int *H, int *W,
                                long long *nnz)
{
    if (!in) return FSCNN_ERR_NULL;
    if (!live(in)) return FSCNN_ERR_HANDLE;
    if (N) *N = in->N;
    if (C) *C = in->C;
    if (H) *H = in->H;
    if (W) *W = in->W;
    if (nnz) {
        *nnz = input_nnz(in);
        if (*nnz < 0) return FSCNN_ERR_DEVICE;
    }
    return FSCNN_OK;
}

fscnn_status_t fscnn_input_export(const fscnn_input_t *in, int *prow_host, unsigned *cidx_host,
                                  float *val_host)
{
    if (!in || !prow_host) return FSCNN_ERR_NULL;
    if (!live(in)) return FSCNN_ERR_HANDLE;
    const long long stored = input_nnz(in);
    if (stored < 0) return FSCNN_ERR_DEVICE;
    if (stored > 0 && (!cidx_host || !val_host)) return FSCNN_ERR_NULL;
    FSCNN_HIP(hipEventSynchronize(in->filled));
    // the row pointers are every NCH-th chunk pointer
    const size_t npix = (size_t)in->N * in->H * in->W;
    FSCNN_HIP(hipMemcpy2D(prow_host, sizeof(int), in->cptr, sizeof(int) * (size_t)in->NCH, sizeof(int), npix,
                          hipMemcpyDeviceToHost));
    FSCNN_HIP(hipMemcpy(prow_host + npix, in->cptr + npix * (size_t)in->NCH, sizeof(int), hipMemcpyDeviceToHost));
    if (stored > 0) {
        FSCNN_HIP(hipMemcpy(cidx_host, in->cidx, sizeof(uint32_t) * (size_t)stored, hipMemcpyDeviceToHost));
        FSCNN_HIP(hipMemcpy(val_host, in->xval, sizeof(float) * (size_t)stored, hipMemcpyDeviceToHost));
    }
    return FSCNN_OK;
}

fscnn_status_t fscnn_input_destroy(fscnn_input_t *in)
{
    if (!in) return FSCNN_ERR_NULL;
    if (!live(in)) return FSCNN_ERR_HANDLE;
    in->magic = 0;
    (void)hipEventSynchronize(in->filled);
    (void)hipEventDestroy(in->filled);
    if (in->ptr_block) (void)hipFree(in->ptr_block);
    if (in->node_block) (void)hipFree(in->node_block);
    delete in;
    return FSCNN_OK;
}

fscnn_status_t fscnn_conv2d_sparse_input(const fscnn_input_t *in, const float *w_dev, int K, int R,
                                         int S, int sh, int sw, int ph, int pw,
                                         const float *bias_dev, int relu, float *y_dev, void *stream)
{
    if (!in || !w_dev || !y_dev) return FSCNN_ERR_NULL;
    if (!live(in)) return FSCNN_ERR_HANDLE;
    if (K <= 0) return FSCNN_ERR_SHAPE;
    int Ho, Wo;
    fscnn_status_t s = out_shape(in->H, in->W, R, S, sh, sw, ph, pw, &Ho, &Wo);
    if (s != FSCNN_OK) return s;
    if (!fits_int((long long)K * in->C * R * S) || !fits_int((long long)in->N * K * Ho * Wo))
        return FSCNN_ERR_UNSUPPORTED;
    int dev;
    s = have_device(&dev);
    if (s != FSCNN_OK) return s;
    if (dev != in->device) return FSCNN_ERR_MISMATCH;
    FSCNN_HIP(after_fill(in, (hipStream_t)stream));
    FSCNN_HIP(launch_conv_si(in, w_dev, K, R, S, Ho, Wo, sh, sw, ph, pw, bias_dev, relu, y_dev,
                             (hipStream_t)stream));
    return FSCNN_OK;
}

fscnn_status_t fscnn_dense_filter_prepare(const float *w_dev, int K, int C, int R, int S, void *stream,
                                          fscnn_dense_t **out)
{
    if (!w_dev || !out) return FSCNN_ERR_NULL;
    if (K <= 0 || C <= 0 || R <= 0 || S <= 0) return FSCNN_ERR_SHAPE;
    const int Kpad = (K + 255) / 256 * 256;
    if (!fits_int((long long)K * C * R * S) || !fits_int((long long)Kpad * C * R * S)) return FSCNN_ERR_SHAPE;
    int dev;
    fscnn_status_t s = have_device(&dev);
    if (s != FSCNN_OK) return s;
    fscnn_dense_t *d = new (std::nothrow) fscnn_dense();
    if (!d) return FSCNN_ERR_ALLOC;
    d->magic = kDenseMagic;
    d->device = dev;
    d->K = K; d->C = C; d->R = R; d->S = S; d->Kpad = Kpad;
    d->wT = nullptr;
    hipError_t e = hipMalloc(&d->wT, sizeof(float) * (size_t)Kpad * C * R * S);
    if (e == hipSuccess) e = launch_dense_transpose(w_dev, K, C, R * S, Kpad, d->wT, (hipStream_t)stream);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        if (d->wT) (void)hipFree(d->wT);
        d->magic = 0;
        delete d;
        return e == hipErrorOutOfMemory ? FSCNN_ERR_ALLOC : FSCNN_ERR_DEVICE;
    }
    *out = d;
    return FSCNN_OK;
}

fscnn_status_t fscnn_dense_filter_destroy(fscnn_dense_t *d)
{
    if (!d) return FSCNN_ERR_NULL;
    if (!live(d)) return FSCNN_ERR_HANDLE;
    d->magic = 0;
    if (d->wT) (void)hipFree(d->wT);
    delete d;
    return FSCNN_OK;
}

int fscnn_si_variant_count(void) { return si_variant_count(); }

fscnn_status_t fscnn_conv2d_sparse_input_prepared(const fscnn_input_t *in, const fscnn_dense_t *d,
                                                  int sh, int sw, int ph, int pw,
                                                  const float *bias_dev, int relu, float *y_dev,
                                                  int variant, void *stream)
{
    if (!in || !d || !y_dev) return FSCNN_ERR_NULL;
    if (!live(in) || !live(d)) return FSCNN_ERR_HANDLE;
    if (d->C != in->C) return FSCNN_ERR_MISMATCH;
    int Ho, Wo;
    fscnn_status_t s = out_shape(in->H, in->W, d->R, d->S, sh, sw, ph, pw, &Ho, &Wo);
    if (s != FSCNN_OK) return s;
    if (variant < 0 || variant > si_variant_count()) return FSCNN_ERR_UNSUPPORTED;
    // the prepared form serves 3x3 / stride 1; other geometries take fscnn_conv2d_sparse_input
    if (d->R != 3 || d->S != 3 || sh != 1 || sw != 1) return FSCNN_ERR_UNSUPPORTED;
    if (!fits_int((long long)in->N * d->K * Ho * Wo)) return FSCNN_ERR_UNSUPPORTED;
    int dev;
    s = have_device(&dev);
    if (s != FSCNN_OK) return s;
    if (dev != in->device || dev != d->device) return FSCNN_ERR_MISMATCH;
    FSCNN_HIP(after_fill(in, (hipStream_t)stream));
    FSCNN_HIP(launch_conv_si_prepared(in, d, Ho, Wo, ph, pw, bias_dev, relu, y_dev, variant,
                                      (hipStream_t)stream));
    return FSCNN_OK;
}

long long fscnn_sparse_transpose_workspace(long long new_rows, long long nnz)
{
    return reorder_workspace_bytes(new_rows, nnz);
}

static fscnn_status_t reorder_common(bool tensor, const int *rowptr, const unsigned *idx,
                                     const float *val, int n_rows, int n_cols, int H,
                                     long long n_buckets, long long nnz, int *tptr,
                                     unsigned *tidx, float *tval, void *ws, long long ws_bytes,
                                     void *stream)
{
    if (!rowptr || !tptr || !ws) return FSCNN_ERR_NULL;
    if (nnz < 0 || nnz >= (1LL << 31)) return FSCNN_ERR_SHAPE;
    if (nnz > 0 && (!idx || !val || !tidx || !tval)) return FSCNN_ERR_NULL;
    if (!fits_int(n_buckets + 1)) return FSCNN_ERR_UNSUPPORTED;
    const long long need = reorder_workspace_bytes(n_buckets, nnz);
    if (need < 0 || ws_bytes < need || ((uintptr_t)ws & 3)) return FSCNN_ERR_UNSUPPORTED;
    int dev;
    fscnn_status_t s = have_device(&dev);
    if (s != FSCNN_OK) return s;
    FSCNN_HIP(launch_reorder(tensor, rowptr, idx, val, n_rows, n_cols, H, n_buckets, nnz, tptr, tidx,
                             tval, ws, (hipStream_t)stream));
    return FSCNN_OK;
}

fscnn_status_t fscnn_sparse_transpose(const int *rowptr_dev, const unsigned *idx_dev,
                                      const float *val_dev, int n_rows, int n_cols, long long nnz,
                                      int *tptr_dev, unsigned *tidx_dev, float *tval_dev,
                                      void *workspace_dev, long long workspace_bytes, void *stream)
{
    if (n_rows <= 0 || n_cols <= 0) return FSCNN_ERR_SHAPE;
    return reorder_common(false, rowptr_dev, idx_dev, val_dev, n_rows, n_cols, 1, n_cols, nnz,
                          tptr_dev, tidx_dev, tval_dev, workspace_dev, workspace_bytes, stream);
}

fscnn_status_t fscnn_sparse_transpose_noalloc(const int *rowptr_dev, const unsigned *idx_dev,
                                              const float *val_dev, int n_rows, int n_cols,
                                              long long nnz, int *tptr_dev, unsigned *tidx_dev,
                                              float *tval_dev, void *stream)
{
    if (n_rows <= 0 || n_cols <= 0) return FSCNN_ERR_SHAPE;
    if (!rowptr_dev || !tptr_dev) return FSCNN_ERR_NULL;
    if (nnz < 0 || nnz >= (1LL << 31)) return FSCNN_ERR_SHAPE;
    const long long need = reorder_workspace_bytes(n_cols, nnz);
    if (need < 0 || need > kStaticScratchBytes) return FSCNN_ERR_UNSUPPORTED;   // beyond the static scratch
    int dev;
    fscnn_status_t s = have_device(&dev);
    if (s != FSCNN_OK) return s;
    void *ws = nullptr;
    FSCNN_HIP(static_scratch(&ws));
    return reorder_common(false, rowptr_dev, idx_dev, val_dev, n_rows, n_cols, 1, n_cols, nnz, tptr_dev,
                          tidx_dev, tval_dev, ws, kStaticScratchBytes, stream);
}

fscnn_status_t fscnn_sparse_tensor_transpose(const int *rowptr_dev, const unsigned *widx_dev,
                                             const float *val_dev, int W, int H, int C,
                                             long long nnz, int *tptr_dev, unsigned *cidx_dev,
                                             float *tval_dev, void *workspace_dev,
                                             long long workspace_bytes, void *stream)
{
    if (W <= 0 || H <= 0 || C <= 0) return FSCNN_ERR_SHAPE;
    if (!fits_int((long long)C * H + 1) || !fits_int((long long)W * H + 1)) return FSCNN_ERR_SHAPE;
    return reorder_common(true, rowptr_dev, widx_dev, val_dev, C * H, W, H, (long long)W * H, nnz,
                          tptr_dev, cidx_dev, tval_dev, workspace_dev, workspace_bytes, stream);
}

fscnn_status_t fscnn_maxpool2x2_ex(const float *x_dev, int N, int C, int H, int W, float *y_dev,
                                   fscnn_layout_t layout, void *stream)
{
    if (!x_dev || !y_dev) return FSCNN_ERR_NULL;
    if (N <= 0 || C <= 0 || H < 2 || W < 2) return FSCNN_ERR_SHAPE;
    if (layout != FSCNN_LAYOUT_NCHW && layout != FSCNN_LAYOUT_N4) return FSCNN_ERR_UNSUPPORTED;
    const int n4 = layout == FSCNN_LAYOUT_N4;
    if (!fits_int(((long long)N + 3) / 4 * 4 * C * H * W)) return FSCNN_ERR_UNSUPPORTED;
    if (n4 && (((uintptr_t)x_dev | (uintptr_t)y_dev) & 15)) return FSCNN_ERR_UNSUPPORTED;
    int dev;
    fscnn_status_t s = have_device(&dev);
    if (s != FSCNN_OK) return s;
    FSCNN_HIP(launch_maxpool2x2(x_dev, N, C, H, W, y_dev, n4, (hipStream_t)stream));
    return FSCNN_OK;
}

fscnn_status_t fscnn_maxpool2x2(const float *x_dev, int N, int C, int H, int W, float *y_dev,
                                void *stream)
{
    return fscnn_maxpool2x2_ex(x_dev, N, C, H, W, y_dev, FSCNN_LAYOUT_NCHW, stream);
}

}  // extern "C"
