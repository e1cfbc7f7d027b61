// Internal declarations shared by the translation units of libfscnn.so.
// Nothing here is part of the C ABI (see include/fscnn.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>
#include <vector>

#include "fscnn.h"

namespace fscnn {

constexpr uint64_t kFilterMagic = 0x4653434e4e464c54ull;  // "FSCNNFLT"
constexpr uint64_t kInputMagic = 0x4653434e4e494e50ull;   // "FSCNNINP"
constexpr uint64_t kDenseMagic = 0x4653434e4e44454eull;   // "FSCNNDEN"

// One nonzero as the convolution kernel streams it: the byte offset of the tap
// (c mod CC, r, s) inside the LDS input tile, and the weight (the paper's node
// {index, value}, Sec. 3, with the index pre-multiplied for the tile geometry).
struct Rec {
    uint32_t off;
    float val;
};

// Geometry of one kernel configuration of the tiled sparse-filter convolution.
struct SfGeom {
    int BV, LW, LHR, NV, SLOTS, WAVES, CC;  // template parameters
    int R, S;                               // filter extent the instance is built for
    int TH, TW, IMGS;                       // output tile and images per work-group
    int IN_ROWS, PITCH;                     // LDS rows per channel, BV-vectors per row
    int KG;                                 // output channels per work-group
    int STRIDE;                             // stride (both axes) the instance is built for
    int DENSE;                              // 1: the plan lists every tap of every chunk, SLOTS weights per tap
    int lds_bytes;
};

// Activation code carried by the kernels' `relu` argument: 0 = none, 1 = ReLU, anything else =
// the bit pattern of a LeakyReLU slope (y > 0 ? y : slope * y).  A slope whose bits are 0 or 1
// (0.0f, the smallest denormal) is ReLU to rounding and is mapped to 1 by act_code().
__host__ __device__ inline float act_apply(float r, int act)
{
    // none / ReLU first (the common cases: one compare-and-select); the LeakyReLU fix-up sits
    // behind a branch on the wave-uniform code so that the other two do not pay for it
    float y = act == 1 ? (r > 0.0f ? r : 0.0f) : r;
    if (__builtin_expect((act & ~1) != 0, 0)) {
        union { int i; float f; } u;
        u.i = act;
        y = r > 0.0f ? r : r * u.f;
    }
    return y;
}
inline int act_code(float negative_slope)
{
    union { int i; float f; } u;
    u.f = negative_slope;
    return (u.i == 0 || u.i == 1) ? 1 : u.i;
}

constexpr int kPlanSpare = 12;  // zero records appended to a plan's stream (reader prefetch)

struct SfPlan {
    int variant = 0;   // 1-based index into the variant table
    bool direct = false;
    SfGeom g{};
    int NCH = 0, NG = 0;
    long long nrec = 0;       // records (= nonzeros); the array carries kPlanSpare spare entries
    int *segptr = nullptr;    // [NG*NCH*KG + 1], bucket order (group, wave, chunk, slot)
    Rec *recs = nullptr;      // [nrec + kPlanSpare]
    // Scratch of the channel-split mode (small problems): one buffer per stream that has used the
    // plan in that mode, so that calls on different streams never share one.  Grown on demand.
    struct SplitScratch {
        hipStream_t stream;
        float *buf;
        size_t bytes;
    };
    std::vector<SplitScratch> split;
};

struct SiGeom {
    int CC;  // channels per chunk of the compressed activation's chunk pointers
};
hipError_t launch_dense_transpose(const float *w, int K, int C, int RS, int Kpad, float *wT,
                                  hipStream_t st);
int si_variant_count();
hipError_t launch_conv_si_prepared(const fscnn_input *in, const fscnn_dense *d, int Ho, int Wo, int ph,
                                   int pw, const float *bias, int relu, float *y, int variant,
                                   hipStream_t st);

}  // namespace fscnn

struct fscnn_filter {
    uint64_t magic;
    int device;
    int K, C, R, S;
    long long nnz;
    int *rowptr;    // device [K+1]
    uint32_t *idx;  // device [nnz]
    float *val;     // device [nnz]
    std::mutex mu;
    std::vector<fscnn::SfPlan *> plans;
};

struct fscnn_input {
    uint64_t magic;
    int device;
    int N, C, H, W;
    long long nnz;   // -1: not fetched yet (the handle was filled without a host synchronisation;
                     // input_nnz() waits for `filled` and reads cptr's last element)
    int CC, NCH;     // chunking of the channel axis used by cptr
    uint32_t *cidx;  // device [nnz]
    float *xval;     // device [nnz]
    int *cptr;       // device [N*H*W*NCH + 1]: cptr[p*NCH + j] = first entry of pixel p with
                     // c >= j*CC; pixel p's row is [cptr[p*NCH], cptr[(p+1)*NCH])
    // the two device allocations behind the arrays: pointers (and the counts they were scanned
    // from), then indices and values
    void *ptr_block, *node_block;
    // a handle made by an emitting convolution has ONE allocation (ptr_block) of emit_bytes, sized
    // for the worst case, with room for the dense result iff emit_has_y; 0 for other handles
    size_t emit_bytes = 0;
    bool emit_has_y = false;
    // the pass that fills the handle runs on `made_on` and may still be in flight when the
    // handle is returned; `filled` is recorded behind it, for users on other streams
    hipStream_t made_on;
    hipEvent_t filled;
};

// Dense filter bank prepared for the sparse-input convolution: a K-contiguous copy
// wT[c][r][s][k] (k padded to Kpad with zeros), built once.
struct fscnn_dense {
    uint64_t magic;
    int device;
    int K, C, R, S, Kpad;
    float *wT;       // device [C*R*S*Kpad]
};

namespace fscnn {

// ---- compress.hip
hipError_t launch_filter_count(const float *w, int K, long long row, int *cnt, hipStream_t st);
// out[0..n] = exclusive scan of in[0..n-1] (out[n] = total); tmp: scan_tmp_elems(n) ints of scratch
long long scan_tmp_elems(long long n);
hipError_t launch_exclusive_scan(const int *in, int *out, long long n, int *tmp, hipStream_t st);
hipError_t launch_filter_pack(const float *w, int K, long long row, const int *rowptr,
                              uint32_t *idx, float *val, hipStream_t st);
hipError_t launch_plan_count(const int *rowptr, const uint32_t *idx, int K, int RS, const SfGeom &g,
                             int NCH, int NG, int *cnt, hipStream_t st);
hipError_t launch_plan_fill(const int *rowptr, const uint32_t *idx, const float *val, int K, int R,
                            int S, const SfGeom &g, int NCH, int NG, const int *segptr, Rec *recs,
                            hipStream_t st);
// the taps-outer plan (SfGeom::DENSE): nrec = NG*WAVES*NCH*CC*R*S*SLOTS records plus the spare ones
hipError_t launch_plan_fill_dense(const int *rowptr, const uint32_t *idx, const float *val, int K, int C,
                                  int R, int S, const SfGeom &g, int NCH, int NG, long long nrec, Rec *recs,
                                  hipStream_t st);
hipError_t launch_input_count(const float *x, int N, int C, int H, int W, int CC, int NCH, int *cnt,
                              hipStream_t st);
// also zeroes the `spare` entries that follow the last stored one (cptr's last element says where)
hipError_t launch_input_fill(const float *x, int N, int C, int H, int W, int CC, int NCH,
                             const int *cptr, uint32_t *cidx, float *xval, int spare, hipStream_t st);
hipError_t launch_maxpool2x2(const float *x, int N, int C, int H, int W, float *y, int n4,
                             hipStream_t st);
hipError_t launch_layout_convert(const float *src, int N, int C, int H, int W, int src_n4, float *dst,
                                 hipStream_t st);

// ---- conv_sf.hip
int sf_variant_count();
const char *sf_variant_name(int variant);
// false if the variant cannot serve RxS filters at this stride
bool sf_variant_geom(int variant, int R, int S, int sh, int sw, SfGeom *g);
int sf_choose_variant(int N, int C, int K, int H, int W, int R, int S, int stride, bool pool, bool n4,
                      bool no_zeros = false, bool banded = false);
bool sf_variant_has_layout(int variant, int in4, int out4, int pool);
// csplit > 1: `parts` is scratch of csplit * sf_split_elems(...) floats (one copy of y per part)
long long sf_split_elems(int N, int K, int Ho, int Wo, int out4);
// emit_cnt != nullptr (NCHW output, no pool, csplit == 1 only): the epilogue also stores, per output
// pixel p = (n*Ho + oy)*Wo + ox and step j of 8 output channels, the number of non-zero results into
// emit_cnt[p * ceil(K/8) + j] -- the counts the activation compressor scans
hipError_t launch_conv_sf_tiled(const SfPlan &p, const float *x, int N, int C, int H, int W, int K,
                                int Ho, int Wo, int ph, int pw, const float *bias, int relu,
                                float *y, int in4, int out4, int pool, int csplit, float *parts,
                                int *emit_cnt, int band_shift, int band_h, hipStream_t st);
// band_shift, band_h of a launch: 4 / N bands of band_h output rows per image where a four-image
// configuration serves one or two images through NCHW tensors (then the work-groups of the launch,
// and with them the channel split, go by N << band_shift slots of band_h rows); else 0 and Ho
void sf_choose_bands(int variant, int N, int Ho, bool n4, bool pool, int *band_shift, int *band_h);
// 1, or the number of parts the input-channel range is split into for a small problem
int sf_choose_csplit(int variant, int N, int K, int Ho, int Wo, int NCH);
hipError_t launch_conv_sf_direct(const int *rowptr, const uint32_t *idx, const float *val,
                                 const float *x, int N, int C, int H, int W, int K, int R, int S,
                                 int Ho, int Wo, int sh, int sw, int ph, int pw, const float *bias,
                                 int relu, float *y, hipStream_t st);

// ---- transpose.hip
long long reorder_workspace_bytes(long long n_buckets, long long nnz);  // -1: too large
// Size of the per-GPU static scratch of fscnn_sparse_transpose_noalloc, and its device address on
// the current GPU (looked up once per device).
constexpr long long kStaticScratchBytes = 8LL << 20;
hipError_t static_scratch(void **ptr);
hipError_t launch_reorder(bool tensor, const int *rowptr, const uint32_t *idx, const float *val,
                          int n_rows, int n_cols, int H, long long n_buckets, long long nnz,
                          int *tptr, uint32_t *tidx, float *tval, void *workspace, hipStream_t st);

// ---- conv_si.hip
constexpr int kSiCC = 8;   // channels per step of the compressed activation's chunk pointers
constexpr int kSiSpare = 8;  // entries allocated past the last (channel, value) pair (reader prefetch)
bool si_tiled_supported(int K, int C, int R, int S, int sh, int sw);
hipError_t launch_conv_si(const fscnn_input *in, const float *w, int K, int R, int S, int Ho, int Wo,
                          int sh, int sw, int ph, int pw, const float *bias, int relu, float *y,
                          hipStream_t st);

}  // namespace fscnn
