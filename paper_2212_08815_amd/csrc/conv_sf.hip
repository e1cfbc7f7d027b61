// Sparse-filter convolution kernels (dense NCHW input x compressed filters -> dense NCHW).
//
// What is computed is the direct forward pass of the paper's Alg. 6: every output element
// is the sum, over the stored nonzeros of its filter, of weight * input tap (Alg. 2's
// sparse . dense inner product), without kernel flip, padding realised as an index shift
// into a zero-filled border (Sec. 5, "Other layers").
//
// How it is mapped to gfx950 (ours, not the paper's CPU loops):
//   * output-stationary: a work-group owns a TH x TW output tile of one image and KG output
//     channels; each wave owns SLOTS of those channels and keeps P = VW*NV vertically
//     adjacent outputs per lane in fp32 registers, lanes running along x (LW lanes per row)
//     so that global loads and stores are coalesced;
//   * the input channels are walked in chunks of CC: the chunk's input tile with its halo is
//     staged in LDS (zero-filled outside the image);
//   * per chunk and output channel the plan holds a contiguous run of records {LDS byte
//     offset of tap (c,r,s), weight}; the run is wave-uniform, so it is fetched with scalar
//     loads, and the hot loop per record is: one address add, NV LDS reads of VW words,
//     P fused multiply-adds;
//   * with VW > 1 the tile is stored as vectors of VW consecutive rows per (row, x) slot so
//     that one ds_read_b64 / ds_read_b128 feeds VW outputs of a lane.
#include "internal.h"

namespace fscnn {

namespace {

template <int LW_, int VW_, int NV_, int SLOTS_, int WAVES_, int CC_, int R_, int S_>
struct Cfg {
    static constexpr int LW = LW_, VW = VW_, NV = NV_, SLOTS = SLOTS_, WAVES = WAVES_, CC = CC_;
    static constexpr int R = R_, S = S_;
    static constexpr int LH = 64 / LW;           // lane rows per wave
    static constexpr int P = VW * NV;            // outputs per lane (vertical)
    static constexpr int TH = LH * P, TW = LW;   // output tile of the work-group
    static constexpr int IN_ROWS = TH + R - 1;
    static constexpr int NSLOT = IN_ROWS - VW + 1;  // vector slots (start rows) per channel
    static constexpr int PITCH = TW + S - 1;        // slots per row
    static constexpr int CH_ELEMS = NSLOT * PITCH;  // slots per channel
    static constexpr int LDS_WORDS = CC * CH_ELEMS * VW;
    static constexpr int KG = SLOTS * WAVES;
    static constexpr int NT = WAVES * 64;
    static constexpr int VSTEP_BYTES = VW * PITCH * VW * 4;  // +VW rows, in bytes
};

template <int VW> struct VecT;
template <> struct VecT<1> { using T = float; };
template <> struct VecT<2> { using T = float2; };
template <> struct VecT<4> { using T = float4; };

template <int VW> __device__ inline float vec_get(const typename VecT<VW>::T &v, int e);
template <> __device__ inline float vec_get<1>(const float &v, int) { return v; }
template <> __device__ inline float vec_get<2>(const float2 &v, int e) { return e == 0 ? v.x : v.y; }
template <> __device__ inline float vec_get<4>(const float4 &v, int e)
{
    return e == 0 ? v.x : e == 1 ? v.y : e == 2 ? v.z : v.w;
}

template <class G>
__global__ void __launch_bounds__(G::NT)
conv_sf_tiled_kernel(const float *__restrict__ x, float *__restrict__ y,
                     const float *__restrict__ bias, const Rec *__restrict__ recs,
                     const int *__restrict__ segptr, int C, int H, int W, int K, int Ho, int Wo,
                     int ph, int pw, int relu, int NCH, int NG, int tiles_x, int tiles_per_img)
{
    using V = typename VecT<G::VW>::T;
    extern __shared__ __align__(16) float lds[];

    // work-group -> (channel group, spatial tile, image); groups of one tile are adjacent
    const int bid = blockIdx.x;
    const int kg = bid % NG;
    const int t = (bid / NG) % tiles_per_img;
    const int n = bid / (NG * tiles_per_img);
    const int ty0 = (t / tiles_x) * G::TH;
    const int tx0 = (t % tiles_x) * G::TW;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lx = lane % G::LW;
    const int row0 = (lane / G::LW) * G::P;  // first output row of this lane inside the tile
    const uint32_t lane_base = (uint32_t)((row0 * G::PITCH + lx) * G::VW * 4);

    float acc[G::SLOTS][G::P];
#pragma unroll
    for (int j = 0; j < G::SLOTS; ++j)
#pragma unroll
        for (int p = 0; p < G::P; ++p) acc[j][p] = 0.0f;

    const float *xn = x + (long long)n * C * H * W;
    const char *ldsb = reinterpret_cast<const char *>(lds);

    for (int ci = 0; ci < NCH; ++ci) {
        if (ci) __syncthreads();  // everyone is done reading the previous chunk
        // ---- stage the chunk's input tile (A4): slot (c, q, col) holds rows q .. q+VW-1
        for (int e = tid; e < G::CC * G::CH_ELEMS; e += G::NT) {
            const int cl = e / G::CH_ELEMS;
            const int rem = e % G::CH_ELEMS;
            const int q = rem / G::PITCH;
            const int col = rem % G::PITCH;
            const int c = ci * G::CC + cl;
            const int gx = tx0 - pw + col;
            float tmp[G::VW];
#pragma unroll
            for (int v = 0; v < G::VW; ++v) {
                const int gy = ty0 - ph + q + v;
                float val = 0.0f;
                if (c < C && gy >= 0 && gy < H && gx >= 0 && gx < W)
                    val = xn[((long long)c * H + gy) * W + gx];
                tmp[v] = val;
            }
            if constexpr (G::VW == 1) {
                lds[e] = tmp[0];
            } else if constexpr (G::VW == 2) {
                reinterpret_cast<float2 *>(lds)[e] = make_float2(tmp[0], tmp[1]);
            } else {
                reinterpret_cast<float4 *>(lds)[e] = make_float4(tmp[0], tmp[1], tmp[2], tmp[3]);
            }
        }
        __syncthreads();

        // ---- gather-FMA over this wave's records of the chunk (A5)
        const int *sp = segptr + ((long long)(kg * NCH + ci) * G::KG + wave * G::SLOTS);
        int bnd[G::SLOTS + 1];
#pragma unroll
        for (int j = 0; j <= G::SLOTS; ++j) bnd[j] = sp[j];
#pragma unroll
        for (int j = 0; j < G::SLOTS; ++j) {
            for (int i = bnd[j]; i < bnd[j + 1]; ++i) {
                const Rec rc = recs[i];
                const char *p = ldsb + (lane_base + rc.off);
#pragma unroll
                for (int v = 0; v < G::NV; ++v) {
                    const V in = *reinterpret_cast<const V *>(p + v * G::VSTEP_BYTES);
#pragma unroll
                    for (int e = 0; e < G::VW; ++e)
                        acc[j][v * G::VW + e] =
                            __builtin_fmaf(rc.val, vec_get<G::VW>(in, e), acc[j][v * G::VW + e]);
                }
            }
        }
    }

    // ---- epilogue (A6): bias, ReLU, coalesced NCHW store
    const int ox = tx0 + lx;
#pragma unroll
    for (int j = 0; j < G::SLOTS; ++j) {
        const int k = kg * G::KG + wave * G::SLOTS + j;
        if (k >= K) break;
        const float b = bias ? bias[k] : 0.0f;
        float *yk = y + ((long long)n * K + k) * Ho * Wo;
#pragma unroll
        for (int p = 0; p < G::P; ++p) {
            const int oy = ty0 + row0 + p;
            if (oy < Ho && ox < Wo) {
                float v = acc[j][p] + b;
                if (relu) v = v > 0.0f ? v : 0.0f;
                yk[(long long)oy * Wo + ox] = v;
            }
        }
    }
}

// Fallback for any stride / filter extent: one thread per output element walks its filter's
// canonical CSR(C) row and reads the taps from global memory.  Lanes run along x.
__global__ void __launch_bounds__(256)
conv_sf_direct_kernel(const int *__restrict__ rowptr, const uint32_t *__restrict__ idx,
                      const float *__restrict__ val, const float *__restrict__ x, int N, int C,
                      int H, int W, int K, int R, int S, int Ho, int Wo, int sh, int sw, int ph,
                      int pw, const float *__restrict__ bias, int relu, float *__restrict__ y)
{
    const int bx = (Wo + 63) / 64, by = (Ho + 3) / 4;
    long long b = blockIdx.x;
    const int ox = (int)(b % bx) * 64 + (threadIdx.x & 63);
    b /= bx;
    const int oy = (int)(b % by) * 4 + (threadIdx.x >> 6);
    b /= by;
    const int k = (int)(b % K);
    const int n = (int)(b / K);
    if (ox >= Wo || oy >= Ho) return;
    const float *xn = x + (long long)n * C * H * W;
    const int RS = R * S;
    float acc = 0.0f;
    const int lo = rowptr[k], hi = rowptr[k + 1];
    for (int i = lo; i < hi; ++i) {
        const uint32_t f = idx[i];
        const int c = (int)(f / RS);
        const int rs = (int)(f % RS);
        const int r = rs / S, s = rs % S;
        const int iy = oy * sh - ph + r;
        const int ix = ox * sw - pw + s;
        if (iy >= 0 && iy < H && ix >= 0 && ix < W)
            acc = __builtin_fmaf(val[i], xn[((long long)c * H + iy) * W + ix], acc);
    }
    if (bias) acc += bias[k];
    if (relu) acc = acc > 0.0f ? acc : 0.0f;
    y[(((long long)n * K + k) * Ho + oy) * Wo + ox] = acc;
}

// ---------------------------------------------------------------- variant table
using LaunchFn = hipError_t (*)(const SfPlan &, const float *, int, int, int, int, int, int, int,
                                int, int, const float *, int, float *, hipStream_t);

template <class G>
hipError_t launch_tiled(const SfPlan &p, const float *x, int N, int C, int H, int W, int K, int Ho,
                        int Wo, int ph, int pw, const float *bias, int relu, float *y,
                        hipStream_t st)
{
    constexpr int lds_bytes = G::LDS_WORDS * 4;
    static_assert(lds_bytes <= 160 * 1024, "tile exceeds the 160 KB LDS of a gfx950 compute unit");
    if (lds_bytes > 64 * 1024) {
        static hipError_t attr = hipFuncSetAttribute(
            reinterpret_cast<const void *>(&conv_sf_tiled_kernel<G>),
            hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (attr != hipSuccess) return attr;
    }
    const int tiles_x = (Wo + G::TW - 1) / G::TW;
    const int tiles_y = (Ho + G::TH - 1) / G::TH;
    const long long nblk = (long long)p.NG * tiles_x * tiles_y * N;
    if (nblk <= 0 || nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(conv_sf_tiled_kernel<G>, dim3((unsigned)nblk), dim3(G::NT), lds_bytes, st, x,
                       y, bias, p.recs, p.segptr, C, H, W, K, Ho, Wo, ph, pw, relu, p.NCH, p.NG,
                       tiles_x, tiles_x * tiles_y);
    return hipGetLastError();
}

template <class G> SfGeom geom_of()
{
    SfGeom g;
    g.LW = G::LW; g.VW = G::VW; g.NV = G::NV; g.SLOTS = G::SLOTS; g.WAVES = G::WAVES; g.CC = G::CC;
    g.R = G::R; g.S = G::S; g.TH = G::TH; g.TW = G::TW; g.NSLOT = G::NSLOT; g.PITCH = G::PITCH;
    g.KG = G::KG; g.lds_bytes = G::LDS_WORDS * 4; g.pad_to = 1;
    return g;
}

struct Variant {
    const char *name;
    SfGeom g;
    LaunchFn fn;
};

#define FSCNN_V(LW, VW, NV, SLOTS, WAVES, CC)                                                  \
    {"lw" #LW "_vw" #VW "_nv" #NV "_s" #SLOTS "_w" #WAVES "_cc" #CC,                        \
     geom_of<Cfg<LW, VW, NV, SLOTS, WAVES, CC, 3, 3>>(),                                      \
     &launch_tiled<Cfg<LW, VW, NV, SLOTS, WAVES, CC, 3, 3>>}

const Variant *variants(int *count)
{
    static const Variant table[] = {
        FSCNN_V(64, 1, 8, 8, 4, 16),   //  1
        FSCNN_V(64, 1, 8, 8, 8, 16),   //  2
        FSCNN_V(64, 1, 4, 8, 4, 16),   //  3
        FSCNN_V(64, 2, 4, 8, 4, 8),    //  4
        FSCNN_V(64, 4, 2, 8, 4, 8),    //  5
        FSCNN_V(32, 1, 8, 8, 4, 16),   //  6
        FSCNN_V(32, 4, 2, 8, 4, 8),    //  7
        FSCNN_V(16, 1, 4, 8, 4, 16),   //  8
        FSCNN_V(16, 4, 1, 8, 4, 8),    //  9
        FSCNN_V(64, 1, 8, 16, 4, 16),  // 10
    };
    *count = (int)(sizeof(table) / sizeof(table[0]));
    return table;
}

}  // namespace

int sf_variant_count()
{
    int n;
    variants(&n);
    return n;
}

const char *sf_variant_name(int variant)
{
    int n;
    const Variant *t = variants(&n);
    if (variant < 1 || variant > n) return "";
    return t[variant - 1].name;
}

bool sf_variant_geom(int variant, int R, int S, SfGeom *g)
{
    int n;
    const Variant *t = variants(&n);
    if (variant < 1 || variant > n) return false;
    if (t[variant - 1].g.R != R || t[variant - 1].g.S != S) return false;
    *g = t[variant - 1].g;
    return true;
}

// Automatic choice: lanes-per-row follows the output width so that few lanes idle.
int sf_choose_variant(int N, int C, int K, int H, int W, int R, int S)
{
    (void)N; (void)C; (void)K; (void)H;
    if (R != 3 || S != 3) return 0;
    if (W > 32) return 1;
    if (W > 16) return 6;
    return 8;
}

hipError_t launch_conv_sf_tiled(const SfPlan &p, const float *x, int N, int C, int H, int W, int K,
                                int Ho, int Wo, int ph, int pw, const float *bias, int relu,
                                float *y, hipStream_t st)
{
    int n;
    const Variant *t = variants(&n);
    if (p.variant < 1 || p.variant > n) return hipErrorInvalidValue;
    return t[p.variant - 1].fn(p, x, N, C, H, W, K, Ho, Wo, ph, pw, bias, relu, y, st);
}

hipError_t launch_conv_sf_direct(const int *rowptr, const uint32_t *idx, const float *val,
                                 const float *x, int N, int C, int H, int W, int K, int R, int S,
                                 int Ho, int Wo, int sh, int sw, int ph, int pw, const float *bias,
                                 int relu, float *y, hipStream_t st)
{
    const long long nblk = (long long)((Wo + 63) / 64) * ((Ho + 3) / 4) * N * K;
    if (nblk <= 0 || nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(conv_sf_direct_kernel, dim3((unsigned)nblk), dim3(256), 0,
                       st, rowptr, idx, val, x, N, C, H, W, K, R, S, Ho, Wo, sh, sw, ph, pw, bias,
                       relu, y);
    return hipGetLastError();
}

}  // namespace fscnn
