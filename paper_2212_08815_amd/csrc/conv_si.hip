// Sparse-input convolution kernels (compressed activation x dense filters -> dense NCHW).
//
// The paper (Sec. 4, end of "Sparse Tensor Convolution") runs the loops of Alg. 1 with the
// sparse operand being the input pixel's channel list and the dense operand the filter's
// channel vector at that tap.  Here this is a gather with one writer per output element:
//   * lanes run along output channels k (64 per wave), so the (channel, value) pairs of an
//     input pixel are wave-uniform and come through scalar loads;
//   * a wave owns a TPH x TPW patch of output pixels in registers; it walks the input pixels
//     of the patch plus halo, and every stored (c, v) of such a pixel feeds up to R*S outputs
//     of the patch:  acc[iy - r][ix - s] += v * w[k, c, r, s];
//   * the dense weights of the current chunk of CC input channels are staged in LDS,
//     transposed to [c][r*S+s][k] so that lanes read consecutive words.
#include "internal.h"

namespace fscnn {

namespace {

template <int TPH_, int TPW_, int WAVES_>
struct SiCfg {
    static constexpr int TPH = TPH_, TPW = TPW_, WAVES = WAVES_;
    static constexpr int CC = kSiCC;
    static constexpr int R = 3, S = 3;
    static constexpr int KT = 64;            // output channels per work-group (lanes)
    static constexpr int KP = KT + 1;        // padded k pitch in LDS (conflict-free staging)
    static constexpr int NT = WAVES * 64;
    static constexpr int LDS_WORDS = CC * R * S * KP;
};

template <class G>
__global__ void __launch_bounds__(G::NT)
conv_si_tiled_kernel(const int *__restrict__ cptr, const uint32_t *__restrict__ cidx,
                     const float *__restrict__ xval, const float *__restrict__ w,
                     const float *__restrict__ bias, float *__restrict__ y, int C, int H, int W,
                     int K, int Ho, int Wo, int ph, int pw, int relu, int NCH, int NKT,
                     int tiles_x, int tiles_per_img)
{
    __shared__ float lds[G::LDS_WORDS];
    constexpr int RS = G::R * G::S;

    const int bid = blockIdx.x;
    const int kt = bid % NKT;
    const int tg = (bid / NKT) % tiles_per_img;   // group of WAVES patches along x
    const int n = bid / (NKT * tiles_per_img);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int oy0 = (tg / tiles_x) * G::TPH;
    const int ox0 = ((tg % tiles_x) * G::WAVES + wave) * G::TPW;
    const int k = kt * G::KT + lane;

    float acc[G::TPH][G::TPW];
#pragma unroll
    for (int a = 0; a < G::TPH; ++a)
#pragma unroll
        for (int b = 0; b < G::TPW; ++b) acc[a][b] = 0.0f;

    const long long wrow = (long long)C * RS;
    for (int ci = 0; ci < NCH; ++ci) {
        if (ci) __syncthreads();
        // stage w[kt*64 .. +63][ci*CC .. +CC-1][:][:] transposed into lds[(c*RS + rs)*KP + kk]
        for (int e = tid; e < G::KT * G::CC * RS; e += G::NT) {
            const int kk = e / (G::CC * RS);
            const int rem = e % (G::CC * RS);
            const int c = ci * G::CC + rem / RS;
            const int kq = kt * G::KT + kk;
            float v = 0.0f;
            if (kq < K && c < C) v = w[(long long)kq * wrow + (long long)ci * G::CC * RS + rem];
            lds[rem * G::KP + kk] = v;
        }
        __syncthreads();

        if (oy0 < Ho && ox0 < Wo) {
#pragma unroll
            for (int a = 0; a < G::TPH + G::R - 1; ++a) {
                const int iy = oy0 - ph + a;
                if (iy < 0 || iy >= H) continue;
#pragma unroll
                for (int b = 0; b < G::TPW + G::S - 1; ++b) {
                    const int ix = ox0 - pw + b;
                    if (ix < 0 || ix >= W) continue;
                    const long long pix = ((long long)n * H + iy) * W + ix;
                    const int beg = cptr[pix * (NCH + 1) + ci];
                    const int end = cptr[pix * (NCH + 1) + ci + 1];
                    for (int i = beg; i < end; ++i) {
                        const int cl = (int)cidx[i] - ci * G::CC;
                        const float v = xval[i];
                        const float *wl = lds + cl * RS * G::KP + lane;
#pragma unroll
                        for (int r = 0; r < G::R; ++r)
#pragma unroll
                            for (int s = 0; s < G::S; ++s) {
                                const int orow = a - r, ocol = b - s;
                                if (orow >= 0 && orow < G::TPH && ocol >= 0 && ocol < G::TPW)
                                    acc[orow][ocol] = __builtin_fmaf(v, wl[(r * G::S + s) * G::KP],
                                                                     acc[orow][ocol]);
                            }
                    }
                }
            }
        }
    }

    if (k < K) {
        const float bv = bias ? bias[k] : 0.0f;
        float *yk = y + ((long long)n * K + k) * Ho * Wo;
#pragma unroll
        for (int a = 0; a < G::TPH; ++a)
#pragma unroll
            for (int b = 0; b < G::TPW; ++b) {
                const int oy = oy0 + a, ox = ox0 + b;
                if (oy < Ho && ox < Wo) {
                    float v = acc[a][b] + bv;
                    if (relu) v = v > 0.0f ? v : 0.0f;
                    yk[(long long)oy * Wo + ox] = v;
                }
            }
    }
}

// Fallback for any stride / filter extent: one wave per output pixel, lanes along k.
__global__ void __launch_bounds__(64)
conv_si_direct_kernel(const int *__restrict__ prow, const uint32_t *__restrict__ cidx,
                      const float *__restrict__ xval, const float *__restrict__ w,
                      const float *__restrict__ bias, float *__restrict__ y, int C, int H, int W,
                      int K, int R, int S, int Ho, int Wo, int sh, int sw, int ph, int pw,
                      int relu, int NKT)
{
    long long b = blockIdx.x;
    const int kt = (int)(b % NKT);
    b /= NKT;
    const int ox = (int)(b % Wo);
    b /= Wo;
    const int oy = (int)(b % Ho);
    const int n = (int)(b / Ho);
    const int k = kt * 64 + (int)threadIdx.x;
    if (k >= K) return;
    float acc = 0.0f;
    for (int r = 0; r < R; ++r) {
        const int iy = oy * sh - ph + r;
        if (iy < 0 || iy >= H) continue;
        for (int s = 0; s < S; ++s) {
            const int ix = ox * sw - pw + s;
            if (ix < 0 || ix >= W) continue;
            const long long pix = ((long long)n * H + iy) * W + ix;
            for (int i = prow[pix]; i < prow[pix + 1]; ++i)
                acc = __builtin_fmaf(xval[i], w[(((long long)k * C + cidx[i]) * R + r) * S + s], acc);
        }
    }
    if (bias) acc += bias[k];
    if (relu) acc = acc > 0.0f ? acc : 0.0f;
    y[(((long long)n * K + k) * Ho + oy) * Wo + ox] = acc;
}

}  // namespace

bool si_tiled_supported(int K, int C, int R, int S, int sh, int sw)
{
    (void)K; (void)C;
    return R == 3 && S == 3 && sh == 1 && sw == 1;
}

hipError_t launch_conv_si(const fscnn_input *in, const float *w, int K, int R, int S, int Ho, int Wo,
                          int sh, int sw, int ph, int pw, const float *bias, int relu, float *y,
                          hipStream_t st)
{
    const int NKT = (K + 63) / 64;
    if (si_tiled_supported(K, in->C, R, S, sh, sw) && in->CC == kSiCC) {
        using G = SiCfg<4, 4, 4>;
        const int tiles_x = (Wo + G::TPW * G::WAVES - 1) / (G::TPW * G::WAVES);
        const int tiles_y = (Ho + G::TPH - 1) / G::TPH;
        const long long nblk = (long long)NKT * tiles_x * tiles_y * in->N;
        if (nblk <= 0 || nblk > 0x7fffffffLL) return hipErrorInvalidValue;
        hipLaunchKernelGGL(conv_si_tiled_kernel<G>, dim3((unsigned)nblk), dim3(G::NT), 0, st,
                           in->cptr, in->cidx, in->xval, w, bias, y, in->C, in->H, in->W, K, Ho, Wo,
                           ph, pw, relu, in->NCH, NKT, tiles_x, tiles_x * tiles_y);
        return hipGetLastError();
    }
    const long long nblk = (long long)NKT * Wo * Ho * in->N;
    if (nblk <= 0 || nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(conv_si_direct_kernel, dim3((unsigned)nblk), dim3(64), 0, st, in->prow,
                       in->cidx, in->xval, w, bias, y, in->C, in->H, in->W, K, R, S, Ho, Wo, sh, sw,
                       ph, pw, relu, NKT);
    return hipGetLastError();
}

}  // namespace fscnn
