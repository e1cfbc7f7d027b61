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
//
// Two tiled forms.  conv_si_tiled_kernel takes the filter bank as the caller holds it
// (K x C x R x S) and transposes each chunk while staging it.  conv_si_kq_kernel takes the
// K-contiguous copy wT[c][rs][k] of a prepared filter bank: chunks arrive by direct-to-LDS
// loads into a two-buffer ring, every lane owns KQ adjacent output channels so that one 8- or
// 16-byte LDS read feeds KQ accumulators, and the list bounds and (channel, value) pairs of the
// patch's 36 input pixels are fetched ahead with vector loads (one lane per pixel) and handed
// out with readlane, so that the walk over the pixels waits for no memory but LDS.
#include "internal.h"
#include "lds_dma.h"

namespace fscnn {

namespace {

template <int TPH_, int TPW_, int WAVES_>
struct SiCfg {
    static constexpr int TPH = TPH_, TPW = TPW_, WAVES = WAVES_;
    static constexpr int CM = 2;             // chunk = CM steps of the chunk pointers
    static constexpr int CC = kSiCC * CM;
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
                     int K, int Ho, int Wo, int ph, int pw, int relu, int NCP, int NKT,
                     int tiles_x, int tiles_per_img)
{
    // NCP: steps of the chunk pointers per pixel (ceil(C / kSiCC)); NCH: chunks of this kernel
    const int NCH = (NCP + G::CM - 1) / G::CM;
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
                    const int last = (ci + 1) * G::CM < NCP ? (ci + 1) * G::CM : NCP;
                    const int beg = cptr[pix * NCP + ci * G::CM];
                    const int end = cptr[pix * NCP + last];
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

// ---- prepared filter bank: K-contiguous weights, KQ output channels per lane -------------
template <int KQ_, int WX_, int WY_, int CM_>
struct SiKqCfg {
    static constexpr int KQ = KQ_, WX = WX_, WY = WY_, CM = CM_;
    static constexpr int TP = 4;                    // a wave owns a TP x TP output patch
    static constexpr int HP = TP + 2;               // patch + halo of a 3x3 filter
    static constexpr int NPIX = HP * HP;            // input pixels a wave walks per chunk
    static constexpr int CC = kSiCC * CM;           // input channels per chunk
    static constexpr int RS = 9;
    static constexpr int WAVES = WX * WY;
    static constexpr int NT = WAVES * 64;
    static constexpr int KT = 64 * KQ;              // output channels per work-group
    static constexpr int ROW_BYTES = KT * 4;        // one (c, rs) row of the chunk in LDS
    static constexpr int BUF_BYTES = CC * RS * ROW_BYTES;
    static constexpr int NB = 2;
    static constexpr int LDS_BYTES = NB * BUF_BYTES;
    static constexpr int NLINE = BUF_BYTES / 1024;  // 1 KiB per direct-to-LDS load of a wave
    static constexpr int NLW = (NLINE + WAVES - 1) / WAVES;
    // (channel, value) pairs of a pixel's chunk list that travel through vector registers; a
    // longer list finishes through scalar loads
    static constexpr int EV = CM == 1 ? 4 : 6;
    static_assert(BUF_BYTES % 1024 == 0, "a chunk must be a whole number of 1 KiB lines");
    static_assert(KQ == 2 || KQ == 4, "8- or 16-byte weight vectors");
    static_assert(NPIX <= 64, "one lane per input pixel of the patch");
    static_assert(EV + 1 <= kSiSpare, "the fetches ahead must stay inside the spare entries");
    // two work-groups per CU when LDS and registers allow it
    static constexpr int WPE = (2 * LDS_BYTES <= 160 * 1024 && TP * TP * KQ <= 32) ? (2 * WAVES + 3) / 4
                                                                                    : (WAVES + 3) / 4;
};

template <class G>
__global__ void __launch_bounds__(G::NT, G::WPE)
conv_si_kq_kernel(const int *__restrict__ cptr, const uint32_t *__restrict__ cidx,
                  const float *__restrict__ xval, const float *__restrict__ wT,
                  const float *__restrict__ bias, float *__restrict__ y, int C, int H, int W, int K,
                  int Kpad, int Ho, int Wo, int ph, int pw, int relu, int NCP, int NKT,
                  int tiles_x, int tiles_per_img)
{
    typedef float wvec __attribute__((ext_vector_type(G::KQ)));
    extern __shared__ __align__(256) char ldsb[];
    const int NCH = (NCP + G::CM - 1) / G::CM;

    const int bid = blockIdx.x;
    const int kt = bid % NKT;
    const int tg = (bid / NKT) % tiles_per_img;
    const int n = bid / (NKT * tiles_per_img);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int oy0 = ((tg / tiles_x) * G::WY + wave / G::WX) * G::TP;
    const int ox0 = ((tg % tiles_x) * G::WX + wave % G::WX) * G::TP;
    const bool patch_live = oy0 < Ho && ox0 < Wo;   // wave-uniform

    // staging: line q of a chunk (1 KiB) holds rows (q*1024 + 16*lane) / ROW_BYTES of the chunk.
    // A wave fills lines wave, wave + WAVES, ...: their global offsets are goff0 + j * gstep (one
    // register instead of a table: the pixel loop below leaves none to spare).
    static_assert(1024 % G::ROW_BYTES == 0, "a line holds whole rows");
    const int byte0 = wave * 1024 + lane * 16;
    const int goff0 = ((byte0 / G::ROW_BYTES) * Kpad + kt * G::KT) * 4 + byte0 % G::ROW_BYTES;
    const int gstep = G::WAVES * (1024 / G::ROW_BYTES) * Kpad * 4;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)ldsb;
    const long long wbytes = (long long)C * G::RS * Kpad * 4;
    auto fetch = [&](int ci, int buf) {
        const long long first = (long long)ci * G::CC * G::RS * Kpad * 4;  // chunk's first row
        const uint64_t base = (uint64_t)(reinterpret_cast<const char *>(wT) + first);
        const long long left = wbytes - first;   // rows past the last channel read as zero
        const int4v rs = {(int)(uint32_t)base, (int)((base >> 32) & 0xffffu),
                          (int)(left > 0x7fffffffLL ? 0x7fffffffLL : left), 0x00020000};
        int off = goff0;
#pragma unroll
        for (int j = 0; j < G::NLW; ++j) {
            const int line = wave + j * G::WAVES;
            // recomputed at every use: hoisted out of the chunk loop the offsets would occupy
            // NLW registers again (and be spilled)
            asm volatile("" : "+v"(off));
            if (line < G::NLINE)
                lds_dma_dwordx4(rs, lds0 + (uint32_t)(buf * G::BUF_BYTES + line * 1024), off);
            off += gstep;
        }
    };

    // Lanes 0..35 stand for the 6x6 input pixels of patch + halo.  Per chunk, each of these lanes
    // loads where its pixel's list continues (three chunks ahead) and the first EV (channel, value)
    // pairs of the list (one chunk ahead) with vector loads; when the wave walks the pixels it
    // picks bounds and pairs out of the registers with readlane.
    const int pa = lane / G::HP, pb = lane % G::HP;
    const int piy = oy0 - ph + pa, pix_ = ox0 - pw + pb;
    const bool pin_img = patch_live && lane < G::NPIX && piy >= 0 && piy < H && pix_ >= 0 && pix_ < W;
    // a lane without a pixel reads the bounds of the image's first pixel and is masked afterwards
    // kept as a 32-bit element offset into the image's part of the pointer array (the whole
    // array has fewer than 2^31 entries) and widened at each use: one register less to hold
    const int *cimg = cptr + (long long)n * H * W * NCP;
    const int cpo = ((pin_img ? piy : 0) * W + (pin_img ? pix_ : 0)) * NCP;
    // The list positions and the first EV pairs of the NEXT chunk are fetched by ONE inline
    // assembly statement that issues the loads AND waits for them (s_waitcnt vmcnt(0)) before it
    // ends: its outputs are complete when the compiler first sees them, so no register is ever
    // "in flight" from the compiler's point of view and it may copy, split or spill them as it
    // likes.  (Loads the compiler itself knows are not an option here: it cannot count the
    // direct-to-LDS loads of the weights, and its own vmcnt waits in front of every use of a
    // loaded register would then also wait for weights that should arrive in the background.)
    // The statement sits in the middle of the pixel walk: the wave that executes it waits for one
    // memory round trip there, while the other waves of the SIMD, which are at other points of
    // their walks, keep the vector ALUs and the LDS busy.  The vmcnt(0) also covers this wave's
    // staging loads of the next chunk, issued at the top of the chunk.
    typedef int i4v __attribute__((ext_vector_type(4)));
    typedef int i2v __attribute__((ext_vector_type(2)));
    static_assert(G::EV == 4 || G::EV == 6, "pairs are fetched as one 16-byte vector, or one of 16 and one of 8 bytes");
    auto load_chunk = [&](const int *pb, int beg, int &b, int (&c)[G::EV], int (&v)[G::EV]) {
        const uint32_t *pc = cidx + beg;
        const float *pv = xval + beg;
        i4v c4, v4;
        if constexpr (G::EV == 4) {
            asm volatile("global_load_dword %0, %3, off\n\t"
                         "global_load_dwordx4 %1, %4, off\n\t"
                         "global_load_dwordx4 %2, %5, off\n\t"
                         "s_waitcnt vmcnt(0)"
                         : "=&v"(b), "=&v"(c4), "=&v"(v4)
                         : "v"(pb), "v"(pc), "v"(pv)
                         : "memory");
        } else {
            i2v c2, v2;
            asm volatile("global_load_dword %0, %5, off\n\t"
                         "global_load_dwordx4 %1, %6, off\n\t"
                         "global_load_dwordx2 %2, %6, off offset:16\n\t"
                         "global_load_dwordx4 %3, %7, off\n\t"
                         "global_load_dwordx2 %4, %7, off offset:16\n\t"
                         "s_waitcnt vmcnt(0)"
                         : "=&v"(b), "=&v"(c4), "=&v"(c2), "=&v"(v4), "=&v"(v2)
                         : "v"(pb), "v"(pc), "v"(pv)
                         : "memory");
            c[4] = c2.x; c[5] = c2.y;
            v[4] = v2.x; v[5] = v2.y;
        }
        c[0] = c4.x; c[1] = c4.y; c[2] = c4.z; c[3] = c4.w;
        v[0] = v4.x; v[1] = v4.y; v[2] = v4.z; v[3] = v4.w;
    };
    // Position of the first pair of chunk ci in the pixel's list; a chunk ends where the next one
    // begins, so one value per chunk is enough (ci may be past the last chunk: the list's end).
    auto beg_ptr = [&](int ci) { return cimg + (cpo + (ci * G::CM < NCP ? ci * G::CM : NCP)); };

    float acc[G::TP][G::TP][G::KQ];
#pragma unroll
    for (int a = 0; a < G::TP; ++a)
#pragma unroll
        for (int b = 0; b < G::TP; ++b)
#pragma unroll
            for (int q = 0; q < G::KQ; ++q) acc[a][b][q] = 0.0f;

    int b0, b1, b2;       // list positions where chunks ci, ci+1, ci+2 begin
    int ec[G::EV], nec[G::EV], ev[G::EV], nev[G::EV];   // pairs of chunks ci, ci+1 (values as bit patterns)
#pragma unroll
    for (int e = 0; e < G::EV; ++e) nec[e] = nev[e] = 0;
    fetch(0, 0);
    b0 = *beg_ptr(0);
    b1 = *beg_ptr(1);
    if (!pin_img) b0 = b1 = 0;
    load_chunk(beg_ptr(2), b0, b2, ec, ev);   // also waits for the staging loads of chunk 0
    if (!pin_img) b2 = 0;
    __syncthreads();

    for (int ci = 0; ci < NCH; ++ci) {
        const int buf = ci & 1;
        if (ci + 1 < NCH) fetch(ci + 1, buf ^ 1);
        int b3 = 0;
        const char *wl0 = ldsb + buf * G::BUF_BYTES + lane * (G::KQ * 4);
        if (patch_live) {
#pragma unroll
            for (int a = 0; a < G::HP; ++a)
#pragma unroll
            for (int b = 0; b < G::HP; ++b) {
                // half way through the walk: where the list continues three chunks on, and the
                // first pairs of the next chunk
                if (a == G::HP / 2 && b == 0) load_chunk(beg_ptr(ci + 3), b1, b3, nec, nev);
                const int j = a * G::HP + b;
                const int beg = __builtin_amdgcn_readlane(b0, j);
                const int cnt = __builtin_amdgcn_readlane(b1, j) - beg;
                // one stored (channel, value) pair of input pixel (a, b): read the weight vectors
                // of every tap the pixel feeds, then multiply
                auto entry = [&](int c, float v) {
                    const char *wl = wl0 + (c - ci * G::CC) * (G::RS * G::ROW_BYTES);
                    wvec wv[3][3];
#pragma unroll
                    for (int r = 0; r < 3; ++r)
#pragma unroll
                        for (int s = 0; s < 3; ++s) {
                            const int orow = a - r, ocol = b - s;
                            if (orow >= 0 && orow < G::TP && ocol >= 0 && ocol < G::TP)
                                wv[r][s] = *reinterpret_cast<const wvec *>(wl + (r * 3 + s) * G::ROW_BYTES);
                        }
#pragma unroll
                    for (int r = 0; r < 3; ++r)
#pragma unroll
                        for (int s = 0; s < 3; ++s) {
                            const int orow = a - r, ocol = b - s;
                            if (orow >= 0 && orow < G::TP && ocol >= 0 && ocol < G::TP) {
#pragma unroll
                                for (int q = 0; q < G::KQ; ++q)
                                    acc[orow][ocol][q] = __builtin_fmaf(v, wv[r][s][q], acc[orow][ocol][q]);
                            }
                        }
                };
                for (int e = 0; e < cnt; ++e) {
                    int c;
                    float v;
                    if (e < G::EV) {   // the pair travels in this pixel's lane of register e
                        c = __builtin_amdgcn_readlane(ec[e], j);
                        v = __int_as_float(__builtin_amdgcn_readlane(ev[e], j));
                    } else {           // rare: a list longer than the registers hold
                        c = (int)cidx[beg + e];
                        v = xval[beg + e];
                    }
                    entry(c, v);
                }
            }
        }
        wait_vmcnt<0>();   // a wave without a patch has not waited for its staging loads yet
        if (!pin_img) b3 = 0;
        b0 = b1; b1 = b2; b2 = b3;
#pragma unroll
        for (int e = 0; e < G::EV; ++e) {
            ec[e] = nec[e];
            ev[e] = nev[e];
        }
        __syncthreads();
    }

    // epilogue: a lane stores, per output channel and patch row, four adjacent pixels
    if (!patch_live) return;
    const bool vec_ok = (Wo % 4 == 0) && ((reinterpret_cast<uintptr_t>(y) & 15) == 0);
#pragma unroll
    for (int q = 0; q < G::KQ; ++q) {
        const int k = kt * G::KT + lane * G::KQ + q;
        if (k >= K) continue;
        const float bv = bias ? bias[k] : 0.0f;
        float *yk = y + ((long long)n * K + k) * Ho * Wo;
#pragma unroll
        for (int a = 0; a < G::TP; ++a) {
            const int oy = oy0 + a;
            if (oy >= Ho) continue;
            float r[G::TP];
#pragma unroll
            for (int b = 0; b < G::TP; ++b) {
                r[b] = acc[a][b][q] + bv;
                if (relu) r[b] = r[b] > 0.0f ? r[b] : 0.0f;
            }
            if (vec_ok && ox0 + G::TP <= Wo) {
                *reinterpret_cast<float4 *>(yk + (long long)oy * Wo + ox0) = make_float4(r[0], r[1], r[2], r[3]);
            } else {
#pragma unroll
                for (int b = 0; b < G::TP; ++b)
                    if (ox0 + b < Wo) yk[(long long)oy * Wo + ox0 + b] = r[b];
            }
        }
    }
}

// wT[(c*RS + rs)*Kpad + k] = w[(k*C + c)*RS + rs] (0 for k >= K)
__global__ void __launch_bounds__(256) dense_transpose_kernel(const float *__restrict__ w, int K, int C,
                                                              int RS, int Kpad, float *__restrict__ wT)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long total = (long long)C * RS * Kpad;
    if (i >= total) return;
    const int k = (int)(i % Kpad);
    const long long crs = i / Kpad;
    wT[i] = k < K ? w[(long long)k * C * RS + crs] : 0.0f;
}

// Fallback for any stride / filter extent: one wave per output pixel, lanes along k.
__global__ void __launch_bounds__(64)
conv_si_direct_kernel(const int *__restrict__ cptr, int NCP, const uint32_t *__restrict__ cidx,
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
            for (int i = cptr[pix * NCP]; i < cptr[(pix + 1) * NCP]; ++i)
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
    hipLaunchKernelGGL(conv_si_direct_kernel, dim3((unsigned)nblk), dim3(64), 0, st, in->cptr, in->NCH,
                       in->cidx, in->xval, w, bias, y, in->C, in->H, in->W, K, R, S, Ho, Wo, sh, sw,
                       ph, pw, relu, NKT);
    return hipGetLastError();
}

hipError_t launch_dense_transpose(const float *w, int K, int C, int RS, int Kpad, float *wT,
                                  hipStream_t st)
{
    const long long total = (long long)C * RS * Kpad;
    hipLaunchKernelGGL(dense_transpose_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       w, K, C, RS, Kpad, wT);
    return hipGetLastError();
}

template <class G>
static hipError_t launch_si_kq(const fscnn_input *in, const fscnn_dense *d, int Ho, int Wo, int ph, int pw,
                               const float *bias, int relu, float *y, hipStream_t st)
{
    static_assert(G::LDS_BYTES <= 160 * 1024, "weight ring exceeds the LDS of a CU");
    if (d->Kpad % G::KT != 0 || in->CC != kSiCC) return hipErrorInvalidValue;
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_si_kq_kernel<G>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES);
    if (attr != hipSuccess) return attr;
    const int NKT = d->Kpad / G::KT;
    const int tiles_x = (Wo + G::TP * G::WX - 1) / (G::TP * G::WX);
    const int tiles_y = (Ho + G::TP * G::WY - 1) / (G::TP * G::WY);
    const long long nblk = (long long)NKT * tiles_x * tiles_y * in->N;
    if (nblk <= 0 || nblk > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(conv_si_kq_kernel<G>, dim3((unsigned)nblk), dim3(G::NT), G::LDS_BYTES, st,
                       in->cptr, in->cidx, in->xval, d->wT, bias, y, in->C, in->H, in->W, d->K, d->Kpad,
                       Ho, Wo, ph, pw, relu, in->NCH, NKT, tiles_x, tiles_x * tiles_y);
    return hipGetLastError();
}

// Configurations <channels per lane, patches in x, patches in y, chunk in steps of 8 channels>.
int si_variant_count() { return 4; }

hipError_t launch_conv_si_prepared(const fscnn_input *in, const fscnn_dense *d, int Ho, int Wo, int ph,
                                   int pw, const float *bias, int relu, float *y, int variant,
                                   hipStream_t st)
{
    if (variant == 0) {
        // automatic: 16-byte weight vectors and 16-wave groups once there are enough patches to
        // fill the chip with them (measured on 28x28, C = K = 512: N = 32 yes, N = 8 no)
        const long long patches = (long long)in->N * ((Ho + 3) / 4) * ((Wo + 3) / 4) * (d->Kpad / 256);
        variant = patches >= 2048 ? 4 : 1;
    }
    switch (variant) {
    case 1:  // 2 channels per lane, 16x8 outputs and 128 channels per group, 74 KB of LDS: two groups per CU
        return launch_si_kq<SiKqCfg<2, 4, 2, 1>>(in, d, Ho, Wo, ph, pw, bias, relu, y, st);
    case 2:  // 16 waves, 16x16 outputs, 16-channel chunks
        return launch_si_kq<SiKqCfg<2, 4, 4, 2>>(in, d, Ho, Wo, ph, pw, bias, relu, y, st);
    case 3:  // 4 channels per lane (16-byte weight vectors), 256 channels per group, 8 waves
        return launch_si_kq<SiKqCfg<4, 4, 2, 1>>(in, d, Ho, Wo, ph, pw, bias, relu, y, st);
    case 4:  // the same with 16 waves
        return launch_si_kq<SiKqCfg<4, 4, 4, 1>>(in, d, Ho, Wo, ph, pw, bias, relu, y, st);
    default:
        return hipErrorInvalidValue;
    }
}

}  // namespace fscnn
