// Sparse-filter convolution kernels (dense NCHW input x compressed filters -> dense NCHW).
//
// What is computed is the direct forward pass of the paper's Alg. 6: every output element
// is the sum, over the stored nonzeros of its filter, of weight * input tap (Alg. 2's
// sparse . dense inner product), without kernel flip, padding realised as an index shift
// into a zero-filled border (Sec. 5, "Other layers").
//
// How it is mapped to gfx950 (ours, not the paper's CPU loops):
//   * output-stationary: a work-group owns a TH x TW output tile of IMGS images and KG output
//     channels; each wave owns SLOTS of those channels.  A lane keeps, per channel, NV
//     vertically adjacent outputs of BV images in fp32 registers (P = NV*BV accumulators);
//     lanes run along x (LW per row), then along LHR row groups and IG image groups, so
//     global loads and stores are coalesced along x;
//   * the input channels are walked in chunks of CC.  The chunk's input tile with its halo
//     sits in LDS with the BV images of a lane interleaved per pixel
//     ([ig][c][row][col][BV]), so one aligned ds_read_b64 / ds_read_b128 feeds BV
//     accumulators whatever the tap shift (gfx950 reads LDS about twice as fast with
//     b64/b128 as with b32; measured).  Staging uses buffer loads that write LDS directly
//     (no registers, no ds_write): lane l of a load fills dword l of a 256-byte LDS line,
//     out-of-image lanes carry an out-of-range offset and deposit 0.0.  Two LDS buffers
//     alternate: the loads of chunk ci+1 are in flight while chunk ci is computed, and one
//     barrier per chunk separates them;
//   * per wave the plan holds ONE contiguous stream of records {LDS byte offset of tap
//     (c mod CC, r, s), weight}, ordered by (chunk, channel slot).  The stream is
//     wave-uniform: it comes through scalar loads into a queue of U records in SGPRs, refilled
//     one trip ahead, and the hot loop handles U records per trip: U address adds, U*NV LDS
//     reads, U*P fused multiply-adds.
#include <type_traits>

#include "internal.h"
#include "lds_dma.h"

namespace fscnn {

namespace {

template <int BV_, int LW_, int LHR_, int NV_, int SLOTS_, int WAVES_, int CC_, int U_, int NB_, int R_, int S_,
          bool IN4_ = false, bool OUT4_ = false, bool POOL_ = false, int STRIDE_ = 1>
struct Cfg {
    static constexpr int BV = BV_, LW = LW_, LHR = LHR_, NV = NV_, SLOTS = SLOTS_, WAVES = WAVES_;
    static constexpr int CC = CC_, U = U_, NB = NB_, R = R_, S = S_;
    // STRIDE 2 (both axes): the input tile is kept as STRIDE*STRIDE planes per channel, plane
    // (y mod 2, x mod 2) holding every second row and column (a space-to-depth view built by the
    // staging loads), so that adjacent lanes still read adjacent 16-byte vectors: tap (r, s) of
    // output (oy, ox) is element (oy + r/2, ox + s/2) of plane (r mod 2, s mod 2), counted from
    // the tile's first input row and column.
    static constexpr int STRIDE = STRIDE_;
    static constexpr int PL = STRIDE * STRIDE;   // planes per input channel
    static_assert(STRIDE == 1 || STRIDE == 2, "strides 1 and 2");
    static_assert(STRIDE == 1 || !POOL_, "no pooled form at stride 2");
    // IN4 / OUT4: the input / output tensor is stored batch-interleaved by four ("N4":
    // [N/4][C][H][W][4]) instead of NCHW; then a lane's four images are 16 contiguous bytes
    static constexpr bool IN4 = IN4_, OUT4 = OUT4_;
    // POOL: the epilogue also applies the 2x2 / stride-2 max-pool (merged convolution and
    // pooling, Alg. 7) and stores the pooled tensor only
    static constexpr bool POOL = POOL_;
    static_assert(!POOL || (LW_ % 2 == 0 && (NV_ % 2 == 0 || (LW_ == 32 && LHR_ == 2))),
                  "pooling pairs columns of lane pairs and rows inside a lane (odd NV: also across lanes l, l^32)");
    static_assert((!IN4 && !OUT4) || BV == 4, "N4 tensors need four images per lane");
    static constexpr int IG = 64 / (LW * LHR);   // image groups across the lanes of a wave
    static_assert(IG * LW * LHR == 64, "lanes must factor as LW * LHR * IG");
    // U = 1, 2, 4: U records per trip of the inner loop, their taps read together, then
    // multiplied; U = 0: software-pipelined loop (the next record's taps are read while the
    // current one is multiplied)
    // U = 5: the form for filter banks without zeros and a handful of input channels (the first
    // layer of a network): the plan lists a wave's weights tap by tap, SLOTS of them per tap, and a
    // trip reads the taps of one (c, r, s) once and multiplies them into all SLOTS channels, so a
    // read feeds SLOTS * BV multiply-adds instead of BV
    static_assert(U == 0 || U == 1 || U == 2 || U == 4 || U == 5, "records per trip");
    static constexpr bool DENSE = U == 5;
    static_assert(U != 0 || BV == 4, "the pipelined loop is written for four images per lane");
    static constexpr int IMGS = BV * IG;         // images per work-group
    static constexpr int P = NV * BV;            // accumulators per lane and channel
    static constexpr int TH = LHR * NV, TW = LW; // output tile
    static constexpr int IN_ROWS = TH + (R - 1) / STRIDE;   // rows of one plane
    // Bank conflicts of the 16-byte LDS reads, measured on gfx950 with per-lane offsets: a wave
    // whose lanes 0-31 and 32-63 each read 512 contiguous bytes is conflict-free wherever the
    // two halves lie; with four groups of 16 lanes (256 contiguous bytes each) the read is
    // conflict-free only if groups 0 and 1 are a multiple of 256 bytes apart and so are groups
    // 2 and 3 (otherwise it takes twice as long).  For LW = 16, LHR = 4 the lane groups are
    // therefore given the row groups 0, 2, 1, 3 (where the kernel derives lh) and the pitch is padded
    // until two row groups are a multiple of 256 bytes apart; for LW = 16, LHR = 2 until one is.
    static constexpr int pick_pitch()
    {
        int p = TW + (S - 1) / STRIDE;
        if (LW == 16 && BV * 4 == 16 && LHR == 4)
            while ((2 * NV * p * 16) % 256 != 0) ++p;
        if (LW == 16 && BV * 4 == 16 && LHR == 2)
            while ((NV * p * 16) % 256 != 0) ++p;
        return p;
    }
    static constexpr int PITCH = pick_pitch();
    static constexpr int IG_ELEMS = CC * PL * IN_ROWS * PITCH;  // BV-vectors per image group
    static constexpr int IG_DW = IG_ELEMS * BV;            // dwords per image group
    // one staging load fills an LDS line of 64 dwords (NCHW input) or 64 BV-vectors (N4 input)
    static constexpr int LINE_BYTES = IN4 ? 1024 : 256;
    static constexpr int NI = IN4 ? (IG_ELEMS + 63) / 64 : (IG_DW + 63) / 64;  // lines per image group
    // padded so that a line never spills (a multiple of 256 bytes, which is also what the
    // lane groups of different image groups need to stay conflict-free)
    static constexpr int pick_ig_bytes() { return NI * LINE_BYTES; }
    static constexpr int IG_BYTES = pick_ig_bytes();
    static constexpr int BUF_BYTES = IG * IG_BYTES;
    static constexpr int LDS_BYTES = NB * BUF_BYTES;
    static constexpr int D = NB - 1;                       // chunks whose loads run ahead
    static_assert(NB >= 2, "at least the chunk being read and the one being loaded");
    static constexpr int KG = SLOTS * WAVES;
    static constexpr int NT = WAVES * 64;
    static constexpr int NIW = (NI + WAVES - 1) / WAVES;   // lines per wave and image group
    static constexpr int ROWSTEP = PITCH * BV * 4;         // bytes from one tile row to the next
    static constexpr int FIFO = U == 0 ? 3 : U;            // records held ahead
    // records fetched with vector loads instead of scalar ones (see rec_at in the kernel)
    static constexpr bool VREC = U == 0;
    // loads a wave may leave in flight once the NEXT chunk has to be complete: every wave
    // issues at least IG*(NI/WAVES) lines per chunk, and D-1 younger chunks follow it
    static constexpr int WAITN = (D - 1) * IG * (NI / WAVES) > 63 ? 63 : (D - 1) * IG * (NI / WAVES);
    // Waves per SIMD the register allocation aims at: as many work-groups per CU as the LDS
    // holds, as long as every wave still gets its accumulators, its taps and about two dozen
    // registers of addressing (512 vector registers per SIMD lane, 4 SIMDs per CU).
    static constexpr int pick_wpe()
    {
        const int need = P * SLOTS + (U == 0 || U == 5 ? 2 : U) * P + 24;
        for (int g = 160 * 1024 / LDS_BYTES; g > 1; --g) {
            const int w = (g * WAVES + 3) / 4;
            if (w <= 8 && 512 / w >= need) return w;
        }
        return (WAVES + 3) / 4;
    }
    static constexpr int WPE = pick_wpe();
};

constexpr int kInvalidOff = 0x7ffffff0;  // beyond any num_records: the buffer load returns 0
static_assert(kPlanSpare >= 2 * 4, "a queue refill past the last record must stay inside the spare records");
static_assert(kPlanSpare >= 8, "the taps-outer form fetches one group of 8 records past the last one");

template <int BV> struct VecT;
template <> struct VecT<1> { using T = float; };
template <> struct VecT<2> { using T = float2; };
template <> struct VecT<4> { using T = float4; };

template <int BV> __device__ inline float vget(const typename VecT<BV>::T &v, int e);
template <> __device__ inline float vget<1>(const float &v, int) { return v; }
template <> __device__ inline float vget<2>(const float2 &v, int e) { return e == 0 ? v.x : v.y; }
template <> __device__ inline float vget<4>(const float4 &v, int e)
{
    return e == 0 ? v.x : e == 1 ? v.y : e == 2 ? v.z : v.w;
}

// Keeps a loaded value live at this point of the program: the optimiser would otherwise sink
// an LDS read into the conditional block that consumes it and serialise the reads of a trip.
__device__ inline void pin(const float2 &v) { asm volatile("" : : "v"(v.x), "v"(v.y)); }
__device__ inline void pin(const float4 &v) { asm volatile("" : : "v"(v.x), "v"(v.y), "v"(v.z), "v"(v.w)); }

// The tap reads of the pipelined loop, written as instructions of their own: the compiler does
// not count them, so the loop can wait for "all but the newest NV reads" (LDS reads return in
// order) where the compiler, which loses count across a loop's back edge, would wait for all.
template <int V, int NV, int ROWSTEP> __device__ inline void lds_read_taps(f4v (&dst)[NV], uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst[V]) : "v"(addr), "n"(V * ROWSTEP));
    if constexpr (V + 1 < NV) lds_read_taps<V + 1, NV, ROWSTEP>(dst, addr);
}
// Waits until at most N of this wave's LDS reads (and scalar loads) are in flight, then names
// the taps so that nothing that uses them is moved in front of the wait.
template <int N, int NV> __device__ inline void lds_taps_landed(f4v (&buf)[NV])
{
    asm volatile("s_waitcnt lgkmcnt(%0)" : : "n"(N));
#pragma unroll
    for (int v = 0; v < NV; ++v) asm volatile("" : "+v"(buf[v]));
    __builtin_amdgcn_sched_barrier(0);
}

// Work-groups are dealt round-robin to the 8 XCDs; renumber them so that consecutive logical
// ids (the channel groups of one input tile) land on the same XCD and share its L2.
__device__ inline int xcd_remap(int bid, int nblk)
{
    const int q = nblk >> 3, rem = nblk & 7;
    const int xcd = bid & 7, slot = bid >> 3;
    return xcd < rem ? xcd * (q + 1) + slot : rem * (q + 1) + (xcd - rem) * q + slot;
}

template <class G>
__global__ void __launch_bounds__(G::NT, G::WPE)
conv_sf_tiled_kernel(const float *__restrict__ x, float *__restrict__ y,
                     const float *__restrict__ bias, const Rec *__restrict__ recs,
                     const int *__restrict__ segptr, int N, int C, int H, int W, int K, int Ho,
                     int Wo, int ph, int pw, int relu, int NCH, int NG, int tiles_x,
                     int tiles_per_img, int nblk, int csplit, long long part_stride,
                     int *__restrict__ emit_cnt, unsigned long long recs_addr, int band_shift,
                     int band_h)
{
    using V = typename VecT<G::BV>::T;
    extern __shared__ __align__(256) char ldsb[];

    // csplit > 1 (small problems): the input-channel chunks are divided among csplit
    // work-groups per (tile, channel group); part cs stores its partial sums (no bias, no
    // activation) into its own copy of the output, y + cs * part_stride, and a separate pass adds
    // the copies up in the order of the parts: one writer per element, the same bits on every run
    const int lid0 = xcd_remap(blockIdx.x, nblk);
    const int cs = lid0 % csplit;
    const int lid = lid0 / csplit;
    const int cper = (NCH + csplit - 1) / csplit;
    const int ci0 = cs * cper < NCH ? cs * cper : NCH;   // a part past the last chunk stores zeros
    const int ci1 = ci0 + cper < NCH ? ci0 + cper : NCH;
    if (csplit > 1) y += (long long)cs * part_stride;
    const int kg = lid % NG;
    const int t = (lid / NG) % tiles_per_img;
    const int n0 = (lid / (NG * tiles_per_img)) * G::IMGS;
    const int ty0 = (t / tiles_x) * G::TH;
    const int tx0 = (t % tiles_x) * G::TW;
    // Band mode (NCHW tensors on both sides, one or two images): the image slots of a lane group
    // would stay empty, so they are given horizontal bands of one image instead: slot v of the
    // launch (n0 counts slots) is band v mod 2^band_shift of image v >> band_shift, a band being
    // band_h output rows; ty0 and the tile's rows then count from the band's first row, a band's
    // halo rows are its neighbours' rows, and rows past band_h belong to the next band and are not
    // stored.  band_shift = 0: slots are images and band_h = Ho.
    const int bsh_in = G::IN4 ? 0 : band_shift, bsh_out = G::OUT4 ? 0 : band_shift;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lx = lane % G::LW;
    const int lg = (lane / G::LW) % G::LHR;
    // row group of this lane group: 0, 2, 1, 3 for four groups of 16 lanes (see PITCH)
    const int lh = (G::LW == 16 && G::LHR == 4) ? (((lg & 1) << 1) | (lg >> 1)) : lg;
    const int ig = lane / (G::LW * G::LHR);
    const uint32_t lane_base = (uint32_t)(ig * G::IG_BYTES + ((lh * G::NV) * G::PITCH + lx) * G::BV * 4);

    // ---- staging table (A4): for each LDS line this wave fills, the global byte offset of the
    // float that lands in this lane's dword, relative to channel ci*CC of the group's first
    // image.  The same table serves every chunk and image group.
    // An element of the region is (channel-plane cp, row, col), numbered in that order; a wave's
    // consecutive lines lie STEP elements apart, so only its first line is taken apart by
    // division and the others follow by adding STEP's digits with carries (with 18 lines per wave
    // for NCHW input, the divisions and 32-bit multiplications of a direct computation kept the
    // vector ALUs busy for several microseconds before the first load was issued, which is most
    // of a work-group's life on a small problem).
    const int HW = H * W;
    int goff[G::NIW];
    {
        constexpr int STEP = G::WAVES * 64 / (G::IN4 ? 1 : G::BV);
        constexpr int RP = G::IN_ROWS * G::PITCH;
        constexpr int S_CP = STEP / RP, S_ROW = (STEP % RP) / G::PITCH, S_COL = (STEP % RP) % G::PITCH;
        static_assert(G::IN4 || (G::WAVES * 64) % G::BV == 0, "a lane keeps its image slot from line to line");
        const int d0 = wave * 64 + lane;   // dword (NCHW) or vector (N4) of the region, first line
        const int e0 = G::IN4 ? d0 : d0 / G::BV, b = G::IN4 ? 0 : d0 % G::BV;
        int cp = e0 / RP, row = (e0 % RP) / G::PITCH, col = (e0 % RP) % G::PITCH;
        const int band = b & ((1 << bsh_in) - 1), img = b >> bsh_in;   // of this lane's image slot
        const int gy0 = (ty0 + band * band_h) * G::STRIDE - ph, gx0 = tx0 * G::STRIDE - pw;
        const uint32_t img_off = G::IN4 ? 0u : (uint32_t)img * (uint32_t)C * (uint32_t)HW;
        // (offsets in unsigned arithmetic: an entry that is not `ok` may wrap, and is not used)
        const uint32_t uW = (uint32_t)W, uHW = (uint32_t)HW;
        uint32_t off = 0;
        if constexpr (G::PL == 1) off = (uint32_t)cp * uHW + (uint32_t)(gy0 + row) * uW + (uint32_t)(gx0 + col);
#pragma unroll
        for (int q = 0; q < G::NIW; ++q) {
            int gy, gx;
            if constexpr (G::PL == 1) {
                gy = gy0 + row;
                gx = gx0 + col;
            } else {
                const int cl = cp / G::PL, plane = cp % G::PL;
                gy = gy0 + row * G::STRIDE + plane / G::STRIDE;
                gx = gx0 + col * G::STRIDE + plane % G::STRIDE;
                off = (uint32_t)cl * uHW + (uint32_t)gy * uW + (uint32_t)gx;
            }
            const bool ok = cp < G::CC * G::PL && gy >= 0 && gy < H && gx >= 0 && gx < W;
            goff[q] = !ok ? kInvalidOff : G::IN4 ? (int)(off * 16u) : (int)((img_off + off) * 4u);
            // the next line of this wave
            const bool c1 = col + S_COL >= G::PITCH;
            const int dcol = S_COL - (c1 ? G::PITCH : 0);
            const int drow0 = S_ROW + (c1 ? 1 : 0);
            const bool c2 = row + drow0 >= G::IN_ROWS;
            col += dcol;
            row += drow0 - (c2 ? G::IN_ROWS : 0);
            cp += S_CP + (c2 ? 1 : 0);
            if constexpr (G::PL == 1)
                off += (c2 ? (uint32_t)(S_CP + 1) * uHW : (uint32_t)S_CP * uHW) +
                       (c1 ? (uint32_t)(S_ROW + 1) * uW : (uint32_t)S_ROW * uW) -
                       (c2 ? (uint32_t)G::IN_ROWS * uW : 0u) + (uint32_t)dcol;
        }
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)ldsb;
    // Lines q with q % nparts == part only: the loads of a chunk are issued in SLOTS portions
    // spread over the computation of the previous chunk, so that the waves do not all queue at
    // the memory pipeline right after a barrier while the vector ALUs idle.
    auto fetch = [&](int ci, int buf, int part, int nparts) {
        const int crem = C - ci * G::CC;  // channels left from this chunk on (> 0)
#pragma unroll
        for (int g = 0; g < G::IG; ++g) {
            const int n = (n0 + g * G::BV) >> bsh_in;   // first image of the group
            int nvalid = N - n;
            nvalid = nvalid > (G::BV >> bsh_in) ? (G::BV >> bsh_in) : nvalid;
            // NCHW: the group's first image from channel ci*CC on, up to the end of its last
            // valid image; N4: the group's block from channel ci*CC on
            const long long first = G::IN4 ? ((long long)(n / 4) * C + (long long)ci * G::CC) * HW * 4
                                           : ((long long)n * C + (long long)ci * G::CC) * HW;
            const uint64_t base = (uint64_t)(nvalid > 0 ? x + first : x);
            const int nbytes = nvalid <= 0 ? 0 : G::IN4 ? crem * HW * 16 : ((nvalid - 1) * C + crem) * HW * 4;
            // raw buffer descriptor: 48-bit base, stride 0, num_records in bytes, 32-bit data
            const int4v rs = {(int)(uint32_t)base, (int)((base >> 32) & 0xffffu), nbytes, 0x00020000};
#pragma unroll
            for (int q = 0; q < G::NIW; ++q) {
                const int line = wave + q * G::WAVES;
                const uint32_t dst =
                    lds0 + (uint32_t)(buf * G::BUF_BYTES + g * G::IG_BYTES + line * G::LINE_BYTES);
                if (line < G::NI && q % nparts == part) {
                    if constexpr (G::IN4) lds_dma_dwordx4(rs, dst, goff[q]);
                    else lds_dma_dword(rs, dst, goff[q]);
                }
            }
        }
    };

    float acc[G::SLOTS][G::P];
#pragma unroll
    for (int j = 0; j < G::SLOTS; ++j)
#pragma unroll
        for (int p = 0; p < G::P; ++p) acc[j][p] = 0.0f;

    // How a record is fetched.  Through the scalar cache (the address is wave-uniform) its fields
    // land in SGPRs for free, but scalar loads share the LDS reads' counter and return out of
    // order, so every wait for taps becomes a wait for everything.  VREC: the same address through
    // a vector load, every lane getting its own copy (the offset of zero is made opaque, or the
    // compiler would pick the scalar load again): the fields live in vector registers, the taps'
    // waits can count down one read at a time, and the load costs a slot of the vector memory
    // pipeline per record -- which only pays where a record feeds many multiply-adds.
    // It is a buffer load with the records' base in the descriptor, the record's byte position as
    // the scalar offset and the zero as the vector offset, so the address arithmetic stays on the
    // scalar unit.  (The host refuses such a configuration for a plan beyond 2^31 bytes.)
    typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
    uint32_t vzero = 0;
    if constexpr (G::VREC) asm volatile("v_mov_b32 %0, 0" : "=v"(vzero));
    auto rec_at = [&](int idx) -> Rec {
        if constexpr (G::VREC) {
            const __amdgpu_buffer_rsrc_t rrs = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<Rec *>(recs), 0, 0x7ffffff0, 0x00020000);
            const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rrs, vzero, idx * (int)sizeof(Rec), 0);
            // (the halves are taken from the pair viewed as one 64-bit number: taken as vector
            // elements, this compiler narrows the load to one dword and hands its value to both)
            const unsigned long long w = __builtin_bit_cast(unsigned long long, v);
            const uint32_t lo = (uint32_t)w, hi = (uint32_t)(w >> 32);
            Rec r;
            r.off = lo;
            r.val = __builtin_bit_cast(float, hi);
            return r;
        } else {
            return recs[idx];
        }
    };
    // this wave's record stream, its (chunk, slot) boundaries, and the queue of records
    // (ci0 == NCH, an empty part: the entry read here is the next wave's first, or the array's
    // last one; no record is applied)
    const int *seg = segptr + ((long long)(kg * G::WAVES + wave) * NCH + ci0) * G::SLOTS;
    int i = seg[0];
    Rec q[G::FIFO];
#pragma unroll
    for (int f = 0; f < G::FIFO; ++f) q[f] = rec_at(i + f);
    int bnd[G::SLOTS];
#pragma unroll
    for (int j = 0; j < G::SLOTS; ++j) bnd[j] = ci0 < ci1 ? seg[j + 1] : i;

    // Pull the head of this wave's record stream towards the L2: the scalar loads of the hot loop
    // run only three records ahead, and a stream that was last read a whole pass of the network
    // ago comes from HBM.  One load, lane l touching the 64-byte line l of the stream (lanes past
    // its end touch nothing); the data goes to ring slot D, which nobody reads or loads before the
    // barrier below, and being the oldest load in flight it has landed by any wait further down.
    // Only where few work-groups share a stream (one per tile and image group): with thousands
    // of them it is in the L2 anyway.
    if (nblk <= 128 * NG) {
        const int iend = ci0 < ci1 ? seg[(ci1 - ci0) * G::SLOTS] : i;
        // (the records' address comes as a plain number of its own: deriving it from `recs` here
        // would let the compiler assume that the loads below may change the records)
        const uint64_t base = recs_addr + (uint64_t)i * sizeof(Rec);
        const int4v rs = {(int)(uint32_t)base, (int)((base >> 32) & 0xffffu), (iend - i) * (int)sizeof(Rec), 0x00020000};
        static_assert(G::WAVES * 256 <= G::BUF_BYTES, "one 256-byte line per wave fits a ring slot");
        lds_dma_dword(rs, lds0 + (uint32_t)(G::D * G::BUF_BYTES + wave * 256), lane * 64);
    }
    // the first D chunks start loading; chunk 0 must have landed before anyone reads it
#pragma unroll
    for (int d = 0; d < G::D; ++d)
        if (ci0 + d < ci1) fetch(ci0 + d, d, 0, 1);
    if (G::D <= ci1 - ci0) wait_vmcnt<G::WAITN>(); else wait_vmcnt<0>();
    __syncthreads();

    int rbuf = 0;         // ring slot of the chunk being computed
    int wbuf = G::D;      // ring slot the next load goes to (last read one chunk ago)
    for (int ci = ci0; ci < ci1; ++ci) {
        int nbnd[G::SLOTS];
        const bool more = ci + G::D < ci1;  // chunk ci+D is loaded while D chunks are computed
        if (ci + 1 < ci1) {
#pragma unroll
            for (int j = 0; j < G::SLOTS; ++j) nbnd[j] = seg[(ci + 1 - ci0) * G::SLOTS + j + 1];
        } else {
#pragma unroll
            for (int j = 0; j < G::SLOTS; ++j) nbnd[j] = bnd[G::SLOTS - 1];
        }
        const char *tile = ldsb + (lane_base + (uint32_t)(rbuf * G::BUF_BYTES));
        const uint32_t tile_lds = lds0 + lane_base + (uint32_t)(rbuf * G::BUF_BYTES);   // the same as an LDS address
        rbuf = rbuf + 1 == G::NB ? 0 : rbuf + 1;

        // ---- gather-FMA over this wave's records of the chunk (A5)
        if constexpr (G::U == 0) {
            // Software pipeline (BV = 4).  Invariant at the top of a trip for record i:
            // q[0..2] = records i, i+1, i+2 and the taps of record i are in flight into `cur`.
            // A trip starts the reads of record i+1 into the other buffer (its values were
            // multiplied a trip ago) and the fetch of record i+3, waits until only those newest
            // NV reads are in flight -- the taps of record i have landed then: a read has two
            // trips to come back -- and multiplies record i.  Trips come in pairs (A then B), so
            // every segment starts with its first record in buffer A; a segment's odd last
            // record is multiplied out of A and only then are the next record's reads issued
            // into A again.  Reads that run past the chunk's last record fetch a valid tap of
            // this chunk's tile and are issued again after the barrier.  The tap reads and their
            // waits are instructions written out here (lds_read_taps, lds_taps_landed): the
            // records come through vector loads, so that nothing else of this loop counts on
            // the counter the waits watch.
            static_assert(G::VREC, "the waits below count LDS reads only");
            f4v tapA[G::NV], tapB[G::NV];
            auto issue = [&](f4v(&dst)[G::NV], uint32_t off) {
                lds_read_taps<0, G::NV, G::ROWSTEP>(dst, tile_lds + off);
            };
            issue(tapA, q[0].off);
#pragma unroll
            for (int j = 0; j < G::SLOTS; ++j) {
                if (more) fetch(ci + G::D, wbuf, j, G::SLOTS);
                const int end = bnd[j];
                auto mul = [&](f4v(&cur)[G::NV]) {
#pragma unroll
                    for (int v = 0; v < G::NV; ++v) {
                        acc[j][v * 4 + 0] = __builtin_fmaf(q[0].val, cur[v].x, acc[j][v * 4 + 0]);
                        acc[j][v * 4 + 1] = __builtin_fmaf(q[0].val, cur[v].y, acc[j][v * 4 + 1]);
                        acc[j][v * 4 + 2] = __builtin_fmaf(q[0].val, cur[v].z, acc[j][v * 4 + 2]);
                        acc[j][v * 4 + 3] = __builtin_fmaf(q[0].val, cur[v].w, acc[j][v * 4 + 3]);
                    }
                };
                auto trip = [&](f4v(&cur)[G::NV], f4v(&nxt)[G::NV]) {
                    // The reads of the next record in one burst, then the multiply-adds, at
                    // raised priority once the taps have landed: such a wave is served before
                    // waves that are about to wait anyway.  (Spreading the reads between the
                    // multiply-adds measured slower.)  The priority changes end the compiler's
                    // scheduling region, so the group hints below order nothing in the trip
                    // itself; they stay because the code the compiler emits for the queue
                    // rotation after them measured 0.7 % faster with them than without.
                    issue(nxt, q[1].off);
                    const Rec fresh = rec_at(i + 3);
                    lds_taps_landed<G::NV, G::NV>(cur);
                    __builtin_amdgcn_s_setprio(3);
                    mul(cur);
                    __builtin_amdgcn_s_setprio(0);
#pragma unroll
                    for (int v = 0; v < G::NV; ++v) {
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
                    }
                    q[0] = q[1];
                    q[1] = q[2];
                    q[2] = fresh;
                    ++i;
                    __builtin_amdgcn_sched_barrier(0);
                };
                while (i + 1 < end) {
                    trip(tapA, tapB);
                    trip(tapB, tapA);
                }
                if (i < end) {  // odd tail
                    lds_taps_landed<0, G::NV>(tapA);
                    const Rec fresh = rec_at(i + 3);
                    mul(tapA);
                    __builtin_amdgcn_sched_barrier(0);
                    issue(tapA, q[1].off);
                    q[0] = q[1];
                    q[1] = q[2];
                    q[2] = fresh;
                    ++i;
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // the read in flight targets this chunk's buffer: let it land before the barrier
            // below allows that buffer to be overwritten
            lds_taps_landed<0, G::NV>(tapA);
        } else if constexpr (G::DENSE) {
            // Taps outer, channels inner.  The plan holds, for this (wave, chunk), CC*R*S groups of
            // SLOTS records {offset of the tap, weight of slot j} -- every tap of the chunk, a zero
            // weight where the bank (or the chunk past the last channel) has none.
            constexpr int T = G::CC * G::R * G::S;
            const Rec *rb = recs + ((long long)(kg * G::WAVES + wave) * NCH + ci) * (T * G::SLOTS);
            if (more) fetch(ci + G::D, wbuf, 0, 1);
            // a tap's group of records is fetched as one block of SLOTS * 2 dwords (one scalar
            // load), the next tap's block while this tap is multiplied
            static_assert(G::SLOTS == 8, "a tap's records are fetched as one 16-dword block");
            // (each record taken as one 64-bit number, its halves by shifting: taken as elements of
            // a dword vector and bit-cast, this compiler hands the first element's value to all)
            struct Group { unsigned long long rec[G::SLOTS]; };
            const Group *blk = reinterpret_cast<const Group *>(rb);
            Group cur = blk[0];
#pragma unroll 3
            for (int t = 0; t < T; ++t) {
                const Group nxt = blk[t + 1];   // past the last tap: the next block of the plan or its spare records
                V in[G::NV];
                const char *p = tile + (uint32_t)cur.rec[0];
#pragma unroll
                for (int v = 0; v < G::NV; ++v) in[v] = *reinterpret_cast<const V *>(p + v * G::ROWSTEP);
#pragma unroll
                for (int j = 0; j < G::SLOTS; ++j) {
                    const float wj = __builtin_bit_cast(float, (uint32_t)(cur.rec[j] >> 32));
#pragma unroll
                    for (int v = 0; v < G::NV; ++v)
#pragma unroll
                        for (int b = 0; b < G::BV; ++b)
                            acc[j][v * G::BV + b] =
                                __builtin_fmaf(wj, vget<G::BV>(in[v], b), acc[j][v * G::BV + b]);
                }
                cur = nxt;
            }
        } else
#pragma unroll
        for (int j = 0; j < G::SLOTS; ++j) {
            if (more) fetch(ci + G::D, wbuf, j, G::SLOTS);
            const int end = bnd[j];
            // U records per trip.  The queue q[0..U-1] always holds the U records that start at
            // stream position i; a trip reads the taps of all U, refills the queue from where the
            // next trip starts (i + U, or the segment end if that comes first: the stream is
            // contiguous, so that is where the next slot's records begin), and multiply-adds only
            // the records that belong to this slot.
            while (i < end) {
                const int left = end - i;
                const int ni = left < G::U ? end : i + G::U;
                V in[G::U][G::NV];
                __builtin_amdgcn_s_setprio(3);   // reads and refill at raised priority (see the pipelined loop)
#pragma unroll
                for (int m = 0; m < G::U; ++m) {
                    const char *p = tile + q[m].off;
#pragma unroll
                    for (int v = 0; v < G::NV; ++v)
                        in[m][v] = *reinterpret_cast<const V *>(p + v * G::ROWSTEP);
                }
                Rec fresh[G::U];
#pragma unroll
                for (int m = 0; m < G::U; ++m) fresh[m] = rec_at(ni + m);
                __builtin_amdgcn_s_setprio(0);
                if constexpr (G::U > 1) {
#pragma unroll
                    for (int m = 1; m < G::U; ++m)
#pragma unroll
                        for (int v = 0; v < G::NV; ++v) pin(in[m][v]);
                    // likewise the refill: issue it with the reads, not after the multiply-adds
#pragma unroll
                    for (int m = 0; m < G::U; ++m) asm volatile("" : : "s"(fresh[m].off), "s"(fresh[m].val));
                }
#pragma unroll
                for (int m = 0; m < G::U; ++m) {
                    if (m == 0 || m < left) {
#pragma unroll
                        for (int v = 0; v < G::NV; ++v)
#pragma unroll
                            for (int b = 0; b < G::BV; ++b)
                                acc[j][v * G::BV + b] = __builtin_fmaf(
                                    q[m].val, vget<G::BV>(in[m][v], b), acc[j][v * G::BV + b]);
                    }
                }
#pragma unroll
                for (int m = 0; m < G::U; ++m) q[m] = fresh[m];
                i = ni;
            }
            i = end;  // boundaries never decrease, so the steps above always end exactly here
        }
        wbuf = wbuf + 1 == G::NB ? 0 : wbuf + 1;
#pragma unroll
        for (int j = 0; j < G::SLOTS; ++j) bnd[j] = nbnd[j];
        // the next chunk's lines of this wave must be in LDS before the barrier lets anyone read
        if (ci + G::D < ci1) wait_vmcnt<G::WAITN>(); else wait_vmcnt<0>();
        __syncthreads();
    }

    // ---- epilogue (A6): bias, ReLU, store (coalesced along x)
    const int ox = tx0 + lx;
    if constexpr (G::POOL) {
        // merged 2x2 max-pool: rows pair up inside a lane (tile rows start even), columns across
        // the lane pair (lx, lx^1); adding the bias and the ReLU commute with the maximum.
        // With an odd number of rows per lane (32x2 lanes only) the second row group starts on
        // an odd row: its pairs are shifted by one, and the pair that straddles the two groups
        // is completed across lanes l and l^32 and stored by the first group.
        constexpr bool ODD = G::NV % 2 != 0;
        const int Hp = Ho / 2, Wp = Wo / 2;
        const int bhp = band_h >> 1;   // pooled rows of a band (band_h is even in band mode, else Ho)
        const long long pplane = (long long)Hp * Wp;
        const int px = ox >> 1;
#pragma unroll
        for (int j = 0; j < G::SLOTS; ++j) {
            const int k = kg * G::KG + wave * G::SLOTS + j;
            if (k >= K) break;
            const float bk = bias ? bias[k] : 0.0f;
            auto put = [&](int py, const float *a0, const float *a1, bool writer) {
                float r[G::BV];
#pragma unroll
                for (int b = 0; b < G::BV; ++b) {
                    float m = a1[b] > a0[b] ? a1[b] : a0[b];
                    const float o = __shfl_xor(m, 1, 64);
                    m = o > m ? o : m;
                    m += bk;
                    m = act_apply(m, relu);
                    r[b] = m;
                }
                const bool ok = writer && (lx & 1) == 0 && py < bhp && px < Wp;   // py: row of the band
                if constexpr (G::OUT4) {
                    const int n = n0 + ig * 4;
                    if (ok && n < N)
                        reinterpret_cast<float4 *>(y)[((long long)(n / 4) * K + k) * pplane +
                                                      (long long)py * Wp + px] =
                            make_float4(r[0], r[1], r[2], r[3]);
                } else {
#pragma unroll
                    for (int b = 0; b < G::BV; ++b) {
                        const int slot = n0 + ig * G::BV + b;
                        const int n = slot >> bsh_out, gpy = (slot & ((1 << bsh_out) - 1)) * bhp + py;
                        if (ok && n < N && gpy < Hp)
                            y[((long long)n * K + k) * pplane + (long long)gpy * Wp + px] = r[b];
                    }
                }
            };
            if constexpr (!ODD) {
#pragma unroll
                for (int v = 0; v < G::NV; v += 2)
                    put((ty0 + lh * G::NV + v) >> 1, &acc[j][v * G::BV], &acc[j][(v + 1) * G::BV], true);
            } else {
                const bool second = lh != 0;  // rows NV .. 2*NV-1 of the tile: pairs start at local row 1
#pragma unroll
                for (int v = 0; v + 1 < G::NV; v += 2) {
                    float a0[G::BV], a1[G::BV];
#pragma unroll
                    for (int b = 0; b < G::BV; ++b) {
                        a0[b] = second ? acc[j][(v + 1) * G::BV + b] : acc[j][v * G::BV + b];
                        a1[b] = second ? acc[j][(v + 2) * G::BV + b] : acc[j][(v + 1) * G::BV + b];
                    }
                    put((ty0 + lh * G::NV + v + (second ? 1 : 0)) >> 1, a0, a1, true);
                }
                float mine[G::BV], other[G::BV];
#pragma unroll
                for (int b = 0; b < G::BV; ++b) {
                    mine[b] = second ? acc[j][b] : acc[j][(G::NV - 1) * G::BV + b];
                    other[b] = __shfl_xor(mine[b], 32, 64);
                }
                put((ty0 + G::NV - 1) >> 1, mine, other, !second);
            }
        }
        return;
    }
    const long long plane = (long long)Ho * Wo;
#pragma unroll
    for (int j = 0; j < G::SLOTS; ++j) {
        const int k = kg * G::KG + wave * G::SLOTS + j;
        if (k >= K) break;
        const float bk = bias ? bias[k] : 0.0f;
        if constexpr (G::OUT4) {
            const int n = n0 + ig * 4;  // first image of this lane's group
            float4 *yk = reinterpret_cast<float4 *>(y) + ((long long)(n / 4) * K + k) * plane;
#pragma unroll
            for (int v = 0; v < G::NV; ++v) {
                const int oy = ty0 + lh * G::NV + v;
                if (n < N && oy < Ho && ox < Wo) {
                    if (csplit > 1) {  // partial sums of this channel range
                        yk[(long long)oy * Wo + ox] =
                            make_float4(acc[j][v * 4], acc[j][v * 4 + 1], acc[j][v * 4 + 2], acc[j][v * 4 + 3]);
                        continue;
                    }
                    float r[4];
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        r[b] = acc[j][v * 4 + b] + bk;
                        r[b] = act_apply(r[b], relu);
                    }
                    yk[(long long)oy * Wo + ox] = make_float4(r[0], r[1], r[2], r[3]);
                }
            }
        } else {
#pragma unroll
            for (int b = 0; b < G::BV; ++b) {
                const int slot = n0 + ig * G::BV + b;
                const int n = slot >> bsh_out, row0 = (slot & ((1 << bsh_out) - 1)) * band_h;
                float *yk = y + ((long long)n * K + k) * plane;
#pragma unroll
                for (int v = 0; v < G::NV; ++v) {
                    const int ly = ty0 + lh * G::NV + v;   // row of the band (of the image without bands)
                    const int oy = row0 + ly;
                    if (n < N && ly < band_h && oy < Ho && ox < Wo) {
                        if (csplit > 1) {
                            yk[(long long)oy * Wo + ox] = acc[j][v * G::BV + b];
                            continue;
                        }
                        float r = acc[j][v * G::BV + b] + bk;
                        r = act_apply(r, relu);
                        yk[(long long)oy * Wo + ox] = r;
                        // sparse output: remember in the accumulator, now dead, whether this result counts
                        acc[j][v * G::BV + b] = r != 0.0f ? 1.0f : 0.0f;
                    } else {
                        acc[j][v * G::BV + b] = 0.0f;
                    }
                }
            }
        }
    }
    // ---- sparse output emission (Sec. 4, the sparse-output remark of "Sparse Tensor Convolution"):
    // per output pixel and step of 8 output channels, the number of non-zero results -- what the
    // activation compressor counts in a pass of its own over a dense tensor.  A step's 8 channels
    // belong to 8 / SLOTS waves of this work-group: every wave drops its per-pixel counts into LDS
    // (free by now), then one thread per (step, pixel) adds them and stores the sum.  One writer per
    // count, no atomics.
    if constexpr (!G::OUT4) {
        if (emit_cnt != nullptr && csplit == 1) {
            static_assert(8 % G::SLOTS == 0 || G::SLOTS % 8 == 0, "channel steps of 8 align with the waves' slots");
            unsigned char *lc = reinterpret_cast<unsigned char *>(ldsb);   // [wave][pixel slot p][lane]
            static_assert(G::WAVES * G::P * 64 <= G::LDS_BYTES, "per-wave counts fit the tile's LDS");
            __syncthreads();   // every wave has left the chunk loop (the tile buffers are free)
            constexpr int SPW = G::SLOTS >= 8 ? G::SLOTS / 8 : 1;   // steps per wave
            constexpr int WPS = G::SLOTS >= 8 ? 1 : 8 / G::SLOTS;   // waves per step
#pragma unroll
            for (int q = 0; q < SPW; ++q)
#pragma unroll
                for (int p = 0; p < G::P; ++p) {
                    float c = 0.0f;
#pragma unroll
                    for (int j = q * (G::SLOTS / SPW); j < (q + 1) * (G::SLOTS / SPW); ++j)
                        if (kg * G::KG + wave * G::SLOTS + j < K) c += acc[j][p];
                    lc[((wave * SPW + q) * G::P + p) * 64 + lane] = (unsigned char)(int)c;
                }
            __syncthreads();
            const int NCH8 = (K + 7) / 8;
            constexpr int STEPS = G::KG / 8;   // steps of 8 channels this work-group owns
            static_assert(G::KG % 8 == 0, "a work-group owns whole steps");
            for (int t = tid; t < STEPS * G::P * 64; t += G::NT) {
                const int ln = t % 64, p = (t / 64) % G::P, st = t / (64 * G::P);
                int c = 0;
                if constexpr (G::SLOTS >= 8) {
                    c = lc[(((st / SPW) * SPW + st % SPW) * G::P + p) * 64 + ln];
                } else {
#pragma unroll
                    for (int u = 0; u < WPS; ++u) c += lc[((st * WPS + u) * G::P + p) * 64 + ln];
                }
                // pixel of (lane ln, accumulator p): the epilogue's own mapping
                const int plx = ln % G::LW, plg = (ln / G::LW) % G::LHR;
                const int plh = (G::LW == 16 && G::LHR == 4) ? (((plg & 1) << 1) | (plg >> 1)) : plg;
                const int pig = ln / (G::LW * G::LHR);
                const int v = p / G::BV, b = p % G::BV;
                const int slot = n0 + pig * G::BV + b, ly = ty0 + plh * G::NV + v, ox2 = tx0 + plx;
                const int n = slot >> bsh_out, oy = (slot & ((1 << bsh_out) - 1)) * band_h + ly;
                const int step = kg * STEPS + st;
                if (n < N && ly < band_h && oy < Ho && ox2 < Wo && step < NCH8)
                    emit_cnt[(((long long)n * Ho + oy) * Wo + ox2) * NCH8 + step] = c;
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
    acc = act_apply(acc, relu);
    y[(((long long)n * K + k) * Ho + oy) * Wo + ox] = acc;
}

// Finishing pass of the channel-split mode: y = act(bias[k] + part 0 + part 1 + ...), the parts
// added in their order.  Element i belongs to channel (i / (plane * inner)) % K, where inner is 1
// for NCHW and 4 for the batch-interleaved layout.
__global__ void __launch_bounds__(256) split_sum_kernel(const float *__restrict__ parts, int nparts,
                                                        long long part_stride, const float *__restrict__ bias,
                                                        int K, long long plane, int inner, int relu,
                                                        long long n, float *__restrict__ y)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    float v = parts[i];
    for (int p = 1; p < nparts; ++p) v += parts[(long long)p * part_stride + i];
    if (bias) v += bias[(int)((i / (plane * inner)) % K)];
    y[i] = act_apply(v, relu);
}

// The same with the merged 2x2 / stride-2 max-pool (Alg. 7): the parts hold full-size partial
// sums, element i of the pooled result is the maximum over its window of the summed parts, then
// bias and activation (they commute with the maximum, as in the merged epilogue of the kernel).
__global__ void __launch_bounds__(256) split_sum_pool_kernel(const float *__restrict__ parts, int nparts,
                                                             long long part_stride, const float *__restrict__ bias,
                                                             int K, int Ho, int Wo, int inner, int relu,
                                                             long long n, float *__restrict__ y)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int Hp = Ho / 2, Wp = Wo / 2;
    const int b = (int)(i % inner);
    const int px = (int)((i / inner) % Wp);
    const int py = (int)((i / ((long long)inner * Wp)) % Hp);
    const long long plane = i / ((long long)inner * Wp * Hp);
    float m = 0.0f;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const long long src = ((plane * Ho + 2 * py + (d >> 1)) * Wo + 2 * px + (d & 1)) * inner + b;
        float v = parts[src];
        for (int p = 1; p < nparts; ++p) v += parts[(long long)p * part_stride + src];
        m = d == 0 || v > m ? v : m;
    }
    if (bias) m += bias[(int)(plane % K)];
    y[i] = act_apply(m, relu);
}

// ---------------------------------------------------------------- variant table
using LaunchFn = hipError_t (*)(const SfPlan &, const float *, int, int, int, int, int, int, int,
                                int, int, const float *, int, float *, int, long long, int *, int, int,
                                hipStream_t);

template <class G>
hipError_t launch_tiled(const SfPlan &p, const float *x, int N, int C, int H, int W, int K, int Ho,
                        int Wo, int ph, int pw, const float *bias, int relu, float *y, int csplit,
                        long long part_stride, int *emit_cnt, int band_shift, int band_h, hipStream_t st)
{
    static_assert(G::LDS_BYTES <= 160 * 1024, "tile exceeds the 160 KB LDS of a gfx950 CU");
    if (G::LDS_BYTES > 64 * 1024) {
        static hipError_t attr = hipFuncSetAttribute(
            reinterpret_cast<const void *>(&conv_sf_tiled_kernel<G>),
            hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS_BYTES);
        if (attr != hipSuccess) return attr;
    }
    // band mode: the image slots of the launch are bands of band_h output rows (see the kernel)
    if (band_shift != 0) {
        if (G::IN4 || G::OUT4 || G::BV != 4 || band_shift < 0 || band_shift > 2 || band_h < 1 ||
            (G::POOL && band_h % 2 != 0) || ((long long)N << band_shift) > 0x7fffffffLL)
            return hipErrorInvalidValue;
    } else {
        band_h = Ho;
    }
    const int tiles_x = (Wo + G::TW - 1) / G::TW;
    const int tiles_y = (band_h + G::TH - 1) / G::TH;
    const int nbat = ((N << band_shift) + G::IMGS - 1) / G::IMGS;
    if (csplit < 1 || (G::POOL && csplit != 1)) return hipErrorInvalidValue;
    const long long nblk = (long long)p.NG * tiles_x * tiles_y * nbat * csplit;
    // (a dispatch counts its work-items in 32 bits)
    if (nblk <= 0 || nblk > 0x7fffffffLL || nblk * G::NT > 0xffffffffLL) return hipErrorInvalidValue;
    // the vector loads of the records address them with 32-bit byte offsets
    if (G::VREC && (p.nrec + kPlanSpare) * (long long)sizeof(Rec) >= 0x7ffffff0LL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(conv_sf_tiled_kernel<G>, dim3((unsigned)nblk), dim3(G::NT), G::LDS_BYTES, st,
                       x, y, bias, p.recs, p.segptr, N, C, H, W, K, Ho, Wo, ph, pw, relu, p.NCH,
                       p.NG, tiles_x, tiles_x * tiles_y, (int)nblk, csplit, part_stride, emit_cnt,
                       (unsigned long long)(uintptr_t)p.recs, band_shift, band_h);
    return hipGetLastError();
}

template <class G> SfGeom geom_of()
{
    SfGeom g;
    g.BV = G::BV; g.LW = G::LW; g.LHR = G::LHR; g.NV = G::NV; g.SLOTS = G::SLOTS;
    g.WAVES = G::WAVES; g.CC = G::CC; g.R = G::R; g.S = G::S; g.TH = G::TH; g.TW = G::TW;
    g.IMGS = G::IMGS; g.IN_ROWS = G::IN_ROWS; g.PITCH = G::PITCH; g.KG = G::KG;
    g.STRIDE = G::STRIDE;
    g.DENSE = G::DENSE ? 1 : 0;
    g.lds_bytes = G::LDS_BYTES;
    return g;
}

struct Variant {
    const char *name;
    SfGeom g;
    LaunchFn fn[2][2];    // [input is N4][output is N4]; null where the configuration has no such form
    LaunchFn pool[2][2];  // same with the merged 2x2 max-pool epilogue
};

#define FSCNN_CFG(BV, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, I4, O4) \
    Cfg<BV, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, 3, 3, I4, O4>
#define FSCNN_CFGP(BV, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, I4, O4) \
    Cfg<BV, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, 3, 3, I4, O4, true>
#define FSCNN_NOPOOL {{nullptr, nullptr}, {nullptr, nullptr}}
#define FSCNN_NAME(BV, LW, LHR, NV, SLOTS, WAVES, CC, U, NB) \
    "bv" #BV "_lw" #LW "x" #LHR "_nv" #NV "_s" #SLOTS "_w" #WAVES "_cc" #CC "_u" #U "_nb" #NB
// four images per lane: all four layout combinations
#define FSCNN_V4(LW, LHR, NV, SLOTS, WAVES, CC, U, NB)                                        \
    {FSCNN_NAME(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB),                                     \
     geom_of<FSCNN_CFG(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, false, false)>(),             \
     {{&launch_tiled<FSCNN_CFG(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, false, false)>,       \
       &launch_tiled<FSCNN_CFG(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, false, true)>},       \
      {&launch_tiled<FSCNN_CFG(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, true, false)>,        \
       &launch_tiled<FSCNN_CFG(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, true, true)>}},       \
     FSCNN_NOPOOL}
// the same plus the pooled forms (the configurations the automatic choice uses)
#define FSCNN_V4P(LW, LHR, NV, SLOTS, WAVES, CC, U, NB)                                       \
    {FSCNN_NAME(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB),                                     \
     geom_of<FSCNN_CFG(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, false, false)>(),             \
     {{&launch_tiled<FSCNN_CFG(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, false, false)>,       \
       &launch_tiled<FSCNN_CFG(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, false, true)>},       \
      {&launch_tiled<FSCNN_CFG(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, true, false)>,        \
       &launch_tiled<FSCNN_CFG(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, true, true)>}},       \
     {{&launch_tiled<FSCNN_CFGP(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, false, false)>,      \
       &launch_tiled<FSCNN_CFGP(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, false, true)>},      \
      {&launch_tiled<FSCNN_CFGP(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, true, false)>,       \
       &launch_tiled<FSCNN_CFGP(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, true, true)>}}}
// four images per lane, N4 in and out only (tuning candidates)
#define FSCNN_V4X(LW, LHR, NV, SLOTS, WAVES, CC, U, NB)                                       \
    {FSCNN_NAME(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB) "_n4only",                           \
     geom_of<FSCNN_CFG(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, true, true)>(),               \
     {{nullptr, nullptr},                                                                     \
      {nullptr, &launch_tiled<FSCNN_CFG(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, true, true)>}}, \
     FSCNN_NOPOOL}
// one or two images per lane: NCHW only
#define FSCNN_V(BV, LW, LHR, NV, SLOTS, WAVES, CC, U, NB)                                     \
    {FSCNN_NAME(BV, LW, LHR, NV, SLOTS, WAVES, CC, U, NB),                                    \
     geom_of<FSCNN_CFG(BV, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, false, false)>(),            \
     {{&launch_tiled<FSCNN_CFG(BV, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, false, false)>, nullptr}, \
      {nullptr, nullptr}},                                                                    \
     {{&launch_tiled<FSCNN_CFGP(BV, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, false, false)>, nullptr}, \
      {nullptr, nullptr}}}

// 3x3 filters at stride 2, four images per lane, all four layout combinations, no pooled form
#define FSCNN_CFGS2(LW, LHR, NV, SLOTS, WAVES, CC, U, NB, I4, O4) \
    Cfg<4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, 3, 3, I4, O4, false, 2>
#define FSCNN_V4S2(LW, LHR, NV, SLOTS, WAVES, CC, U, NB)                                      \
    {FSCNN_NAME(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB) "_st2",                              \
     geom_of<FSCNN_CFGS2(LW, LHR, NV, SLOTS, WAVES, CC, U, NB, false, false)>(),              \
     {{&launch_tiled<FSCNN_CFGS2(LW, LHR, NV, SLOTS, WAVES, CC, U, NB, false, false)>,        \
       &launch_tiled<FSCNN_CFGS2(LW, LHR, NV, SLOTS, WAVES, CC, U, NB, false, true)>},        \
      {&launch_tiled<FSCNN_CFGS2(LW, LHR, NV, SLOTS, WAVES, CC, U, NB, true, false)>,         \
       &launch_tiled<FSCNN_CFGS2(LW, LHR, NV, SLOTS, WAVES, CC, U, NB, true, true)>}},        \
     FSCNN_NOPOOL}
// 1x1 filters, four images per lane, all four layout combinations, no pooled form
#define FSCNN_CFG11(LW, LHR, NV, SLOTS, WAVES, CC, U, NB, I4, O4) \
    Cfg<4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB, 1, 1, I4, O4>
#define FSCNN_V411(LW, LHR, NV, SLOTS, WAVES, CC, U, NB)                                      \
    {FSCNN_NAME(4, LW, LHR, NV, SLOTS, WAVES, CC, U, NB) "_r1s1",                             \
     geom_of<FSCNN_CFG11(LW, LHR, NV, SLOTS, WAVES, CC, U, NB, false, false)>(),              \
     {{&launch_tiled<FSCNN_CFG11(LW, LHR, NV, SLOTS, WAVES, CC, U, NB, false, false)>,        \
       &launch_tiled<FSCNN_CFG11(LW, LHR, NV, SLOTS, WAVES, CC, U, NB, false, true)>},        \
      {&launch_tiled<FSCNN_CFG11(LW, LHR, NV, SLOTS, WAVES, CC, U, NB, true, false)>,         \
       &launch_tiled<FSCNN_CFG11(LW, LHR, NV, SLOTS, WAVES, CC, U, NB, true, true)>}},        \
     FSCNN_NOPOOL}

const Variant *variants(int *count)
{
    static const Variant table[] = {
        FSCNN_V4P(32, 2, 2, 4, 8, 3, 1, 2),    //  1  wide, few-channel layers (an RGB image is one chunk): 32x4 tiles, 8 waves
        FSCNN_V4P(32, 2, 4, 4, 16, 14, 0, 2),  //  2  32x8 tiles, 16 waves, 4 channels each, large chunks, pipelined (second choice after 6)
        FSCNN_V4P(16, 4, 2, 2, 16, 25, 4, 2),  //  3  14x14: 16x8 tiles, 2 channels per wave, 4 records per trip; 25 channels fill the LDS (512 channels = 21 chunks)
        FSCNN_V4P(32, 2, 4, 2, 16, 7, 1, 2),   //  4  32x8 tiles, 2 channels per wave, two groups per CU (second choice after 26 on 112x112)
        FSCNN_V4P(32, 2, 2, 4, 16, 12, 1, 2),  //  5  32x4 tiles, two groups per CU (second choice after 26 on 224x224)
        FSCNN_V4P(32, 2, 7, 2, 16, 9, 0, 2),   //  6  32x14 tiles: heights 28 and 56 without idle rows, pipelined
        FSCNN_V4(64, 1, 4, 4, 16, 8, 1, 3),    //  7  64-wide rows
        FSCNN_V4(16, 1, 4, 4, 8, 4, 1, 3),     //  8  16 images per group
        FSCNN_V4(16, 4, 4, 2, 8, 14, 1, 2),    //  9  16x16 tiles, 8 waves
        FSCNN_V4X(32, 2, 4, 4, 16, 14, 1, 2),  // 10  as 2, not pipelined
        FSCNN_V(1, 64, 1, 8, 8, 8, 8, 1, 2),   // 11  one image per lane (N < 4)
        FSCNN_V(1, 32, 2, 8, 8, 8, 8, 1, 2),   // 12
        FSCNN_V(1, 16, 4, 4, 8, 8, 8, 1, 2),   // 13
        FSCNN_V(2, 64, 1, 4, 8, 8, 8, 2, 2),   // 14  two images per lane
        FSCNN_V4X(32, 2, 4, 4, 16, 14, 2, 2),  // 15  as 2, two records per trip
        FSCNN_V4X(32, 2, 7, 2, 16, 9, 1, 2),   // 16  as 6, not pipelined
        FSCNN_V4X(16, 4, 2, 2, 16, 24, 1, 2),  // 17  as 3, one record per trip
        // 1x1 filters: no halo, so the chunks hold more channels; a (chunk, channel) segment is
        // still 9 times shorter than for 3x3 at the same density
        FSCNN_V411(32, 2, 4, 4, 16, 18, 1, 2), // 18  32x8 tiles
        FSCNN_V411(32, 2, 7, 2, 16, 10, 0, 2), // 19  32x14 tiles, pipelined
        FSCNN_V411(16, 4, 2, 2, 16, 36, 4, 2), // 20  16x8 tiles
        FSCNN_V411(32, 2, 4, 4, 16, 18, 2, 2), // 21  as 18, two records per trip
        // 3x3 at stride 2: four planes per channel, so fewer channels fit a chunk
        FSCNN_V4S2(16, 4, 2, 2, 16, 7, 1, 2),  // 22  16x8 tiles, 2 channels per wave
        FSCNN_V4S2(32, 2, 4, 2, 16, 4, 1, 2),  // 23  32x8 tiles
        FSCNN_V4S2(16, 4, 2, 4, 16, 7, 1, 2),  // 24  16x8 tiles, 4 channels per wave
        FSCNN_V4S2(16, 4, 2, 2, 16, 7, 4, 2),  // 25  as 22, four records per trip
        FSCNN_V4P(16, 4, 2, 4, 16, 12, 1, 2),  // 26  112x112 and 224x224: 16x8 tiles (widths 7*2^k without idle columns), 4 channels per wave
        FSCNN_V4S2(32, 2, 4, 4, 16, 4, 1, 2),  // 27  stride 2, outputs 17..64 wide: 32x8 tiles, 4 channels per wave
        FSCNN_V4S2(16, 4, 2, 4, 16, 3, 1, 2),  // 28  stride 2, wider outputs: 16x8 tiles, 4 channels per wave, small chunks
        FSCNN_V411(32, 2, 2, 4, 16, 40, 4, 2), // 29  1x1, 17..32 wide: 32x4 tiles, 40-channel chunks
        FSCNN_V411(16, 4, 1, 4, 16, 80, 4, 2), // 30  1x1, up to 16 wide: 16x4 tiles, 80-channel chunks
        FSCNN_V411(32, 2, 2, 2, 16, 20, 4, 2), // 31  1x1, wider than 128: 32x4 tiles, 2 channels per wave
        FSCNN_V4P(16, 4, 4, 2, 16, 15, 0, 2),  // 32  up to 16x16 images with many output channels: one 16x16 tile per image, pipelined
        FSCNN_V4P(16, 4, 2, 8, 8, 3, 5, 2),    // 33  banks without zeros over up to 3 input channels (an RGB first layer): taps outer, 8 channels per wave, 16x8 tiles (32x4: 4 % slower, 64x2: 20 %)
        FSCNN_V4P(16, 4, 2, 8, 4, 3, 5, 2),    // 34  the same with 32 channels per work-group (4 waves), for banks of 32, 96, ... channels
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

bool sf_variant_geom(int variant, int R, int S, int sh, int sw, SfGeom *g)
{
    int n;
    const Variant *t = variants(&n);
    if (variant < 1 || variant > n) return false;
    if (t[variant - 1].g.R != R || t[variant - 1].g.S != S) return false;
    if (t[variant - 1].g.STRIDE != sh || sh != sw) return false;
    *g = t[variant - 1].g;
    return true;
}

bool sf_variant_has_layout(int variant, int in4, int out4, int pool)
{
    int n;
    const Variant *t = variants(&n);
    if (variant < 1 || variant > n) return false;
    const Variant &v = t[variant - 1];
    return (pool ? v.pool : v.fn)[in4 ? 1 : 0][out4 ? 1 : 0] != nullptr;
}

// Work-groups a configuration launches for a layer.
static long long sf_blocks(const SfGeom &g, int N, int K, int Ho, int Wo)
{
    const long long tiles = (long long)((Wo + g.TW - 1) / g.TW) * ((Ho + g.TH - 1) / g.TH);
    return tiles * ((K + g.KG - 1) / g.KG) * ((N + g.IMGS - 1) / g.IMGS);
}

// Automatic choice.  Batches of at least four images use the image-interleaved (b128)
// configurations.  Preference order measured on VGG16-shaped layers (N = 32, 95 % sparse):
// 8-wave groups with small chunks for the wide layers with a handful of input channels; from
// 224x224 down to 56x56, 16-wave groups whose 64 registers and half-size tiles let two groups
// share a CU (32 waves hide the LDS latency, and a group that waits at its barrier leaves the
// CU to the other); at 56x56 and 28x28 without pooling, 32x14 tiles (7 rows per lane: no idle
// rows for heights 28 and 56, and 28 multiply-adds per record fetched) with the pipelined
// loop; with pooling, 4 channels per wave with the largest chunks LDS holds twice, pipelined;
// 16x8 tiles with two channels per wave for 14x14, which keeps 256 groups of 16 waves in flight.  A configuration that
// would launch too few work-groups to cover the 256 compute units, or that has no pooled form
// when one is asked for, yields to the next one.
int sf_choose_variant(int N, int C, int K, int H, int W, int R, int S, int stride, bool pool, bool n4,
                      bool no_zeros, bool banded)
{
    int n;
    const Variant *t = variants(&n);
    // a bank without zeros over at most 3 input channels (the first layer of a network fed RGB
    // images): the taps-outer form, where it fills the chip and its 64 channels per work-group
    // are all real ones (measured on 3->64 at 224x224, N = 32: 0.148 -> 0.123 ms)
    if (no_zeros && stride == 1 && R == 3 && S == 3 && C <= 3 && N >= 4 && K % 32 == 0) {
        const int v = K % 64 == 0 ? 33 : 34;
        if (sf_blocks(t[v - 1].g, N, K, H, W) >= 512) return v;
    }
    if (stride == 2) {   // 3x3 only, four-image forms, no pooled form; H, W are the output's here
        if (R != 3 || S != 3 || pool) return 0;
        const int first = W > 64 ? 28 : W > 16 ? 27 : 24;   // measured on Darknet-53's down-sampling layers, N = 32
        if (sf_blocks(t[first - 1].g, N, K, H, W) >= 192) return first;
        return sf_blocks(t[24 - 1].g, N, K, H, W) >= 192 ? 24 : 22;
    }
    if (stride != 1) return 0;
    if (R == 1 && S == 1) {   // 1x1: four-image forms only, no pooled form
        if (pool) return 0;
        // measured on Darknet-53's 1x1 layers, N = 32
        const int cand[4] = {W > 128 ? 31 : W > 32 ? 18 : W > 16 ? 29 : 30, W > 16 ? 18 : 20, 20, 19};
        for (int i = 0; i < 4; ++i)
            if (sf_blocks(t[cand[i] - 1].g, N, K, H, W) >= 192) return cand[i];
        return 20;
    }
    if (R != 3 || S != 3) return 0;
    // One or two images in band mode (N counts the slots, H a band's rows): the work is small and
    // what counts is the number of work-groups and how short each one's chain of chunks is, so the
    // form with two channels per wave and the largest chunks, which the channel split then cuts
    // into parts (measured on the VGG16-shaped stack at N = 1, every layer from 224x224 to 14x14)
    if (banded && !(W > 64 && C <= 8)) return 3;
    int pref[4];
    // Fewer than four images: the one-image-per-lane forms only pay on the widest layers; from
    // 112x112 down they launch too few work-groups, and the four-image forms with idle image
    // slots are faster (measured on the same stack at N = 1).
    if (N >= 4 || W <= 112) {
        if (W > 64 && C <= 8) { pref[0] = 1; pref[1] = 4; pref[2] = 3; pref[3] = 3; }
        else if (W > 128) { pref[0] = 26; pref[1] = 5; pref[2] = 4; pref[3] = 3; }
        else if (W > 64) { pref[0] = 26; pref[1] = 4; pref[2] = 2; pref[3] = 3; }
        else if (W > 32) { pref[0] = 6; pref[1] = 2; pref[2] = 4; pref[3] = 3; }
        else if (W > 16) { pref[0] = 6; pref[1] = 2; pref[2] = 4; pref[3] = 3; }
        else { pref[0] = 32; pref[1] = 3; pref[2] = 9; pref[3] = 9; }
    } else {
        if (W > 32) { pref[0] = 11; pref[1] = 12; pref[2] = 13; pref[3] = 13; }
        else if (W > 16) { pref[0] = 12; pref[1] = 13; pref[2] = 13; pref[3] = 13; }
        else { pref[0] = 13; pref[1] = 13; pref[2] = 13; pref[3] = 13; }
    }
    // NCHW tensors on both sides: staging costs four times the load instructions, so the form
    // that stages the input half as often (64 channels per group) comes first
    if (!n4 && pref[0] == 6) { pref[0] = 2; pref[1] = 6; pref[2] = 4; pref[3] = 3; }
    // ... and on the wide layers the 32x4 tiles, whose staging lines are the longest runs of x
    if (!n4 && pref[0] == 26) { pref[3] = pref[2]; pref[2] = pref[1] == 5 ? 4 : pref[1]; pref[1] = 26; pref[0] = 5; }
    // the 14-row tiles do not pay where they waste more rows than the 8-row ones
    auto covered = [&](const SfGeom &g) {
        return (long long)((W + g.TW - 1) / g.TW) * g.TW * ((H + g.TH - 1) / g.TH) * g.TH;
    };
    if (pref[0] == 6 && covered(t[5].g) > covered(t[pref[1] - 1].g)) {
        pref[0] = pref[1];
        pref[1] = 6;
    }
    int best = 0;
    long long best_blocks = -1;
    for (int i = 0; i < 4; ++i) {
        const Variant &v = t[pref[i] - 1];
        if (pool && !v.pool[0][0]) continue;
        const long long b = sf_blocks(v.g, N, K, H, W);  // Ho, Wo ~ H, W for this purpose
        if (b >= 192) return pref[i];
        if (b > best_blocks) { best_blocks = b; best = pref[i]; }
    }
    return best;
}

// Band mode (see the kernel): with NCHW tensors on both sides and one or two images, a four-image
// configuration fills its image slots with 4 / N horizontal bands of each image.  band_h: output
// rows per band, even where the merged pool pairs rows.  shift = 0: no bands, band_h = Ho.
void sf_choose_bands(int variant, int N, int Ho, bool n4, bool pool, int *shift, int *band_h)
{
    int n;
    const Variant *t = variants(&n);
    *shift = 0;
    *band_h = Ho;
    if (variant < 1 || variant > n || t[variant - 1].g.BV != 4 || n4 || N > 2) return;
    *shift = N == 1 ? 2 : 1;
    int h = (Ho + (1 << *shift) - 1) >> *shift;
    if (pool) h += h & 1;
    *band_h = h;
}

long long sf_split_elems(int N, int K, int Ho, int Wo, int out4)
{
    return (out4 ? ((long long)N + 3) / 4 * 4 : (long long)N) * K * Ho * Wo;
}

hipError_t launch_conv_sf_tiled(const SfPlan &p, const float *x, int N, int C, int H, int W, int K,
                                int Ho, int Wo, int ph, int pw, const float *bias, int relu,
                                float *y, int in4, int out4, int pool, int csplit, float *parts,
                                int *emit_cnt, int band_shift, int band_h, hipStream_t st)
{
    int n;
    const Variant *t = variants(&n);
    if (p.variant < 1 || p.variant > n) return hipErrorInvalidValue;
    const Variant &v = t[p.variant - 1];
    // (the channel-split mode launches the form without the pool: its finishing pass pools)
    LaunchFn fn = (pool && csplit == 1 ? v.pool : v.fn)[in4 ? 1 : 0][out4 ? 1 : 0];
    if (!fn) return hipErrorInvalidValue;
    if (csplit > 1) {
        // every part stores its partial sums into its own copy of the full-size output (parts:
        // csplit * sf_split_elems floats of scratch), then one pass adds the copies, pools where
        // asked to, and applies bias and activation
        if (!parts) return hipErrorInvalidValue;
        const long long total = sf_split_elems(N, K, Ho, Wo, out4);
        if (emit_cnt) return hipErrorInvalidValue;   // the parts' sums are not final results
        hipError_t e = fn(p, x, N, C, H, W, K, Ho, Wo, ph, pw, bias, relu, parts, csplit, total, nullptr,
                          band_shift, band_h, st);
        if (e != hipSuccess) return e;
        if (pool) {
            const long long pooled = sf_split_elems(N, K, Ho / 2, Wo / 2, out4);
            hipLaunchKernelGGL(split_sum_pool_kernel, dim3((unsigned)((pooled + 255) / 256)), dim3(256), 0, st,
                               parts, csplit, total, bias, K, Ho, Wo, out4 ? 4 : 1, relu, pooled, y);
        } else {
            hipLaunchKernelGGL(split_sum_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, parts,
                               csplit, total, bias, K, (long long)Ho * Wo, out4 ? 4 : 1, relu, total, y);
        }
        return hipGetLastError();
    }
    if (emit_cnt && (out4 || pool)) return hipErrorInvalidValue;
    return fn(p, x, N, C, H, W, K, Ho, Wo, ph, pw, bias, relu, y, 1, 0, emit_cnt, band_shift, band_h, st);
}

// How many ways the input channels are split for a launch: small problems (deep layers at small
// batch) leave most of the 256 CUs idle and serialise hundreds of channels in a few groups;
// splitting the chunk range restores parallelism at the price of one copy of the output per part
// and a finishing pass that adds them up, which only pays while y is small (measured: 14x14 and
// 28x28 at N <= 8 gain up to 3.7x, 56x56 and wider lose).
int sf_choose_csplit(int variant, int N, int K, int Ho, int Wo, int NCH)
{
    int n;
    const Variant *t = variants(&n);
    if (variant < 1 || variant > n) return 1;
    const long long b = sf_blocks(t[variant - 1].g, N, K, Ho, Wo);
    if (b > 128 || NCH < 4) return 1;   // with more groups the extra passes cost more than they gain
    long long s = (256 + b - 1) / b;
    if (s > NCH / 2) s = NCH / 2;   // at least two chunks per part
    if (s > 8) s = 8;
    const long long outputs = (long long)N * K * Ho * Wo;
    if (s * outputs > (4LL << 20)) s = (4LL << 20) / outputs;   // bound the scratch and its traffic
    return s < 1 ? 1 : (int)s;
}

hipError_t launch_conv_sf_direct(const int *rowptr, const uint32_t *idx, const float *val,
                                 const float *x, int N, int C, int H, int W, int K, int R, int S,
                                 int Ho, int Wo, int sh, int sw, int ph, int pw, const float *bias,
                                 int relu, float *y, hipStream_t st)
{
    const long long nblk = (long long)((Wo + 63) / 64) * ((Ho + 3) / 4) * N * K;
    if (nblk <= 0 || nblk > 0x7fffffffLL || nblk * 256 > 0xffffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(conv_sf_direct_kernel, dim3((unsigned)nblk), dim3(256), 0, st, rowptr, idx,
                       val, x, N, C, H, W, K, R, S, Ho, Wo, sh, sw, ph, pw, bias, relu, y);
    return hipGetLastError();
}

}  // namespace fscnn
