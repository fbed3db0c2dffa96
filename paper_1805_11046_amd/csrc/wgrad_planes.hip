// Weight gradient of 3x3 convolutions whose result planes are 14x14 or 7x7 (stride 1 or 2, pad 1) or 28x28 (stride 2):
//   dW[k,c,r,s] = sum_{n,p,q} g16[n,k,p,q] * x8[n,c,p*st+r-1,q*st+s-1]      (Section 4, eq. (grad_weight))
// with the 16-bit copy of the gradient (Sections 1, 7) and the 8-bit layer input, exact in integers; and of the 1x1
// convolution at stride 2 without padding on the same result planes (one tap, x8[n,c,2p,2q]).
//
// GEMM view: rows = output channel k (two byte planes: s = 256*hi + lo + 128), cols = (input
// channel c, tap), reduction = (image, position).  Both operands are contiguous along the
// reduction in NCHW, so nothing is transposed; no operand is rewritten in HBM.
//
// Padded planes.  Inside LDS a 14x14 plane is a 16x16 block of bytes (7x7: 8x8): pad columns, then
// the data of an image row, and pad rows after the last image row, all pads holding the operand's
// zero point.  A chunk of the reduction is 256 such padded positions (one 14x14 plane or four 7x7
// planes) = 8 MFMA K-steps of 32.  In these coordinates a filter tap is a byte offset; the pad
// before one row is the pad after the previous one, and the pad rows of one plane separate it from
// the next one.  Staging writes data positions only, the pads are set once per workgroup.  A 28x28 plane (32x32
// padded) is four chunks: a chunk is a band of 8 padded rows, the rows of the last band that lie past the plane are
// staged as zero codes, and the input row above a band is carried over from the previous band inside LDS.
//   * the vertical tap is an offset of +-pitch on the input operand (aligned 16-byte LDS reads for
//     pitch 16, 8-byte reads for pitch 8);
//   * the horizontal tap is moved to the gradient operand (p' = p + s - 1), whose fragment is
//     shifted by one byte with v_alignbyte: two aligned reads instead of an unaligned one;
//   * stride 2: the input plane (2P x 2P) is de-interleaved into its four (row parity, column
//     parity) classes while it is staged; every tap then reads one class at offset 0 or -1 in
//     either direction, the same structure as stride 1.
// Because position 0 and the last position of a chunk are pads and the margins of a row hold zero
// codes, the row sums of the gradient do not depend on the shift; the column sums of the input
// depend on the vertical offset (one per variant of the input fragment).
//
// What bounds kernels of this kind on gfx950 is the number of instructions a wavefront issues per
// MFMA, so the product runs on v_mfma_i32_32x32x32_i8 (twice the work per instruction and per
// fragment of v_mfma_i32_16x16x64_i8) with a register tile that reuses every fragment three times:
// a wavefront holds 32 rows x 32 channels x 9 taps of one byte plane = 9 accumulator tiles (144
// registers, all of them in the accumulation registers), fed per K-step by one gradient read
// (shifted twice in registers) and 3 (stride 2: 6) input reads.  A workgroup is eight wavefronts
// (row half, byte plane, channel half), two per SIMD: 64 output channels x 64 input channels and a
// range of images.  Row and column sums for the zero-point correction are v_dot4 on fragments,
// dealt out over the wavefronts that share them.  Partial sums
// per image range are int32 (a range stays below the 32-bit bound) and are combined in int64 by
// wgrad_planes_finish together with the zero-point correction and the dequantization.
#include <type_traits>

#include "q8t_common.h"
#include "q8t_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kThreads = 512;
constexpr int KC = 256;                 // padded positions per chunk (8 K-steps of 32)
constexpr int ROWP = 336;               // LDS bytes per operand row: 16 + 256 + 16 and a spare 48, so that the pitch is
                                        // 84 dwords = 20 mod 64: 16 rows of 16-byte fragments fall into 16 distinct bank groups
constexpr int KT = 64;                  // output channels per workgroup
constexpr int CT = 64;                  // input channels per workgroup

struct PGeom {
    int N, C, K;
    int S, ipr;      // image ranges, images per range (a multiple of the images per chunk)
    int nrg, ncg;    // row groups (K/64), channel groups (C/64)
};

// KS_ = 3: 3x3 filter, pad 1.  KS_ = 1: the 1x1 filter at stride 2 without padding (the projection shortcut of a
// down-sampling block): one tap, which reads the (even row, even column) class of the input plane only.
template <int P_, int STRIDE_, int KS_ = 3>
struct Shape {
    static constexpr int P = P_, STRIDE = STRIDE_, KS = KS_;
    static_assert(KS == 3 || (KS == 1 && STRIDE == 2), "filters served: 3x3 at stride 1 or 2, 1x1 at stride 2");
    static_assert(P == 7 || P == 14 || (P == 28 && STRIDE == 2), "result planes served: 7x7, 14x14, and 28x28 at stride 2");
    static constexpr int PT = P == 28 ? 32 : (P == 14 ? 16 : 8);   // padded row pitch
    static constexpr int LEADC = PT - P;                 // pad columns, at the start of a row (so that position 0 is a pad)
    static constexpr int PL = PT * PT;                   // padded positions per plane
    static constexpr int NBAND = PL > KC ? PL / KC : 1;  // chunks per plane: a 28x28 plane goes in four bands of 8 padded rows
    static constexpr int NIMG = NBAND > 1 ? 1 : KC / PL; // planes per chunk
    static constexpr int LEFT = PT > 16 ? PT : 16;       // bytes before the chunk in an LDS row: margin, and the row above a band
    static constexpr int TAPS = KS * KS;
    static constexpr int NCLS = STRIDE == 1 || KS == 1 ? 1 : 4;     // parity classes of the input plane that are staged
    static constexpr int NBV = KS == 1 ? 1 : (STRIDE == 1 ? 3 : 6); // distinct input fragments per K-step
    static constexpr int NAS = KS == 1 ? 1 : (STRIDE == 1 ? 3 : 2); // distinct shifts of the gradient fragment
    static constexpr int WIN = P * STRIDE;               // input plane edge
    static constexpr int A_BYTES = 2 * KT * ROWP;
    static constexpr int CLSB = CT * ROWP;               // bytes of one parity class
    static constexpr int B_BYTES = NCLS * CLSB;
    static constexpr int BUF = A_BYTES + B_BYTES;
    static constexpr bool DB = NCLS == 1 && NBAND == 1;  // two LDS buffers (four classes leave room for one; bands keep to one)
    static constexpr int SMEM = (DB ? 2 : 1) * BUF;
    static constexpr int HALF_INTS = 4 * TAPS * 16 * 64;     // accumulators of one byte plane: [row half][channel half][tap][reg][lane]
    static constexpr int TILE_INTS = 2 * HALF_INTS;
    static constexpr int PART_INTS = TILE_INTS + NBV * CT + 2 * KT;   // + column sums [variant][ch] + row sums [plane][row]
    static constexpr int CSW = (NBV + 3) / 4;            // column sums gathered per wavefront (variants 4i + its index among the four that share a channel half)

    // tap t = 3r + s -> variant of the input fragment, shift index of the gradient fragment (0: g[p' + 1], 1: g[p'], 2: g[p' - 1])
    //   stride 1: variant r (offset (r-1)*PT), gradient g[p' - (s-1)]: shift index s = {+1, 0, -1}
    //   stride 2: input row 2p+r-1 -> (parity, offset) r=0:(1,-PT) r=1:(0,0) r=2:(1,0); column likewise
    //             s=0:(1,-1) s=1:(0,0) s=2:(1,0); the -1 moves to the gradient as g[p'+1]: shift index {+1, 0}
    //   1x1: the one tap reads class (0, 0) at offset 0 against the unshifted gradient
    static __host__ __device__ constexpr int bvar(int t) { return KS == 1 ? 0 : (STRIDE == 1 ? t / 3 : (t / 3) * 2 + (((t % 3) & 1) ? 0 : 1)); }
    static __host__ __device__ constexpr int ashift(int t) { return KS == 1 ? 1 : (STRIDE == 1 ? t % 3 : ((t % 3) == 0 ? 0 : 1)); }
    static __host__ __device__ constexpr int bcls(int v) { return STRIDE == 1 || KS == 1 ? 0 : ((v >> 1) == 1 ? 0 : 2) + (v & 1); }
    static __host__ __device__ constexpr int boff(int v) { return KS == 1 ? 0 : (STRIDE == 1 ? (v - 1) * PT : ((v >> 1) == 0 ? -PT : 0)); }
};

__device__ __forceinline__ int dot4_ones(int v, int acc) { return __builtin_amdgcn_sdot4(v, 0x01010101, acc, false); }

template <class SH>
__global__ __launch_bounds__(kThreads) void wgrad_planes(const int16_t *__restrict__ g16, const int8_t *__restrict__ x,
                                                         const q8t_qparams *__restrict__ qpg,
                                                         const q8t_qparams *__restrict__ qpx, PGeom g,
                                                         int *__restrict__ partial)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    constexpr int P = SH::P, PT = SH::PT, PL = SH::PL, NIMG = SH::NIMG, TAPS = SH::TAPS;
    constexpr int NBV = SH::NBV, NAS = SH::NAS, WIN = SH::WIN, STRIDE = SH::STRIDE, KS = SH::KS;
    constexpr int LEFT = SH::LEFT, NBAND = SH::NBAND, LEADC = SH::LEADC;
    constexpr int PP = P * P, WW = WIN * WIN;
    constexpr int NPART = 4;                                                // staging is spread over 4 of the 8 K-steps

    // XCD-aware decode (workgroup b runs on XCD b % 8): every XCD gets a contiguous run of the
    // (image range, tile pair) list, so workgroups that share an image range, and with it their
    // operands, share an L2, and all XCDs are busy whatever the number of ranges
    const int per = g.ncg * g.nrg;
    const int wi = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    if (wi >= g.S * per) return;
    const int kr = wi / per, sub = wi - kr * per;
    const int cg = sub % g.ncg, rg = sub / g.ncg;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r32 = lane & 31, kh = lane >> 5;    // row (or channel) of the lane's fragment, its 16-byte half of the K-step
    const int kt = wave & 1, pl = (wave >> 1) & 1, ch = wave >> 2;   // row half (32 output channels), byte plane, channel half (32 input channels)

    const int zsg = qpg->zero_point - (1 << (qpg->bits - 1)), zsx = qpx->zero_point - (1 << (qpx->bits - 1));
    const uint32_t a_pad = (uint32_t)(zsg & 0xFFFF) * 0x00010001u;   // two zero codes of the gradient
    const uint32_t b_pad = (uint32_t)(zsx & 255) * 0x01010101u;

    // ---- pads, margins and halos: every byte of the buffers starts as its operand's zero code ----
    {
        const uint32_t hi4 = (uint32_t)((zsg >> 8) & 255) * 0x01010101u;
        const uint32_t lo4 = (uint32_t)((zsg & 255) ^ 0x80) * 0x01010101u;
        for (int i = tid; i < SH::SMEM / 16; i += kThreads) {
            const int o = (i * 16) % SH::BUF;
            const uint32_t v = o < KT * ROWP ? hi4 : (o < SH::A_BYTES ? lo4 : b_pad);
            *reinterpret_cast<uint4 *>(&smem[i * 16]) = make_uint4(v, v, v, v);
        }
    }

    // ---- staging plan ----
    // Staging goes by image rows.  (A 16-byte piece of the contiguous tile covers parts of several image rows at byte (7x7)
    // or 2-byte (14x14) granularity; staging by pieces, a narrow LDS store per value or pair, cost as much as the MFMAs.)
    // A thread stages whole image rows: the P values of a row and the LEADC values before them (for the
    // first row of a plane: the values behind them, shifted in registers) are one or two unaligned global loads of a
    // padded row's size, the values before the row become the pads, and a padded row goes to LDS as one aligned 8- or
    // 16-byte store per byte plane.
    // An input row at stride 2 is 2 * PT bytes (2 * LEADC of them before the row) that fall apart into the padded rows
    // of the even-column and the odd-column class of the row's parity: two byte permutes per pair of dwords.
    // Row tasks are dealt out so that a thread's tasks differ by constants only: 448 = 64 * 7 = 32 * 14 = 16 * 28 rows
    // (the rows of 64, 32 or 16 channels of one image) go to threads 0..447 per slot, and the slots walk the channel
    // groups of an image, then the images of the chunk.  One offset pair per operand describes all of a thread's tasks
    // (a table per slot cost enough registers to spill, and a reload from scratch waits for every global load in flight).
    // A 28x28 plane goes in four bands of 8 padded rows (a chunk each): 8 gradient rows x 64 channels and 16 input
    // rows x 32 channels are 512 tasks, one per thread; rows past the plane (the last band) are staged as zero codes.
    constexpr int kRowThreads = NBAND > 1 ? kThreads : 448;
    constexpr int GRB = NBAND > 1 ? KC / PT : P;                      // gradient rows per channel and chunk
    constexpr int XRB = KS == 1 ? GRB : GRB * STRIDE;                 // input rows staged per channel and chunk (1x1: the even ones)
    constexpr int G_CPS = kRowThreads / GRB, G_SPI = KT / G_CPS;      // gradient: channels per slot, slots per image
    constexpr int X_CPS = kRowThreads / XRB, X_SPI = CT / X_CPS;      // input
    static_assert(G_CPS * GRB == kRowThreads && X_CPS * XRB == kRowThreads && G_SPI * G_CPS == KT && X_SPI * X_CPS == CT, "whole groups");
    constexpr int GT = NIMG * G_SPI, XT = NIMG * X_SPI;   // row tasks per thread and chunk
    constexpr int GW = PT / 8;      // 16-byte pieces of a padded gradient row (2 * PT bytes)
    constexpr int XWB = STRIDE * PT, XW = (XWB + 15) / 16, XSB = STRIDE * LEADC;   // bytes / 16-byte pieces of an input row task, bytes before the row
    const int rt = tid < kRowThreads ? tid : tid - kRowThreads;   // the last 64 threads repeat the first 64 tasks: no thread-dependent branch
    const int gk0 = rt / GRB, gr0 = rt - gk0 * GRB, xc0 = rt / XRB, xr0 = rt - xc0 * XRB;
    // LDS byte offset of slot 0's row (the same in every band)
    const int rg_lds0 = gk0 * ROWP + LEFT + gr0 * PT;
    const int rx_lds0 = STRIDE == 1 || KS == 1
                            ? xc0 * ROWP + LEFT + xr0 * PT
                            : ((xr0 & 1) ? 2 * SH::CLSB : 0) + xc0 * ROWP + LEFT + (xr0 >> 1) * PT;   // even-column class of the row's parity
    auto rg_img = [](int i) { return i / G_SPI; };
    auto rg_lds = [&](int i) { return rg_lds0 + (i / G_SPI) * PL + (i % G_SPI) * G_CPS * ROWP; };
    auto rx_img = [](int i) { return i / X_SPI; };
    auto rx_lds = [&](int i) { return rx_lds0 + (i / X_SPI) * PL + (i % X_SPI) * X_CPS * ROWP; };
    // plane row of a task in band b (gradient) / input row; a row past the plane has nothing to load
    auto g_row = [&](int b) { return b * GRB + gr0; };
    auto x_row = [&](int b) { return (KS == 1 ? 2 : 1) * (b * XRB + xr0); };
    // byte offset in the image's tile: LEADC values (XSB bytes) before the row, but for the first row of a plane
    const int rg_off0 = (gk0 * PP + gr0 * P - (gr0 ? LEADC : 0)) * 2;                       // band 0, slot 0
    const int rx_off0 = xc0 * WW + x_row(0) * WIN - (xr0 ? XSB : 0);
    auto rg_off = [&](int i, int b) {
        if (NBAND == 1) return rg_off0 + (i % G_SPI) * G_CPS * PP * 2;
        const int r = g_row(b) < P ? g_row(b) : 0;
        return ((gk0 + (i % G_SPI) * G_CPS) * PP + r * P - (r ? LEADC : 0)) * 2;
    };
    auto rx_off = [&](int i, int b) {
        if (NBAND == 1) return rx_off0 + (i % X_SPI) * X_CPS * WW;
        const int r = x_row(b) < WIN ? x_row(b) : 0;
        return (xc0 + (i % X_SPI) * X_CPS) * WW + r * WIN - (r ? XSB : 0);
    };

    const int img0 = kr * g.ipr, img1 = min(g.N, img0 + g.ipr);
    const int units = NBAND > 1 ? (img1 - img0) * NBAND : (img1 - img0 + NIMG - 1) / NIMG;

    v16i acc[TAPS];
#pragma unroll
    for (int t = 0; t < TAPS; ++t)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[t][j] = 0;
    int rsum = 0, csum[SH::CSW];
#pragma unroll
    for (int i = 0; i < SH::CSW; ++i) csum[i] = 0;

    uint4 rgr[GT * GW], rxr[XT * XW];
    const uint4 *gsrc = reinterpret_cast<const uint4 *>(g16 + ((int64_t)img0 * g.K + rg * KT) * PP);
    const uint4 *xsrc = reinterpret_cast<const uint4 *>(x + ((int64_t)img0 * g.C + cg * CT) * WW);
    const int64_t gstep = (int64_t)g.K * PP * 2 / 16, xstep = (int64_t)g.C * WW / 16;   // 16-byte pieces per image
    int l_img = img0, l_band = 0;          // first image of the chunk that is being loaded, its band
    // The rows that write_part(., part) puts into LDS, for the chunk starting at image l_img.  Every load is issued
    // unconditionally (straight-line code lets the compiler wait for exactly the loads it needs instead of for all of
    // them): an image past the range re-reads the chunk's first image and is replaced by zero codes.  Every address
    // stays inside the tile of an image of the range.
    auto load_part = [&](int part) {
        {
#pragma unroll
            for (int i = 0; i < GT; ++i)
                if (i % NPART == part) {
                    const bool img_ok = rg_img(i) == 0 || l_img + rg_img(i) < img1;
                    const bool have = img_ok && g_row(l_band) < P;
                    const uint8_t *src = reinterpret_cast<const uint8_t *>(gsrc) + (img_ok ? rg_img(i) * gstep * 16 : 0) + rg_off(i, l_band);
#pragma unroll
                    for (int w = 0; w < GW; ++w) {
                        uint4 v;
                        __builtin_memcpy(&v, src + 16 * w, 16);
                        rgr[i * GW + w] = have ? v : make_uint4(a_pad, a_pad, a_pad, a_pad);
                    }
                }
        }
        {
#pragma unroll
            for (int i = 0; i < XT; ++i)
                if ((i + 2) % NPART == part) {
                    const bool img_ok = rx_img(i) == 0 || l_img + rx_img(i) < img1;
                    const bool have = img_ok && x_row(l_band) < WIN;
                    const uint8_t *src = reinterpret_cast<const uint8_t *>(xsrc) + (img_ok ? rx_img(i) * xstep * 16 : 0) + rx_off(i, l_band);
#pragma unroll
                    for (int w = 0; w < XW; ++w) {
                        uint4 v = make_uint4(0u, 0u, 0u, 0u);
                        if (XWB >= 16) {
                            __builtin_memcpy(&v, src + 16 * w, 16);
                        } else {
                            uint2 h;
                            __builtin_memcpy(&h, src, 8);
                            v.x = h.x;
                            v.y = h.y;
                        }
                        rxr[i * XW + w] = have ? v : make_uint4(b_pad, b_pad, b_pad, b_pad);
                    }
                }
        }
    };
    // the chunk after this one, or this one again when it is the last (its reload is never used)
    auto next_chunk = [&]() {
        if (NBAND > 1) {
            const bool last_band = l_band + 1 == NBAND;
            const bool more = !last_band || l_img + 1 < img1;
            const bool step_img = more && last_band;
            l_band = more ? (last_band ? 0 : l_band + 1) : l_band;
            gsrc += step_img ? gstep : 0;
            xsrc += step_img ? xstep : 0;
            l_img += step_img ? 1 : 0;
        } else {
            const bool more = l_img + NIMG < img1;
            gsrc += more ? NIMG * gstep : 0;
            xsrc += more ? NIMG * xstep : 0;
            l_img += more ? NIMG : 0;
        }
    };
    auto abu = [](uint32_t hi, uint32_t lo, int n) { return __builtin_amdgcn_alignbyte(hi, lo, n); };
    auto write_part = [&](int buf, int part, int band) {
        uint8_t *A = smem + buf * SH::BUF, *B = A + SH::A_BYTES;
        const bool rg_first = g_row(band) == 0, rx_first = x_row(band) == 0;
        {
#pragma unroll
            for (int i = 0; i < GT; ++i)
                if (i % NPART == part) {
                    uint32_t w[4 * GW];   // a padded row: LEADC pad values, then the P values of the row
#pragma unroll
                    for (int q = 0; q < GW; ++q) {
                        w[4 * q] = rgr[i * GW + q].x;
                        w[4 * q + 1] = rgr[i * GW + q].y;
                        w[4 * q + 2] = rgr[i * GW + q].z;
                        w[4 * q + 3] = rgr[i * GW + q].w;
                    }
                    if (rg_first) {   // loaded from the row's own start: move up by LEADC values
                        constexpr int D = LEADC / 2;   // whole dwords (LEADC = 1: half a dword)
#pragma unroll
                        for (int q = 4 * GW - 1; q > 0; --q) w[q] = LEADC == 1 ? abu(w[q], w[q - 1], 2) : (q >= D ? w[q - D] : w[q]);
                        if (LEADC == 1) w[0] = w[0] << 16;
                    }
                    if (LEADC == 1) w[0] = (w[0] & 0xFFFF0000u) | (a_pad & 0xFFFFu);
#pragma unroll
                    for (int q = 0; q < LEADC / 2; ++q) w[q] = a_pad;
                    uint32_t hi[2 * GW], lo[2 * GW];
#pragma unroll
                    for (int q = 0; q < 2 * GW; ++q) {
                        const uint32_t d0 = w[2 * q] ^ 0x00800080u, d1 = w[2 * q + 1] ^ 0x00800080u;
                        hi[q] = __builtin_amdgcn_perm(d1, d0, 0x07050301u);
                        lo[q] = __builtin_amdgcn_perm(d1, d0, 0x06040200u);
                    }
                    if (GW >= 2) {
#pragma unroll
                        for (int h = 0; h < GW / 2; ++h) {
                            *reinterpret_cast<uint4 *>(A + rg_lds(i) + 16 * h) = make_uint4(hi[4 * h], hi[4 * h + 1], hi[4 * h + 2], hi[4 * h + 3]);
                            *reinterpret_cast<uint4 *>(A + rg_lds(i) + KT * ROWP + 16 * h) = make_uint4(lo[4 * h], lo[4 * h + 1], lo[4 * h + 2], lo[4 * h + 3]);
                        }
                    } else {
                        *reinterpret_cast<uint2 *>(A + rg_lds(i)) = make_uint2(hi[0], hi[1]);
                        *reinterpret_cast<uint2 *>(A + rg_lds(i) + KT * ROWP) = make_uint2(lo[0], lo[1]);
                    }
                }
        }
        {
#pragma unroll
            for (int i = 0; i < XT; ++i)
                if ((i + 2) % NPART == part) {
                    uint32_t w[4 * XW];
#pragma unroll
                    for (int q = 0; q < XW; ++q) {
                        w[4 * q] = rxr[i * XW + q].x;
                        w[4 * q + 1] = rxr[i * XW + q].y;
                        w[4 * q + 2] = rxr[i * XW + q].z;
                        w[4 * q + 3] = rxr[i * XW + q].w;
                    }
                    constexpr int LW = XWB / 4;  // dwords loaded for the row
                    constexpr int NW = PT / 4;   // dwords of a padded row in LDS
                    if (rx_first) {   // loaded from the row's own start: move up by the bytes before a row
                        constexpr int D = XSB / 4;     // whole dwords (XSB = 1, 2: part of one)
#pragma unroll
                        for (int q = LW - 1; q > 0; --q) w[q] = XSB % 4 ? abu(w[q], w[q - 1], 4 - XSB % 4) : (q >= D ? w[q - D] : w[q]);
                        w[0] = XSB % 4 ? w[0] << (8 * (XSB % 4)) : w[0];
                    }
                    constexpr uint32_t keep = LEADC == 4 ? 0u : (LEADC == 2 ? 0xFFFF0000u : 0xFFFFFF00u);   // bytes of the first dword that are data
                    if (STRIDE == 1) {
                        w[0] = (w[0] & keep) | (b_pad & ~keep);
                        if (NW == 4) *reinterpret_cast<uint4 *>(B + rx_lds(i)) = make_uint4(w[0], w[1], w[2], w[3]);
                        else *reinterpret_cast<uint2 *>(B + rx_lds(i)) = make_uint2(w[0], w[1]);
                    } else {
                        uint32_t ev[NW], od[NW];
#pragma unroll
                        for (int q = 0; q < NW; ++q) {
                            ev[q] = __builtin_amdgcn_perm(w[2 * q + 1], w[2 * q], 0x06040200u);
                            od[q] = __builtin_amdgcn_perm(w[2 * q + 1], w[2 * q], 0x07050301u);
                        }
                        ev[0] = (ev[0] & keep) | (b_pad & ~keep);
                        od[0] = (od[0] & keep) | (b_pad & ~keep);
                        if (NBAND > 1 && KS != 1 && xr0 == XRB - 1) {
                            // the last odd input row of a band is the row above the next band: before it is overwritten, its
                            // two class rows move to the margin in front of the chunk (first band of a plane: they hold the
                            // zero codes of a row past the previous plane, or of the initial fill)
#pragma unroll
                            for (int h = 0; h < 2 * (NW / 4); ++h) {
                                const int o = rx_lds(i) + (h & 1) * SH::CLSB + 16 * (h >> 1);
                                *reinterpret_cast<uint4 *>(B + o - GRB * PT) = *reinterpret_cast<const uint4 *>(B + o);
                            }
                        }
                        if (NW >= 4) {
#pragma unroll
                            for (int h = 0; h < NW / 4; ++h) {
                                *reinterpret_cast<uint4 *>(B + rx_lds(i) + 16 * h) = make_uint4(ev[4 * h], ev[4 * h + 1], ev[4 * h + 2], ev[4 * h + 3]);
                                if (KS != 1)
                                    *reinterpret_cast<uint4 *>(B + rx_lds(i) + SH::CLSB + 16 * h) =
                                        make_uint4(od[4 * h], od[4 * h + 1], od[4 * h + 2], od[4 * h + 3]);
                            }
                        } else {
                            *reinterpret_cast<uint2 *>(B + rx_lds(i)) = make_uint2(ev[0], ev[1]);
                            if (KS != 1) *reinterpret_cast<uint2 *>(B + rx_lds(i) + SH::CLSB) = make_uint2(od[0], od[1]);
                        }
                    }
                }
        }
    };
    auto ab = [](int hi, int lo, int n) { return (int)__builtin_amdgcn_alignbyte((uint32_t)hi, (uint32_t)lo, n); };

    // Column sums: the NBV input fragments of a channel half are dealt out over the four wavefronts
    // that share them (variant 4i + (wave & 3) in slot i); each reads its fragments once more for the
    // sums (no branches in the K-step; a slot beyond the last variant repeats variant 0 and is not
    // written out).  Row sums of the gradient come from the wavefront's own fragment.
    int cs_off[SH::CSW];
#pragma unroll
    for (int i = 0; i < SH::CSW; ++i) {
        int v = 4 * i + (wave & 3);
        if (v >= NBV) v = 0;
        int cls, off;
        if (KS == 1) { cls = 0; off = 0; }
        else if (STRIDE == 1) { cls = 0; off = (v - 1) * PT; }
        else { cls = ((v >> 1) == 1 ? 0 : 2) + (v & 1); off = (v >> 1) == 0 ? -PT : 0; }
        cs_off[i] = __builtin_amdgcn_readfirstlane(cls * SH::CLSB + off);
    }

    auto read_b = [&](const uint8_t *bp, bool aligned) {
        v4i fb;
        if (aligned) {
            fb = *reinterpret_cast<const v4i *>(bp);
        } else {   // pitch 8: the vertical offset is half a fragment, two 8-byte reads
            const int2 b0 = *reinterpret_cast<const int2 *>(bp), b1 = *reinterpret_cast<const int2 *>(bp + 8);
            fb = (v4i){b0.x, b0.y, b1.x, b1.y};
        }
        return fb;
    };

    // stage: the chunk held in registers goes to the other buffer, a quarter after the fragment reads
    // of every other K-step, and the registers just written are loaded again at once with the chunk
    // after that one, so that a load has a whole chunk of MFMAs to arrive
    auto compute = [&](int buf, auto stage_tag) {
        constexpr bool stage = decltype(stage_tag)::value;
        const uint8_t *A = smem + buf * SH::BUF, *B = A + SH::A_BYTES;
        // the fragment addresses are rebuilt from the lane index in every chunk: held across the loop they were the
        // registers that spilled, and a reload from scratch waits for the global loads in flight
        int ln = lane;
        asm volatile("" : "+v"(ln));
        const uint8_t *Ar = A + (pl * KT + kt * 32 + (ln & 31)) * ROWP + LEFT + (ln >> 5) * 16;
        const uint8_t *Br = B + (ch * 32 + (ln & 31)) * ROWP + LEFT + (ln >> 5) * 16;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            v4i fa[3];   // by shift index: g[p' + 1], g[p'], g[p' - 1] (as many as the filter needs)
            {
                const uint8_t *ap = Ar + ks * 32;
                const v4i c = *reinterpret_cast<const v4i *>(ap);
                fa[1] = c;
                if (NAS >= 2) {
                    const int dp1 = *reinterpret_cast<const int *>(ap + 16);
                    fa[0] = (v4i){ab(c[1], c[0], 1), ab(c[2], c[1], 1), ab(c[3], c[2], 1), ab(dp1, c[3], 1)};
                }
                if (NAS == 3) {
                    const int dm1 = *reinterpret_cast<const int *>(ap - 4);
                    fa[2] = (v4i){ab(c[0], dm1, 3), ab(c[1], c[0], 3), ab(c[2], c[1], 3), ab(c[3], c[2], 3)};
                }
                rsum = dot4_ones(c[0], dot4_ones(c[1], dot4_ones(c[2], dot4_ones(c[3], rsum))));
            }
            if (stage && (ks & 1) == 0) {
                write_part(buf ^ 1, ks >> 1, 0);
                load_part(ks >> 1);
            }
            {
#pragma unroll
                for (int i = 0; i < SH::CSW; ++i) {
                    const v4i fb = read_b(Br + cs_off[i] + ks * 32, PT >= 16);
                    csum[i] = dot4_ones(fb[0], dot4_ones(fb[1], dot4_ones(fb[2], dot4_ones(fb[3], csum[i]))));
                }
#pragma unroll
                for (int v = 0; v < NBV; ++v) {
                    const v4i fb = read_b(Br + SH::bcls(v) * SH::CLSB + ks * 32 + SH::boff(v), PT >= 16 || SH::boff(v) == 0);
#pragma unroll
                    for (int t = 0; t < TAPS; ++t)
                        if (SH::bvar(t) == v)
                            acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[SH::ashift(t)], fb, acc[t], 0, 0, 0);
                }
            }
        }
    };

    __syncthreads();                       // the zero codes are in place
    if (SH::DB) {
        if (units > 0) {
#pragma unroll
            for (int part = 0; part < NPART; ++part) load_part(part);
            next_chunk();
#pragma unroll
            for (int part = 0; part < NPART; ++part) write_part(0, part, 0);
#pragma unroll
            for (int part = 0; part < NPART; ++part) load_part(part);
            next_chunk();
        }
        __syncthreads();
        for (int u = 0; u + 1 < units; ++u) {
            compute(u & 1, std::true_type());   // multiplies chunk u; chunk u+1: registers -> other buffer; chunk u+2: loads issued
            next_chunk();
            q8t_lds_barrier();
        }
        if (units > 0) compute((units - 1) & 1, std::false_type());
    } else {
        // one buffer: multiply, then (behind a barrier) write the chunk held in registers and load the next
        if (units > 0) {
#pragma unroll
            for (int part = 0; part < NPART; ++part) load_part(part);
            next_chunk();
        }
        for (int u = 0; u < units; ++u) {
#pragma unroll
            for (int part = 0; part < NPART; ++part) write_part(0, part, u & (NBAND - 1));   // a range is whole planes: chunk u is band u % NBAND
#pragma unroll
            for (int part = 0; part < NPART; ++part) load_part(part);
            next_chunk();
            q8t_lds_barrier();
            compute(0, std::false_type());
            q8t_lds_barrier();
        }
    }

    // ---- partial result of this image range: accumulators in register order, then the sums ----
    int *out = partial + ((int64_t)(kr * g.nrg + rg) * g.ncg + cg) * SH::PART_INTS;
#pragma unroll
    for (int t = 0; t < TAPS; ++t)
#pragma unroll
        for (int j = 0; j < 16; ++j)
            out[((((pl * 2 + kt) * 2 + ch) * TAPS + t) * 16 + j) * 64 + lane] = acc[t][j];
    // a lane holds the sum over its 16-byte half of every K-step: fold the two halves
    rsum += __shfl_xor(rsum, 32, 64);
    if (kh == 0 && ch == 0) out[SH::TILE_INTS + NBV * CT + pl * KT + kt * 32 + r32] = rsum;
#pragma unroll
    for (int i = 0; i < SH::CSW; ++i) {
        const int v = 4 * i + (wave & 3);
        const int c = csum[i] + __shfl_xor(csum[i], 32, 64);
        if (kh == 0 && v < NBV) out[SH::TILE_INTS + v * CT + ch * 32 + r32] = c;
    }
}

// int64 reduction over the image ranges + zero-point correction + dequantization.  With
// a = 256*hi + lo + (128 - zg) the gradient level minus its zero point and b = x - zx:
//   sum a*b = 256*sum(hi*x) + sum(lo*x) + (128 - zg)*colsum(x) - zx*(256*rowsum(hi) + rowsum(lo) + (128 - zg)*Kp)
// over the Kp padded positions of the range (pads contribute a = 0 and b = 0).
// A thread owns four neighbouring accumulator entries (four input channels of one output channel and tap) and walks
// its share of the image ranges with 16-byte loads, several ranges in flight; the wavefronts of a workgroup take
// interleaved subsets of the ranges and fold through LDS.  (One entry per thread and one range per wavefront, the
// first form of this kernel, spent most of its time starting workgroups: 31 -> 18 us for 256 -> 256 @14 at batch 256.)
constexpr int kFinishMaxQ = 16;
template <class SH>
__global__ __launch_bounds__(64 * kFinishMaxQ) void wgrad_planes_finish(const int *__restrict__ partial, PGeom g,
                                                                       const q8t_qparams *__restrict__ qpg,
                                                                       const q8t_qparams *__restrict__ qpx,
                                                                       float *__restrict__ dw, int64_t *__restrict__ acc_out)
{
    __shared__ int64_t fold[kFinishMaxQ][4][64];
    constexpr int TAPS = SH::TAPS, NBV = SH::NBV;
    const int sub = blockIdx.y;
    const int cg = sub % g.ncg, rg = sub / g.ncg;
    const int ln = threadIdx.x & 63, quarter = threadIdx.x >> 6, nq = blockDim.x >> 6;
    const int idx = (blockIdx.x * 64 + ln) * 4;   // ((((kt*2 + ch)*TAPS + tap)*16 + reg)*64 + lane; HALF_INTS is a multiple of 256
    const int lane = idx & 63, reg = (idx >> 6) & 15, rest = idx >> 10;
    const int tap = rest % TAPS, ch = (rest / TAPS) & 1, kt = rest / (2 * TAPS);
    // 32x32 accumulator tile: lane = column + 32 * ((row / 4) % 2), register = 4 * (row / 8) + row % 4
    const int row_l = kt * 32 + 8 * (reg >> 2) + 4 * (lane >> 5) + (reg & 3), ch_l = ch * 32 + (lane & 31);
    const int bv = SH::bvar(tap);

    const int zsg = qpg->zero_point - (1 << (qpg->bits - 1)), zsx = qpx->zero_point - (1 << (qpx->bits - 1));
    const int64_t ca = 128 - zsg;
    int64_t v[4] = {0, 0, 0, 0};
#pragma unroll 4
    for (int kr = quarter; kr < g.S; kr += nq) {
        const int *p = partial + ((int64_t)(kr * g.nrg + rg) * g.ncg + cg) * SH::PART_INTS;
        const int nimg = min(g.N, (kr + 1) * g.ipr) - kr * g.ipr;
        const int64_t Kp = (int64_t)((nimg + SH::NIMG - 1) / SH::NIMG) * SH::NBAND * KC;
        const v4i hi = *reinterpret_cast<const v4i *>(p + idx), lo = *reinterpret_cast<const v4i *>(p + SH::HALF_INTS + idx);
        const v4i csv = *reinterpret_cast<const v4i *>(p + SH::TILE_INTS + bv * CT + ch_l);
        const int64_t rsh = p[SH::TILE_INTS + NBV * CT + row_l], rsl = p[SH::TILE_INTS + NBV * CT + KT + row_l];
        const int64_t common = (int64_t)zsx * (256 * rsh + rsl + ca * Kp);
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] += 256 * (int64_t)hi[j] + (int64_t)lo[j] + ca * (int64_t)csv[j] - common;
    }
    if (nq > 1) {
#pragma unroll
        for (int j = 0; j < 4; ++j) fold[quarter][j][ln] = v[j];
        __syncthreads();
        if (quarter != 0) return;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v[j] = 0;
            for (int q = 0; q < nq; ++q) v[j] += fold[q][j][ln];
        }
    }
    const double sc = (double)(qpg->scale * qpx->scale);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t o = ((int64_t)(rg * KT + row_l) * g.C + cg * CT + ch_l + j) * TAPS + tap;
        if (acc_out) acc_out[o] = v[j];
        if (dw) dw[o] = (float)((double)v[j] * sc);
    }
}

// 0 = not served; else the result plane edge (14 or 7)
int planes_edge(const q8t_conv_desc *d)
{
    const bool k3 = d->R == 3 && d->S == 3 && d->pad == 1 && (d->stride == 1 || d->stride == 2);
    const bool k1 = d->R == 1 && d->S == 1 && d->pad == 0 && d->stride == 2;
    if (!k3 && !k1) return 0;
    if (d->H != d->W || d->K % KT || d->C % CT) return 0;
    const int P = (d->H + 2 * d->pad - d->R) / d->stride + 1;
    if ((P != 14 && P != 7 && !(P == 28 && d->stride == 2)) || d->H != P * d->stride) return 0;
    return P;
}

template <class SH>
PGeom planes_geom(const q8t_conv_desc *d)
{
    PGeom g;
    g.N = d->N; g.C = d->C; g.K = d->K;
    g.nrg = d->K / KT;
    g.ncg = d->C / CT;
    const int chunks = (d->N + SH::NIMG - 1) / SH::NIMG;
    int want = 256 / (g.nrg * g.ncg);          // one workgroup per compute unit
    if (want < 1) want = 1;
    if (want > chunks) want = chunks;
    int cpr = (chunks + want - 1) / want;      // chunks per range
    if (cpr > 511 / SH::NBAND) cpr = 511 / SH::NBAND;   // 2^14 * 256 * 511 < 2^31: the 32-bit partial sums cannot overflow
    g.ipr = cpr * SH::NIMG;
    g.S = (d->N + g.ipr - 1) / g.ipr;
    return g;
}

template <class SH>
int launch_planes(const q8t_conv_desc *d, const int16_t *g16, const q8t_qparams *qg, const int8_t *x,
                  const q8t_qparams *qx, float *dw, int64_t *acc_out, void *ws, hipStream_t st)
{
    const PGeom g = planes_geom<SH>(d);
    const int per = g.nrg * g.ncg;
    const int blocks = ((g.S * per + 7) / 8) * 8;
    static Q8tLdsOptIn optin;
    if (q8t_allow_lds(optin, (const void *)wgrad_planes<SH>, SH::SMEM) != Q8T_OK) return Q8T_ERR_HIP;
    hipLaunchKernelGGL(wgrad_planes<SH>, dim3(blocks), dim3(kThreads), SH::SMEM, st, g16, x, qg, qx, g, (int *)ws);
    Q8T_LAUNCH_CHECK();
    // wavefronts per workgroup: each walks two ranges or more (measured best: 16 wavefronts of one range each spend their time starting up)
    int nq = 1;
    while (nq < kFinishMaxQ && g.S >= 4 * nq) nq *= 2;
    hipLaunchKernelGGL(wgrad_planes_finish<SH>, dim3(SH::HALF_INTS / 256, per), dim3(64 * nq), 0, st, (const int *)ws, g, qg, qx,
                       dw, acc_out);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

template <class SH>
size_t planes_ws(const q8t_conv_desc *d)
{
    const PGeom g = planes_geom<SH>(d);
    return (size_t)g.S * g.nrg * g.ncg * SH::PART_INTS * sizeof(int);
}

}  // namespace

bool q8t_planes_wgrad_supported(const q8t_conv_desc *d, const void *g16, const void *x, const void *dw, const void *acc)
{
    const int P = planes_edge(d);
    if (!P) return false;
    return q8t_aligned(g16, 16) && q8t_aligned(x, 16) && q8t_aligned(dw, 4) && q8t_aligned(acc, 8);
}

size_t q8t_planes_wgrad_ws(const q8t_conv_desc *d)
{
    const int P = planes_edge(d);
    if (!P) return 0;
    if (P == 28) return d->R == 1 ? planes_ws<Shape<28, 2, 1>>(d) : planes_ws<Shape<28, 2>>(d);
    if (d->R == 1) return P == 14 ? planes_ws<Shape<14, 2, 1>>(d) : planes_ws<Shape<7, 2, 1>>(d);
    if (d->stride == 1) return P == 14 ? planes_ws<Shape<14, 1>>(d) : planes_ws<Shape<7, 1>>(d);
    return P == 14 ? planes_ws<Shape<14, 2>>(d) : planes_ws<Shape<7, 2>>(d);
}

int q8t_planes_wgrad(const q8t_conv_desc *d, const int16_t *g16, const q8t_qparams *qg, const int8_t *x,
                     const q8t_qparams *qx, float *dw, int64_t *acc_out, void *ws, hipStream_t st)
{
    if (!ws || !q8t_aligned(ws, 16)) return Q8T_ERR_WORKSPACE;
    const int P = planes_edge(d);
    if (!P) return Q8T_ERR_SHAPE;
    if (P == 28)
        return d->R == 1 ? launch_planes<Shape<28, 2, 1>>(d, g16, qg, x, qx, dw, acc_out, ws, st)
                         : launch_planes<Shape<28, 2>>(d, g16, qg, x, qx, dw, acc_out, ws, st);
    if (d->R == 1)
        return P == 14 ? launch_planes<Shape<14, 2, 1>>(d, g16, qg, x, qx, dw, acc_out, ws, st)
                       : launch_planes<Shape<7, 2, 1>>(d, g16, qg, x, qx, dw, acc_out, ws, st);
    if (d->stride == 1)
        return P == 14 ? launch_planes<Shape<14, 1>>(d, g16, qg, x, qx, dw, acc_out, ws, st)
                       : launch_planes<Shape<7, 1>>(d, g16, qg, x, qx, dw, acc_out, ws, st);
    return P == 14 ? launch_planes<Shape<14, 2>>(d, g16, qg, x, qx, dw, acc_out, ws, st)
                   : launch_planes<Shape<7, 2>>(d, g16, qg, x, qx, dw, acc_out, ws, st);
}
