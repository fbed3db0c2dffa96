// Specialised int8 implicit-GEMM convolution for the ResNet hot shapes: stride 1, 3x3 pad 1 or
// 1x1 pad 0, channel counts that are multiples of 64 (forward, and the layer gradient, which for
// stride 1 is the same convolution with the filter flipped and its channel roles swapped;
// Section 4, eq. (grad_layer)).
//
// GEMM view: rows = flattened (image, y, x) output positions, cols = output channels,
// reduction = (tap, input channel); one MFMA K-step (v_mfma_i32_16x16x64_i8) = one filter tap over
// 64 input channels.  Persistent workgroups of 8 wavefronts own contiguous row ranges and walk them
// in sub-tiles of 256 rows x 64 output channels (two 16-row m-tiles per wavefront), the next
// sub-tile's activations prefetched into registers while the current one is multiplied.
//
// Data movement (64-channel layers move 1 byte in and 4 bytes out per element; what bounds the
// kernel in practice is instruction issue: staging, transposition and epilogue outweigh the MFMAs):
//  * activations are NCHW int8, but MFMA wants the reduction index contiguous per lane, so the
//    tile (with its halo) is transposed on the way into LDS: each lane loads 16 positions x 4
//    channels as four 16-byte loads, transposes 4x4 bytes with v_perm and writes
//    [position][channel] rows of 80 bytes (64 + 16 pad: conflict-free ds_read_b128 fragments);
//  * LDS rows use padded coordinates: one row holding the operand's zero point after every image row
//    and between images, so a tap is a constant row offset and padding needs no per-lane masks
//    (a padded tap contributes exactly nothing to the corrected accumulator);
//  * weights are repacked once per call into [tap][out-channel][in-channel] (and their per-channel
//    sums taken) by a small pre-pass; row sums of A come from one extra MFMA per m-tile and tap
//    against an all-ones operand, which delivers them in the accumulator layout.  Epilogue:
//    zero-point correction, dequantization, float4 stores (4 consecutive positions of one output
//    channel per lane); the STATS variant also folds the exact integer sum / min / max per channel.
#include <type_traits>

#include "q8t_common.h"
#include "q8t_internal.h"
#include "repack.h"

namespace {

constexpr int BM_ROWS = 256;

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kThreads = 512;     // 8 wavefronts: two 16-row m-tiles each per sub-tile
constexpr int kWaves = kThreads / 64;
constexpr int MT = BM_ROWS / 16 / kWaves;   // m-tiles per wavefront
constexpr int BM = BM_ROWS;          // rows per sub-tile
constexpr int CH = 64;           // channels per reduction chunk / output channels per workgroup
constexpr int ROWB = 80;         // LDS bytes per staged activation row (64 + 16: conflict-free b128 reads)
constexpr int MAXR9 = 464;       // staged rows (padded coordinates) of the 3x3 variant
constexpr int MAXR1 = BM;        // 1x1 variant: no halo, no padding
constexpr int MAX_SLABS = 4;     // staging iterations per wavefront (28 slabs of 64 lanes at most)
constexpr int kSkip = -1000000;  // marks a staging slot with nothing to store
constexpr int MARGIN = 20;       // spare LDS rows on either side of the staged rows: a staging lane whose group of
                                 // positions hangs over the staged range stores there instead of testing every row

struct FastDiv {
    uint32_t d;
    float r;
};

struct FastGeom {
    int N, C, K;      // images, reduction channels, output channels
    int H, W, PQ;     // plane
    int M;            // N * PQ (< 2^31)
    FastDiv dPQ, dW, dIMG, dW1;
};

// quotient of n / d for quotients below 2^16 (image index, row index): float estimate + fix-up
__device__ __forceinline__ uint32_t fdiv(uint32_t n, const FastDiv fd)
{
    uint32_t q = (uint32_t)((float)n * fd.r);
    const int32_t rem = (int32_t)(n - q * fd.d);
    if (rem < 0) --q;
    else if ((uint32_t)rem >= fd.d) ++q;
    return q;
}
template <int D>
__device__ __forceinline__ uint32_t divc(uint32_t n, const FastDiv fd)
{
    if (D > 0) return n / (uint32_t)(D > 0 ? D : 1);
    return fdiv(n, fd);
}

// ---- weight pre-pass: repack + per-output-channel sums (layout and body: repack.h) --------------
__global__ __launch_bounds__(kRepackThreads) void repack_weights(const int8_t *__restrict__ w, int Kf, int Cf, int R,
                                                           int S, int dgrad, int8_t *__restrict__ out,
                                                           int *__restrict__ colsum)
{
    __shared__ int red[kRepackThreads / 64];
    q8t_repack_tile64(w, Kf, Cf, R, S, dgrad, out, colsum, (int)blockIdx.x, red);
}

// 4x4 byte transpose: in[j] = 4 consecutive positions of channel j; out[i] = 4 channels of position i
__device__ __forceinline__ void transpose4x4(const uint32_t in[4], uint32_t out[4])
{
    // v_perm_b32(hi, lo, sel): bytes 0-3 index lo, 4-7 index hi
    const uint32_t t0 = __builtin_amdgcn_perm(in[1], in[0], 0x05010400);  // a0 b0 a1 b1
    const uint32_t t1 = __builtin_amdgcn_perm(in[1], in[0], 0x07030602);  // a2 b2 a3 b3
    const uint32_t t2 = __builtin_amdgcn_perm(in[3], in[2], 0x05010400);  // c0 d0 c1 d1
    const uint32_t t3 = __builtin_amdgcn_perm(in[3], in[2], 0x07030602);  // c2 d2 c3 d3
    out[0] = __builtin_amdgcn_perm(t2, t0, 0x05040100);                    // a0 b0 c0 d0
    out[1] = __builtin_amdgcn_perm(t2, t0, 0x07060302);                    // a1 b1 c1 d1
    out[2] = __builtin_amdgcn_perm(t3, t1, 0x05040100);
    out[3] = __builtin_amdgcn_perm(t3, t1, 0x07060302);
}

__device__ __forceinline__ int dot4_ones(int v, int acc) { return __builtin_amdgcn_sdot4(v, 0x01010101, acc, false); }

// Persistent workgroups: each owns one contiguous range of output rows (a multiple of 16) and walks
// it in sub-tiles of 256 rows.  Consecutive workgroup ids go round-robin over the 8 XCDs, so the
// ranges are dealt out such that each XCD works on one contiguous stretch of the tensor
// (neighbouring ranges share halo rows, and then an L2).
typedef Q8tConvStat ConvStat;

struct Sched {
    int nbx;          // workgroups along the rows (multiple of 8)
    int rpb;          // rows per workgroup (multiple of 16)
    int halo_al;      // real positions staged on either side of a sub-tile (multiple of 4)
    int pg_blocks;    // ceil((BM + 2*halo_al)/4 / 16)
    int maxr;         // LDS rows a sub-tile can touch (padded coordinates)
};

// Padded coordinates (3x3 only).  Inside LDS the staged positions are laid out with one extra
// row after every image row and one extra image row between images, all holding the operand's
// zero point:  A(b,p,q) = b*(H+1)*(W+1) + (p+1)*(W+1) + q.  A filter tap is then the constant
// row offset dr*(W+1) + ds for every output position, borders included -- no per-lane masks.
// WC > 0 fixes a square image size at compile time (cheap index arithmetic, immediate offsets).
template <int TAPS, int WC, bool V16, bool STATS, bool FUSE>
__global__ __launch_bounds__(kThreads, 4) void conv_s1_kernel(const int8_t *__restrict__ x,
                                                              const int8_t *__restrict__ wpk,
                                                              const int *__restrict__ colsum,
                                                              const q8t_qparams *__restrict__ qpa,
                                                              const q8t_qparams *__restrict__ qpb,
                                                              const FastGeom g, const Sched sch,
                                                              float *__restrict__ y, int32_t *__restrict__ acc_out,
                                                              ConvStat *__restrict__ bnpart, const Q8tReluSum fuse)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    // per-channel statistics of this workgroup's outputs (integer accumulators: exact, order-free)
    __shared__ unsigned long long st_sum[STATS ? CH : 1];
    __shared__ int st_min[STATS ? CH : 1], st_max[STATS ? CH : 1];
    constexpr int A_BYTES = ((TAPS == 9 ? MAXR9 : MAXR1) + 2 * MARGIN) * ROWB;
    constexpr int B_PIECES = TAPS * CH * 4;            // 16-byte pieces of the weight chunk
    constexpr int B_VEC = (B_PIECES + kThreads - 1) / kThreads;
    constexpr int PQC = WC * WC, W1C = (TAPS == 9 && WC) ? WC + 1 : WC, IMGC = (TAPS == 9 && WC) ? (WC + 1) * (WC + 1) : PQC;
    uint8_t *As = smem + MARGIN * ROWB;
    uint8_t *Bs = smem + A_BYTES;

    const int W = WC ? WC : g.W, PQ = WC ? PQC : g.PQ;
    const int W1 = (TAPS == 9) ? W + 1 : W;
    const int IMG = WC ? IMGC : (int)g.dIMG.d;

    const int bidx = (blockIdx.x & 7) * (sch.nbx >> 3) + (blockIdx.x >> 3);
    const int row_begin = bidx * sch.rpb;
    const int row_end = min(g.M, row_begin + sch.rpb);
    if (row_begin >= row_end) return;
    const int occ = blockIdx.y;  // output-channel chunk
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (STATS && tid < CH) {
        st_sum[tid] = 0ull;
        st_min[tid] = 2147483647;
        st_max[tid] = -2147483647 - 1;
    }
    const int l16 = lane & 15, kb = lane >> 4;

    const int za = qpa->zero_point - (1 << (qpa->bits - 1)), zb = qpb->zero_point - (1 << (qpb->bits - 1));
    const float sc = qpa->scale * qpb->scale;
    const uint32_t zavec = (uint32_t)(za & 255) * 0x01010101u;

    // padded coordinate of a real row index
    auto apad = [&](uint32_t gr) -> int {
        if (TAPS != 9) return (int)gr;
        const uint32_t b = divc<PQC>(gr, g.dPQ);
        const uint32_t pos = gr - b * PQ;
        const uint32_t p = divc<WC>(pos, g.dW);
        return (int)(b * IMG + pos + p + W1);
    };

    const int CC = g.C / CH;
    // The first sub-tile is shorter by a workgroup-dependent amount, so that the workgroups of a
    // compute unit (and of the chip) are in different phases (load / MFMA / store) at any moment
    // instead of marching in lock-step and using the memory system in bursts.
    const int stag = ((blockIdx.x >> 3) + (blockIdx.x >> 8)) & 3;
    const int len0 = min(row_end - row_begin, 64 * (1 + stag));
    const int nsub = 1 + (row_end - row_begin - len0 + BM - 1) / BM;
    const int nsteps = nsub * CC;
    auto tile_begin = [&](int sub) { return row_begin + (sub == 0 ? 0 : len0 + (sub - 1) * BM); };
    auto tile_end = [&](int sub) { return sub == 0 ? row_begin + len0 : min(row_end, tile_begin(sub) + BM); };
    const int npg = (BM + 2 * sch.halo_al) >> 2;

    // ---- register prefetch of the next step's operands ----
    uint32_t pa[MAX_SLABS][4];
    int prow[MAX_SLABS], pthr[MAX_SLABS];   // LDS row of the group's first position (kSkip: nothing), straddle point
    uint4 pq[4];                            // wide staging variant: 4 channels x 16 positions
    auto prefetch = [&](int step) {
        const int sub = step / CC, cc = step - sub * CC;
        const int g0 = tile_begin(sub);
        const int a0 = apad((uint32_t)g0) - ((TAPS == 9) ? W1 + 1 : 0);   // padded coordinate of LDS row 0
        const int stage = tile_end(sub) - g0 + 2 * sch.halo_al;           // real positions to stage
        if (V16) {
            // wide variant: one lane = 16 positions x 4 channels, four 16-byte loads.  The vector
            // memory pipeline takes about as long for a 4-byte as for a 16-byte access per lane,
            // so this issues a quarter of the load instructions.  lane -> channel group (l16),
            // (wavefront, kb) -> group of 16 positions: 64-byte segments per channel plane.
            const int pg16 = wave * 4 + kb, cg = l16;
            const int gr = g0 - sch.halo_al + pg16 * 16;
            prow[0] = kSkip;
            if (pg16 * 16 < stage && gr >= 0 && gr < g.M) {
                const uint32_t b = divc<PQC>((uint32_t)gr, g.dPQ);
                const uint32_t pos = (uint32_t)gr - b * PQ;
                int r = gr - g0;
                pthr[0] = 0;
                if (TAPS == 9) {
                    const uint32_t p = divc<WC>(pos, g.dW);
                    r = (int)(b * IMG + pos + p + W1) - a0;
                    pthr[0] = (int)(pos - p * W);   // column of the first position
                }
                if (r > -20 && r < sch.maxr) {
                    prow[0] = r;
                    const int8_t *src = x + ((size_t)(b * g.C + cc * CH + cg * 4) * PQ + pos);
#pragma unroll
                    for (int j = 0; j < 4; ++j) pq[j] = *reinterpret_cast<const uint4 *>(src + (size_t)j * PQ);
                }
            }
        } else
#pragma unroll
        for (int it = 0; it < MAX_SLABS; ++it) {
            // one wavefront instruction = 16 position groups x 4 channel groups: 64-byte global
            // segments per channel, 16 distinct LDS banks per transposed store
            const int slab = wave + it * (kThreads / 64);
            const int pgb = slab % sch.pg_blocks, cgb = slab / sch.pg_blocks;
            const int pg = pgb * 16 + l16, cg = cgb * 4 + kb;
            const int gr = g0 - sch.halo_al + pg * 4;
            prow[it] = kSkip;
            pthr[it] = 4;
            if (cgb < 4 && pg * 4 < stage && gr >= 0 && gr < g.M) {
                const uint32_t b = divc<PQC>((uint32_t)gr, g.dPQ);
                const uint32_t pos = (uint32_t)gr - b * PQ;
                int r = gr - g0;
                if (TAPS == 9) {
                    const uint32_t p = divc<WC>(pos, g.dW);
                    r = (int)(b * IMG + pos + p + W1) - a0;
                    pthr[it] = W - 1 - (int)(pos - p * W);   // positions after this one sit one row further
                }
                if (r > -4 && r < sch.maxr) {   // rows outside [0, maxr) land in the spare rows
                    prow[it] = r;
                    const int8_t *src = x + ((size_t)(b * g.C + cc * CH + cg * 4) * PQ + pos);
#pragma unroll
                    for (int j = 0; j < 4; ++j) pa[it][j] = *reinterpret_cast<const uint32_t *>(src + (size_t)j * PQ);
                }
            }
        }
    };
    auto commit = [&](int step) {
        if (V16) {
            if (prow[0] != kSkip) {
                const int cg = l16;
#pragma unroll
                for (int j4 = 0; j4 < 4; ++j4) {
                    const uint32_t in[4] = {j4 == 0 ? pq[0].x : j4 == 1 ? pq[0].y : j4 == 2 ? pq[0].z : pq[0].w,
                                            j4 == 0 ? pq[1].x : j4 == 1 ? pq[1].y : j4 == 2 ? pq[1].z : pq[1].w,
                                            j4 == 0 ? pq[2].x : j4 == 1 ? pq[2].y : j4 == 2 ? pq[2].z : pq[2].w,
                                            j4 == 0 ? pq[3].x : j4 == 1 ? pq[3].y : j4 == 2 ? pq[3].z : pq[3].w};
                    uint32_t out[4];
                    transpose4x4(in, out);
                    // positions 4*j4 .. 4*j4+3 lie in one image row (W % 4 == 0); every row end
                    // passed since the first position shifts the LDS row by one (the pad row)
                    int bump = 0;
                    if (TAPS == 9) {
                        const int col = pthr[0] + 4 * j4;
                        bump = (col >= W) + (col >= 2 * W) + (col >= 3 * W) + (col >= 4 * W);
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int row = prow[0] + 4 * j4 + i + bump;   // in (-MARGIN, maxr + MARGIN)
                        *reinterpret_cast<uint32_t *>(&As[row * ROWB + cg * 4]) = out[i];
                    }
                }
            }
        } else
#pragma unroll
        for (int it = 0; it < MAX_SLABS; ++it) {
            if (prow[it] != kSkip) {
                const int cg = ((wave + it * (kThreads / 64)) / sch.pg_blocks) * 4 + kb;
                uint32_t out[4];
                transpose4x4(pa[it], out);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int row = prow[it] + i + ((TAPS == 9 && i > pthr[it]) ? 1 : 0);   // in (-4, maxr + 4)
                    *reinterpret_cast<uint32_t *>(&As[row * ROWB + cg * 4]) = out[i];
                }
            }
        }
        if (TAPS == 9) {
            // zero-point rows: the pad column after every image row and the pad row between images
            const int sub = step / CC;
            const int g0 = tile_begin(sub);
            const int a0 = apad((uint32_t)g0) - (W1 + 1);
            for (int rr = tid; rr < sch.maxr; rr += kThreads) {
                const int ac = a0 + rr;
                bool pad = ac < 0;
                if (!pad) {
                    const uint32_t bi = divc<IMGC>((uint32_t)ac, g.dIMG);
                    const uint32_t rem = (uint32_t)ac - bi * IMG;
                    const uint32_t ri = divc<W1C>(rem, g.dW1);
                    pad = (ri == 0) || (rem - ri * W1 == (uint32_t)W);
                }
                if (pad) {
                    const uint4 z = make_uint4(zavec, zavec, zavec, zavec);
#pragma unroll
                    for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4 *>(&As[rr * ROWB + i * 16]) = z;
                }
            }
        }
    };
    // weights of (occ, cc): [tap][64 oc][64 ch] from the packed copy (L2-resident) into LDS.
    // 16-byte pieces; the 4 pieces of a row are XOR-swizzled by bits 1..2 of the row, which keeps the
    // b128 fragment reads of 16 consecutive rows conflict-free (a 16-byte LDS read is served in
    // phases of lanes {0-3, 12-15, 20-23, 24-27}, ...: see gemm_core.h)
    auto stage_b = [&](int cc) {
        const int8_t *src = wpk + (size_t)(occ * CC + cc) * TAPS * CH * CH;
#pragma unroll
        for (int i = 0; i < B_VEC; ++i) {
            const int e = tid + i * kThreads, row = e >> 2, part = e & 3;
            if (e < B_PIECES)
                *reinterpret_cast<uint4 *>(&Bs[row * CH + ((part ^ ((row >> 1) & 3)) << 4)]) =
                    *reinterpret_cast<const uint4 *>(src + (size_t)e * 16);
        }
    };

    v4i acc[MT][4], accrs[MT];
    int abase[MT];
    v4i ones = (v4i){0x01010101, 0x01010101, 0x01010101, 0x01010101};
    asm volatile("" : "+v"(ones));   // opaque: kept in four registers instead of being rebuilt before every use
    const int bbase = l16 * CH + ((kb ^ ((l16 >> 1) & 3)) << 4);

    prefetch(0);
    for (int step = 0; step < nsteps; ++step) {
        const int sub = step / CC, cc = step - sub * CC;
        const int g0 = tile_begin(sub), g1 = tile_end(sub);
        const bool with_b = (CC > 1) || (step == 0);
        q8t_lds_barrier();
        commit(step);
        if (with_b) stage_b(cc);
        q8t_lds_barrier();
        if (step + 1 < nsteps) prefetch(step + 1);

        if (cc == 0) {
            const int ag0 = apad((uint32_t)g0);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = (v4i){0, 0, 0, 0};
                accrs[mt] = (v4i){0, 0, 0, 0};
                // LDS address of this lane's A row in m-tile (mt*4 + wave), before the tap offset
                int gr = g0 + (mt * kWaves + wave) * 16 + l16;
                if (gr >= g.M) gr = g0;
                abase[mt] = (apad((uint32_t)gr) - ag0) * ROWB + kb * 16;
            }
        }
        // ---- MFMA: one K-step per tap, plus an all-ones column tile that yields the row sums of A
        // in the accumulator layout.  M-tiles are interleaved over the wavefronts so that a ragged
        // last sub-tile stays balanced ----
#pragma unroll
        for (int tap = 0; tap < TAPS; ++tap) {
            const int toff = (TAPS == 9) ? ((tap / 3) * W1 + (tap % 3)) * ROWB : 0;
            v4i bf[4];
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
                bf[nt] = *reinterpret_cast<const v4i *>(&Bs[bbase + (tap * CH + nt * 16) * CH]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                if (g0 + (mt * kWaves + wave) * 16 >= g1) continue;   // wavefront-uniform
                const v4i a = *reinterpret_cast<const v4i *>(&As[abase[mt] + toff]);
#pragma unroll
                for (int nt = 0; nt < 4; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, bf[nt], acc[mt][nt], 0, 0, 0);
                accrs[mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, ones, accrs[mt], 0, 0, 0);
            }
        }
        if (cc != CC - 1) continue;

        // ---- epilogue: zero-point correction (wrapping 32-bit arithmetic: the corrected value fits
        // by contract), dequantization, 4 consecutive positions of one output channel per lane ----
        const uint32_t Kp = (uint32_t)(g.C * TAPS);
        const uint32_t kzz = Kp * (uint32_t)za * (uint32_t)zb;
        uint32_t ncs[4];   // minus the column term, so that a correction is one three-operand add
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) ncs[nt] = 0u - (uint32_t)za * (uint32_t)colsum[occ * CH + nt * 16 + l16];
        // FLOAT_ONLY: the usual call (float result, no integer copy) without the two pointer tests per store
        auto emit = [&](auto float_only) {
        constexpr bool FLOAT_ONLY = decltype(float_only)::value;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int gr = g0 + (mt * kWaves + wave) * 16 + kb * 4;
            if (gr >= g1) continue;
            const uint32_t b = divc<PQC>((uint32_t)gr, g.dPQ);
            const uint32_t pos = (uint32_t)gr - b * PQ;
            uint32_t t[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) t[j] = kzz - (uint32_t)zb * (uint32_t)accrs[mt][j];
            const size_t o0 = (size_t)(b * g.K + occ * CH + l16) * PQ + pos;
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                const size_t o = o0 + (size_t)(nt * 16) * PQ;
                const int c0 = (int)((uint32_t)acc[mt][nt][0] + t[0] + ncs[nt]);
                const int c1 = (int)((uint32_t)acc[mt][nt][1] + t[1] + ncs[nt]);
                const int c2 = (int)((uint32_t)acc[mt][nt][2] + t[2] + ncs[nt]);
                const int c3 = (int)((uint32_t)acc[mt][nt][3] + t[3] + ncs[nt]);
                if (STATS) {
                    // every lane adds its 4 rows straight into the workgroup's LDS slots (4 lanes per
                    // channel collide; cheaper than folding them first through cross-lane moves, which
                    // occupy the same LDS pipe)
                    atomicAdd(&st_sum[nt * 16 + l16], (unsigned long long)((long long)c0 + c1 + c2 + c3));
                    atomicMin(&st_min[nt * 16 + l16], min(min(c0, c1), min(c2, c3)));
                    atomicMax(&st_max[nt * 16 + l16], max(max(c0, c1), max(c2, c3)));
                }
                if (!FLOAT_ONLY && acc_out) *reinterpret_cast<int4 *>(acc_out + o) = make_int4(c0, c1, c2, c3);
                if (FLOAT_ONLY || y) {
                    float4 f;
                    f.x = sc * (float)c0;
                    f.y = sc * (float)c1;
                    f.z = sc * (float)c2;
                    f.w = sc * (float)c3;
                    *reinterpret_cast<float4 *>(y + o) = f;
                }
            }
        }
        };
        // With the end of a residual block in the epilogue (relu_sum.h) the two extra operands of a store are loaded one
        // store ahead: a load issued only where its value is needed would put a full memory latency in front of every store.
        auto emit_fused = [&]() {
            size_t ob[MT];
            bool live[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const int gr = g0 + (mt * kWaves + wave) * 16 + kb * 4;
                live[mt] = gr < g1;
                const uint32_t b = divc<PQC>((uint32_t)(live[mt] ? gr : 0), g.dPQ);
                const uint32_t pos = (uint32_t)(live[mt] ? gr : 0) - b * PQ;
                ob[mt] = (size_t)(b * g.K + occ * CH + l16) * PQ + pos;
            }
            float4 nx_o = make_float4(0.0f, 0.0f, 0.0f, 0.0f), nx_a = nx_o;
            auto fetch = [&](size_t o) {
                nx_a = *reinterpret_cast<const float4 *>(fuse.act + o);
                if (fuse.other) nx_o = *reinterpret_cast<const float4 *>(fuse.other + o);
            };
            if (live[0]) fetch(ob[0]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                if (!live[mt]) continue;
                uint32_t t[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) t[j] = kzz - (uint32_t)zb * (uint32_t)accrs[mt][j];
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) {
                    const size_t o = ob[mt] + (size_t)(nt * 16) * PQ;
                    const float4 cu_o = nx_o, cu_a = nx_a;
                    if (nt < 3) fetch(o + (size_t)16 * PQ);
                    else if (mt + 1 < MT && live[mt + 1 < MT ? mt + 1 : mt]) fetch(ob[mt + 1 < MT ? mt + 1 : mt]);
                    float4 f;
                    f.x = sc * (float)(int)((uint32_t)acc[mt][nt][0] + t[0] + ncs[nt]);
                    f.y = sc * (float)(int)((uint32_t)acc[mt][nt][1] + t[1] + ncs[nt]);
                    f.z = sc * (float)(int)((uint32_t)acc[mt][nt][2] + t[2] + ncs[nt]);
                    f.w = sc * (float)(int)((uint32_t)acc[mt][nt][3] + t[3] + ncs[nt]);
                    if (fuse.other) {
                        f.x = f.x + cu_o.x;
                        f.y = f.y + cu_o.y;
                        f.z = f.z + cu_o.z;
                        f.w = f.w + cu_o.w;
                    }
                    f.x = cu_a.x > 0.0f ? f.x : 0.0f;
                    f.y = cu_a.y > 0.0f ? f.y : 0.0f;
                    f.z = cu_a.z > 0.0f ? f.z : 0.0f;
                    f.w = cu_a.w > 0.0f ? f.w : 0.0f;
                    *reinterpret_cast<float4 *>(y + o) = f;
                }
            }
        };
        if (FUSE) emit_fused();
        else if (y && !acc_out) emit(std::true_type{});
        else emit(std::false_type{});
    }
    if (STATS) {
        __syncthreads();
        if (tid < CH) {
            ConvStat r;
            r.sum = (long long)st_sum[tid];
            r.mn = st_min[tid];
            r.mx = st_max[tid];
            bnpart[((size_t)occ * sch.nbx + bidx) * CH + tid] = r;
        }
    }
}

// statistics of the float outputs from the integer partials: stats[0][k] = mean, [1] = min, [2] = max
// with y = scale * (float)acc as in the epilogue above (so min / max are bit-identical to a scan of y)
__global__ __launch_bounds__(256) void conv_stats_finalize(const ConvStat *__restrict__ bnpart, int K, int nbx, int nact,
                                                           double n, const q8t_qparams *__restrict__ qpa,
                                                           const q8t_qparams *__restrict__ qpb, float *__restrict__ stats)
{
    // one workgroup per output channel; its threads share the workgroups of the convolution
    __shared__ long long ssum[4];
    __shared__ int smn[4], smx[4];
    const int k = blockIdx.x;
    const int occ = k / CH, ch = k - occ * CH;
    long long s = 0;
    int mn = 2147483647, mx = -2147483647 - 1;
    for (int b = threadIdx.x; b < nact; b += 256) {
        const ConvStat r = bnpart[((size_t)occ * nbx + b) * CH + ch];
        s += r.sum;
        mn = min(mn, r.mn);
        mx = max(mx, r.mx);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        s += __shfl_xor(s, off, 64);
        mn = min(mn, __shfl_xor(mn, off, 64));
        mx = max(mx, __shfl_xor(mx, off, 64));
    }
    if ((threadIdx.x & 63) == 0) {
        ssum[threadIdx.x >> 6] = s;
        smn[threadIdx.x >> 6] = mn;
        smx[threadIdx.x >> 6] = mx;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        s = ssum[0] + ssum[1] + ssum[2] + ssum[3];
        mn = min(min(smn[0], smn[1]), min(smn[2], smn[3]));
        mx = max(max(smx[0], smx[1]), max(smx[2], smx[3]));
        const float sc = qpa->scale * qpb->scale;
        stats[k] = (float)((double)sc * (double)s / n);
        stats[K + k] = sc * (float)mn;
        stats[2 * K + k] = sc * (float)mx;
    }
}

template <int TAPS>
constexpr size_t smem_bytes()
{
    return (size_t)((TAPS == 9 ? MAXR9 : MAXR1) + 2 * MARGIN) * ROWB + (size_t)TAPS * CH * CH;
}

// LDS rows (padded coordinates) one sub-tile can touch
int rows_needed(int taps, int W, int PQ)
{
    if (taps != 9) return BM;
    const int W1 = W + 1;
    return (BM - 1) + (BM + W - 1) / W + W1 * (BM / PQ + 1) + 2 * W1 + 8;
}

bool shape_ok(int which, const q8t_conv_desc *d)
{
    if (which > 1) return false;
    if (d->stride != 1 || d->R != d->S) return false;
    if (!((d->R == 3 && d->pad == 1) || (d->R == 1 && d->pad == 0))) return false;
    if (d->C % CH || d->K % CH) return false;
    if ((d->H * d->W) % 4) return false;
    if (d->H < 2 || d->W < 2 || d->N > 32768 || d->H > 32768) return false;   // quotient range of fdiv
    if (d->R == 3 && (rows_needed(9, d->W, d->H * d->W) > MAXR9 || ((d->W + 1 + 3) & ~3) * 2 + BM > MAX_SLABS * kWaves / 4 * 64))
        return false;
    return true;
}

FastDiv mkdiv(int d)
{
    FastDiv f;
    f.d = (uint32_t)d;
    f.r = 1.0f / (float)d;
    return f;
}

}  // namespace

int q8t_conv_stats_finalize(const Q8tConvStat *part, int K, int nbx, int nact, double n, const q8t_qparams *qa,
                            const q8t_qparams *qb, float *stats, hipStream_t st)
{
    hipLaunchKernelGGL(conv_stats_finalize, dim3((unsigned)K), dim3(256), 0, st, part, K, nbx, nact, n, qa, qb, stats);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

bool q8t_fast_conv_supported(int which, const q8t_conv_desc *d, const void *a, const void *b, const void *out_f,
                             const void *out_acc)
{
    if (!shape_ok(which, d)) return false;
    (void)b;
    return q8t_aligned(a, 4) && q8t_aligned(out_f, 16) && q8t_aligned(out_acc, 16);
}

size_t q8t_fast_conv_ws(int which, const q8t_conv_desc *d)
{
    if (!shape_ok(which, d)) return 0;
    const size_t wbytes = (size_t)d->K * d->C * d->R * d->S;
    const int oc = which == 0 ? d->K : d->C;
    // packed filter, column sums, per-workgroup statistics (at most 512 workgroups per channel chunk)
    return ((wbytes + 255) & ~(size_t)255) + (((size_t)oc * sizeof(int) + 255) & ~(size_t)255) +
           (size_t)oc * 512 * sizeof(ConvStat);
}

template <int TAPS, int WC, bool V16, bool STATS, bool FUSE>
int launch_conv(dim3 grid, hipStream_t st, const int8_t *a, const int8_t *wpk, const int *colsum,
                const q8t_qparams *qa, const q8t_qparams *qb, const FastGeom &g, const Sched &sch, float *out_f,
                int32_t *out_acc, ConvStat *bnpart, const Q8tReluSum &fuse)
{
    static Q8tLdsOptIn optin;
    if (smem_bytes<TAPS>() > 65536 &&
        q8t_allow_lds(optin, (const void *)conv_s1_kernel<TAPS, WC, V16, STATS, FUSE>, smem_bytes<TAPS>()) != Q8T_OK)
        return Q8T_ERR_HIP;
    hipLaunchKernelGGL((conv_s1_kernel<TAPS, WC, V16, STATS, FUSE>), grid, dim3(kThreads), smem_bytes<TAPS>(), st, a, wpk, colsum, qa,
                       qb, g, sch, out_f, out_acc, bnpart, fuse);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

int q8t_fast_conv(int which, const q8t_conv_desc *d, const void *a, const q8t_qparams *qa, const void *b,
                  const q8t_qparams *qb, float *out_f, void *out_acc, float *bn_stats, void *ws, hipStream_t st,
                  const Q8tReluSum *relu_sum, const void *packed)
{
    if (!ws || !q8t_aligned(ws, 16)) return Q8T_ERR_WORKSPACE;
    if (packed && !q8t_aligned(packed, 16)) return Q8T_ERR_WORKSPACE;
    Q8tReluSum fuse = {nullptr, nullptr};
    if (relu_sum) {
        if (bn_stats || which != 1) return Q8T_ERR_SHAPE;
        if (!out_f || !q8t_aligned(relu_sum->act, 16) || !q8t_aligned(relu_sum->other, 16)) return Q8T_ERR_SHAPE;
        fuse = *relu_sum;
    }
    const int taps = d->R * d->S;
    const size_t wbytes = (size_t)d->K * d->C * taps;
    const int oc_all = which == 0 ? d->K : d->C;
    // the packed filter and its column sums: made here in the workspace, or handed in (q8t_qconv_pack_multi)
    int8_t *wpk = packed ? (int8_t *)packed : (int8_t *)ws;
    int *colsum = (int *)((char *)wpk + ((wbytes + 255) & ~(size_t)255));
    ConvStat *bnpart = bn_stats ? (ConvStat *)((char *)ws + ((wbytes + 255) & ~(size_t)255) +
                                               (((size_t)oc_all * sizeof(int) + 255) & ~(size_t)255))
                                : (ConvStat *)nullptr;
    int rc = 0;
    FastGeom g;
    g.N = d->N;
    g.H = d->H;
    g.W = d->W;
    g.PQ = d->H * d->W;
    g.C = which == 0 ? d->C : d->K;   // reduction channels
    g.K = which == 0 ? d->K : d->C;   // output channels
    g.M = g.N * g.PQ;
    const int W1 = taps == 9 ? d->W + 1 : d->W;
    g.dPQ = mkdiv(g.PQ);
    g.dW = mkdiv(g.W);
    g.dW1 = mkdiv(W1);
    g.dIMG = mkdiv(taps == 9 ? (d->H + 1) * W1 : g.PQ);
    if (!packed) {
        hipLaunchKernelGGL(repack_weights, dim3(g.K), dim3(kRepackThreads), 0, st, (const int8_t *)b, d->K, d->C, d->R, d->S,
                           which, wpk, colsum);
        Q8T_LAUNCH_CHECK();
    }
    Sched sch;
    const int occs = g.K / CH;
    int nbx = 512 / occs;                       // two workgroups (16 wavefronts) per compute unit in total
    const int max_useful = (g.M + 63) / 64;     // no point in ranges shorter than 64 rows
    if (nbx > max_useful) nbx = max_useful;
    nbx = ((nbx + 7) / 8) * 8;
    sch.nbx = nbx;
    sch.rpb = ((g.M + nbx - 1) / nbx + 15) / 16 * 16;
    // wide staging needs 16-position groups that never straddle an image or start mid-row group
    const bool v16 = (g.PQ % 16 == 0) && (g.W % 4 == 0) && g.W >= 4 && q8t_aligned(a, 16);
    sch.halo_al = taps == 9 ? (v16 ? ((g.W + 1 + 15) & ~15) : ((g.W + 1 + 3) & ~3)) : 0;
    sch.pg_blocks = (((BM + 2 * sch.halo_al) >> 2) + 15) / 16;
    sch.maxr = rows_needed(taps, g.W, g.PQ);
    const dim3 grid((unsigned)nbx, (unsigned)occs);
    const int8_t *pa = (const int8_t *)a;
    int32_t *pacc = (int32_t *)out_acc;
    const bool sq = d->H == d->W;
#define Q8T_CONV(T, WCV, V)                                                                                        \
    (bnpart ? launch_conv<T, WCV, V, true, false>(grid, st, pa, wpk, colsum, qa, qb, g, sch, out_f, pacc, bnpart, fuse)      \
            : (fuse.act ? launch_conv<T, WCV, V, false, true>(grid, st, pa, wpk, colsum, qa, qb, g, sch, out_f, pacc, bnpart, fuse) \
                        : launch_conv<T, WCV, V, false, false>(grid, st, pa, wpk, colsum, qa, qb, g, sch, out_f, pacc, bnpart, fuse)))
    if (taps == 9) {
        if (sq && d->W == 56 && v16) rc = Q8T_CONV(9, 56, true);
        else if (sq && d->W == 28 && v16) rc = Q8T_CONV(9, 28, true);
        else if (sq && d->W == 14) rc = Q8T_CONV(9, 14, false);
        else if (v16) rc = Q8T_CONV(9, 0, true);
        else rc = Q8T_CONV(9, 0, false);
    } else {
        if (sq && d->W == 56 && v16) rc = Q8T_CONV(1, 56, true);
        else if (v16) rc = Q8T_CONV(1, 0, true);
        else rc = Q8T_CONV(1, 0, false);
    }
#undef Q8T_CONV
    if (rc) return rc;
    if (bn_stats) {
        const int nact = (g.M + sch.rpb - 1) / sch.rpb;
        hipLaunchKernelGGL(conv_stats_finalize, dim3((unsigned)g.K), dim3(256), 0, st, bnpart, g.K, nbx, nact,
                           (double)g.M, qa, qb, bn_stats);
        Q8T_LAUNCH_CHECK();
    }
    return Q8T_OK;
}

