// int8 implicit-GEMM convolution for the layers with many channels on small planes (3x3, stride 1,
// pad 1; reduction channels a multiple of 64, output channels a multiple of 128, planes up to 32 wide; e.g.
// 128 -> 128 on 28x28, 256 -> 256 on 14x14 and 512 -> 512 on 7x7): forward, and the layer gradient as the same convolution with the
// filter flipped and its channel roles swapped (Section 4, eq. (grad_layer)).
//
// GEMM view: rows = flattened (image, y, x) positions, cols = output channels, reduction = (64
// input channels, tap).  A workgroup of 4 wavefronts owns 128 rows x 256 output channels (128 where the
// layer has no multiple of 256); every wavefront multiplies all 128 rows against its own 64 (32) output
// channels (eight or four 32x32 accumulators, v_mfma_i32_32x32x32_i8).  What this buys over a 64-channel output tile:
//  * the activations of a 64-channel chunk (128 rows + halo) are staged ONCE and serve 9 taps x 256
//    output channels: they sit in LDS in padded coordinates (a zero-point row after every image row
//    and one between images), so a tap is a constant row offset, an immediate in the LDS read;
//  * the weights never touch LDS: a wavefront's 64 output channels are its own, so its MFMA operands are
//    loaded from the packed filter (L2-resident, laid out in fragment order) straight into registers, two
//    steps ahead; LDS carries the activations only, and the workgroup meets at one barrier per chunk;
//  * NCHW int8 activations are transposed on the way into LDS with v_perm (4 positions x 4 channels
//    per piece).  Planes whose size is not a multiple of 4 (7x7) have no aligned dwords per channel:
//    there a piece is cut out of two aligned dwords with v_alignbyte.
// LDS rows are 80 bytes apart (64 + 16): with the 32x32x32 fragment pattern (lane ->
// row lane % 32, 16-byte group lane / 32) an odd number of 16-byte groups per row keeps the 16 lanes of
// every read phase on distinct bank groups.
// Row sums of the activations (zero-point correction) do not cost MFMAs: a thread per LDS row adds up
// its 64 bytes per chunk (v_dot4), and the sum of a row over the 9 taps is formed once at the end.
#include <type_traits>

#include "q8t_common.h"
#include "q8t_internal.h"
#include "repack.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int BM = 128, CH = 64;   // rows per workgroup, channels per chunk; columns per workgroup: 128 or 256
constexpr int ROWB = 80;
constexpr int MARG = 8;          // spare LDS rows on either side of an activation buffer (pieces that hang over)
constexpr int MAXR = 256;        // rows of one activation buffer (one thread per row sums it)
constexpr int MAXSLOT = 5;       // staging pieces per thread and chunk
constexpr int kSkip = -1000000;   // a piece with nothing to store

struct WideGeom {
    int N, C, K;         // images, reduction channels, output channels
    int H, W, PQ, M;     // plane, rows of the GEMM
    int W1, IMG;         // padded row pitch (W + 1) and padded image ((H + 1) * W1)
    int maxr;            // LDS rows of one activation buffer (<= MAXR)
    int halo;            // real positions staged on either side of the tile (multiple of 4)
    int nbx;             // row tiles
    int pg_blocks;       // blocks of 16 position groups per channel-group block
    int nslot;           // staging iterations per thread (<= MAXSLOT)
    int igroups;         // unaligned planes: position groups per image, ceil(PQ / 4)
    int last_dword;      // index of the last aligned dword of the operand
};

// Packed filter (layout and body: repack.h, q8t_repack_wide)
__global__ __launch_bounds__(kRepackThreads) void repack_wide(const int8_t *__restrict__ w, int Kf, int Cf, int dgrad, int BN,
                                                              int8_t *__restrict__ out, int *__restrict__ colsum)
{
    __shared__ int red[kRepackThreads / 64];
    q8t_repack_wide(w, Kf, Cf, dgrad, BN, out, colsum, (int)blockIdx.x, red);
}

// in[j] = 4 consecutive positions of channel j; out[i] = 4 channels of position i
__device__ __forceinline__ void transpose4x4(const uint32_t in[4], uint32_t out[4])
{
    const uint32_t t0 = __builtin_amdgcn_perm(in[1], in[0], 0x05010400);
    const uint32_t t1 = __builtin_amdgcn_perm(in[1], in[0], 0x07030602);
    const uint32_t t2 = __builtin_amdgcn_perm(in[3], in[2], 0x05010400);
    const uint32_t t3 = __builtin_amdgcn_perm(in[3], in[2], 0x07030602);
    out[0] = __builtin_amdgcn_perm(t2, t0, 0x05040100);
    out[1] = __builtin_amdgcn_perm(t2, t0, 0x07060302);
    out[2] = __builtin_amdgcn_perm(t3, t1, 0x05040100);
    out[3] = __builtin_amdgcn_perm(t3, t1, 0x07060302);
}

// AL: the plane size is a multiple of 4 (aligned dwords per channel).  NS: staging pieces per thread.
// NTW: 32-column tiles per wavefront (2: 256 output channels per workgroup, 1: 128).
template <bool AL, int NS, bool STATS, int NTW>
__global__ __launch_bounds__(kThreads, AL ? 2 : 1) void conv_wide_kernel(const int8_t *__restrict__ x,
                                                                        const int8_t *__restrict__ wpk,
                                                                        const int *__restrict__ colsum,
                                                                        const q8t_qparams *__restrict__ qpa,
                                                                        const q8t_qparams *__restrict__ qpb,
                                                                        const WideGeom g, float *__restrict__ y,
                                                                        int32_t *__restrict__ acc_out,
                                                                        Q8tConvStat *__restrict__ bnpart)
{
    constexpr int BN = 128 * NTW, WN = 32 * NTW;   // columns of the workgroup, of a wavefront
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const int A_BYTES = (g.maxr + 2 * MARG) * ROWB;   // one activation buffer with its spare rows
    uint8_t *As = smem + MARG * ROWB;                  // buffer b at As + b * A_BYTES
    int *Srow = reinterpret_cast<int *>(smem + 2 * A_BYTES);   // [maxr] byte sums of the staged rows over all channels
    int *RS = Srow + MAXR;                             // [BM] row sums over the taps
    int *OOFF = RS + BM;                               // [BM] offset of the row's position in the result (channel 0)

    // row tiles dealt out so that neighbours (shared halo) run on one XCD
    const int bidx = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    if (bidx >= g.nbx) return;
    const int n0 = blockIdx.y * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hk = lane >> 5;
    const int g0 = bidx * BM, g1 = min(g.M, g0 + BM);
    const int W = g.W, PQ = g.PQ, W1 = g.W1, IMG = g.IMG;

    const int za = qpa->zero_point - (1 << (qpa->bits - 1)), zb = qpb->zero_point - (1 << (qpb->bits - 1));
    const float sc = qpa->scale * qpb->scale;
    const uint32_t zavec = (uint32_t)(za & 255) * 0x01010101u;

    // padded coordinate of a real row index: b * IMG + (p + 1) * W1 + q
    auto apad = [&](int gr) -> int {
        const int b = gr / PQ, pos = gr - b * PQ;
        const int p = pos / W;
        return b * IMG + pos + p + W1;
    };
    const int a0 = apad(g0) - (W1 + 1);   // padded coordinate of LDS row 0

    // ---- both activation buffers start as zero-point rows; staging overwrites the real positions only ----
    {
        const uint4 z = make_uint4(zavec, zavec, zavec, zavec);
        uint4 *p = reinterpret_cast<uint4 *>(smem);
        const int n16 = 2 * A_BYTES / 16;
        for (int i = tid; i < n16; i += kThreads) p[i] = z;
    }

    // ---- staging pieces of this thread: the same for every chunk but for the channel offset ----
    // a wavefront instruction covers 16 position groups x 4 channel groups (64-byte runs per channel)
    int s_off[NS], s_row[NS], s_thr[NS], s_nv[NS];
    const int l16 = lane & 15, kb = lane >> 4;
    const int CC = g.C / CH;
    int imgA = 0;
    if (!AL) imgA = max(0, g0 - g.halo) / PQ;
#pragma unroll
    for (int it = 0; it < NS; ++it) {
        const int slab = wave + it * (kThreads / 64);
        const int pgb = slab % g.pg_blocks, cgb = slab / g.pg_blocks;
        const int pg = pgb * 16 + l16, cg = cgb * 4 + kb;
        s_row[it] = kSkip;
        s_off[it] = 0;
        s_thr[it] = 4;
        s_nv[it] = 4;
        int gr, b, pos;
        bool ok = cgb < 4;
        if (AL) {
            gr = g0 - g.halo + pg * 4;
            ok = ok && pg * 4 < (g1 - g0) + 2 * g.halo && gr >= 0 && gr < g.M;
            b = ok ? gr / PQ : 0;
            pos = gr - b * PQ;
        } else {
            b = imgA + pg / g.igroups;
            pos = (pg - (pg / g.igroups) * g.igroups) * 4;
            gr = b * PQ + pos;
            ok = ok && b < g.N && gr + 3 >= g0 - g.halo && gr < g1 + g.halo;
            if (ok) s_nv[it] = min(4, PQ - pos);
        }
        if (ok) {
            const int p = pos / W;
            const int r = b * IMG + pos + p + W1 - a0;
            if (r > -MARG && r + 5 < g.maxr + MARG) {
                s_row[it] = r * ROWB + cg * 4;
                s_thr[it] = W - 1 - (pos - p * W);   // positions after this one sit one LDS row further
                s_off[it] = (b * g.C + cg * 4) * PQ + pos;
            }
        }
    }
    uint32_t pa[NS][AL ? 4 : 8];
    auto load_a = [&](int cc) {
#pragma unroll
        for (int it = 0; it < NS; ++it) {
            const int e0 = s_off[it] + cc * CH * PQ;   // pieces with nothing to store read element 0.. of the chunk: in bounds
            if (AL) {
#pragma unroll
                for (int j = 0; j < 4; ++j) pa[it][j] = *reinterpret_cast<const uint32_t *>(x + e0 + j * PQ);
            } else {
                const uint32_t *x32 = reinterpret_cast<const uint32_t *>(x);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int idx = (e0 + j * PQ) >> 2;
                    pa[it][2 * j] = x32[idx];
                    pa[it][2 * j + 1] = x32[min(idx + 1, g.last_dword)];
                }
            }
        }
    };
    auto commit_a = [&](int cc, int buf) {
        uint8_t *dst = As + buf * A_BYTES;
#pragma unroll
        for (int it = 0; it < NS; ++it) {
            if (s_row[it] == kSkip) continue;
            uint32_t in[4], out[4];
            if (AL) {
#pragma unroll
                for (int j = 0; j < 4; ++j) in[j] = pa[it][j];
            } else {
                const int e0 = s_off[it] + cc * CH * PQ;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    in[j] = __builtin_amdgcn_alignbyte(pa[it][2 * j + 1], pa[it][2 * j], (uint32_t)((e0 + j * PQ) & 3));
            }
            transpose4x4(in, out);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (!AL && i >= s_nv[it]) continue;
                const int o = s_row[it] + (i + (i > s_thr[it] ? 1 : 0)) * ROWB;
                *reinterpret_cast<uint32_t *>(dst + o) = out[i];
            }
        }
    };

    // ---- weights: a wavefront's 64 output channels are its own, so their fragments go from memory straight to
    // registers; block (chunk, tap) holds, per wavefront, four 1 KB fragments (column tile, K half) in lane order ----
    const int nsteps = CC * 9;
    const int8_t *wsrc = wpk + (size_t)blockIdx.y * CC * 9 * BN * CH + wave * (2048 * NTW) + lane * 16;
    struct BFrag {
        v4i n0k0, n0k1, n1k0, n1k1;   // named members: the sets stay in registers
    };
    auto load_b = [&](int q) -> BFrag {
        const int qc = min(q, nsteps - 1);   // past the end: the last block again, never used
        const int8_t *src = wsrc + (size_t)qc * (BN * CH);
        BFrag f;
        f.n0k0 = *reinterpret_cast<const v4i *>(src);
        f.n0k1 = *reinterpret_cast<const v4i *>(src + 1024);
        if (NTW == 2) {
            f.n1k0 = *reinterpret_cast<const v4i *>(src + 2048);
            f.n1k1 = *reinterpret_cast<const v4i *>(src + 3072);
        } else {
            f.n1k0 = f.n0k0;
            f.n1k1 = f.n0k1;
        }
        return f;
    };

    // fragment addresses: lane -> row l32 of a 32-row tile, 16-byte group hk (+2 for the second K half)
    int arow[4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
        int gr = g0 + mt * 32 + l32;
        if (gr >= g.M) gr = g0;
        arow[mt] = (apad(gr) - a0 - (W1 + 1)) * ROWB + hk * 16;   // row of the tap (0, 0); tap (dr, ds) adds dr * W1 + ds
    }

    v16i acc[4][NTW];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0;
    int srow = 0;

    // Operands are fetched ahead of their use so that no MFMA waits: the activation fragments of the next
    // 32-row group one group ahead (LDS), the weight fragments two steps ahead (three register sets, used in
    // turn: 9 steps per chunk keep set = tap % 3).
    struct AFrag {
        v4i k0, k1;
    };
    AFrag af0, af1;
    BFrag bf0, bf1, bf2;
    auto read_a = [&](int buf, int tap, int mt) -> AFrag {
        const uint8_t *p = As + buf * A_BYTES + ((tap / 3) * W1 + (tap % 3)) * ROWB + arow[mt];
        AFrag f;
        f.k0 = *reinterpret_cast<const v4i *>(p);
        f.k1 = *reinterpret_cast<const v4i *>(p + 32);
        return f;
    };
    auto mma = [&](int mt, const AFrag a, const BFrag b) {
        acc[mt][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a.k0, b.n0k0, acc[mt][0], 0, 0, 0);
        if (NTW == 2) acc[mt][NTW - 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a.k0, b.n1k0, acc[mt][NTW - 1], 0, 0, 0);
        acc[mt][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a.k1, b.n0k1, acc[mt][0], 0, 0, 0);
        if (NTW == 2) acc[mt][NTW - 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a.k1, b.n1k1, acc[mt][NTW - 1], 0, 0, 0);
    };

    load_a(0);
    bf0 = load_b(0);
    bf1 = load_b(1);
    __syncthreads();          // the fill above is complete
    commit_a(0, 0);

    // One step = one tap of one chunk: 16 MFMAs per wavefront.  The scheduler is told the order outright (per
    // 32-row group: the LDS reads of the next group, a quarter of the weight fetch for the step after next, four
    // MFMAs); left alone it sinks every read to just before its use.
    auto step = [&](auto tap_c, int cc) {
        constexpr int T = decltype(tap_c)::value;
        const int s = cc * 9 + T, buf = cc & 1;
        const BFrag &cur = T % 3 == 0 ? bf0 : (T % 3 == 1 ? bf1 : bf2);
        const BFrag nxt = load_b(s + 2);
        constexpr int NM = 2 * NTW;   // MFMAs per 32-row group
        af1 = read_a(buf, T, 1);
        mma(0, af0, cur);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, NM, 0);
        af0 = read_a(buf, T, 2);
        mma(1, af1, cur);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        if (NTW == 2) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, NM, 0);
        af1 = read_a(buf, T, 3);
        mma(2, af0, cur);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, NM, 0);
        if (T < 8) af0 = read_a(buf, T + 1, 0);   // the next chunk's activations may not be in LDS yet
        mma(3, af1, cur);
        if (T < 8) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        if (NTW == 2) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, NM, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (T % 3 == 0) bf2 = nxt;        // set (T + 2) % 3 was last used in the previous step
        else if (T % 3 == 1) bf0 = nxt;
        else bf1 = nxt;
    };
    for (int cc = 0; cc < CC; ++cc) {
        const int buf = cc & 1;
        // chunk cc is complete in buffer buf, and every wavefront is past its reads of the other buffer
        q8t_lds_barrier();
        af0 = read_a(buf, 0, 0);
        // byte sum of this thread's LDS row over the chunk's 64 channels
        if (tid < g.maxr) {
            const uint8_t *row = As + buf * A_BYTES + tid * ROWB;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const v4i v = *reinterpret_cast<const v4i *>(row + q * 16);
#pragma unroll
                for (int d = 0; d < 4; ++d) srow = __builtin_amdgcn_sdot4(v[d], 0x01010101, srow, false);
            }
        }
        const int cnext = min(cc + 1, CC - 1);
        load_a(cnext);
        step(std::integral_constant<int, 0>{}, cc);
        step(std::integral_constant<int, 1>{}, cc);
        step(std::integral_constant<int, 2>{}, cc);
        step(std::integral_constant<int, 3>{}, cc);
        step(std::integral_constant<int, 4>{}, cc);
        commit_a(cnext, buf ^ 1);
        step(std::integral_constant<int, 5>{}, cc);
        step(std::integral_constant<int, 6>{}, cc);
        step(std::integral_constant<int, 7>{}, cc);
        step(std::integral_constant<int, 8>{}, cc);
    }

    // ---- row sums over the taps and result offsets, one row per thread ----
    if (tid < g.maxr) Srow[tid] = srow;
    __syncthreads();
    if (tid < BM) {
        int gr = g0 + tid;
        if (gr >= g.M) gr = g0;
        const int b = gr / PQ, pos = gr - b * PQ;
        const int r = b * IMG + pos + pos / W + W1 - a0 - (W1 + 1);
        int rs = 0;
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) rs += Srow[r + (tap / 3) * W1 + (tap % 3)];
        RS[tid] = rs;
        OOFF[tid] = b * g.K * PQ + pos;
    }
    __syncthreads();

    // ---- epilogue: zero-point correction in wrapping 32-bit arithmetic, dequantization; a lane holds
    // rows 8i + 4hk + j (j = 0..3: four consecutive positions) of one output channel per 32x32 tile ----
    const uint32_t kzz = (uint32_t)(g.C * 9) * (uint32_t)za * (uint32_t)zb;
    // planes without aligned runs of four positions: a wavefront turns each 32x32 tile round in its own LDS patch,
    // so that a store instruction writes 32 consecutive positions of two channels instead of 64 lone dwords
    int *T = reinterpret_cast<int *>(smem) + wave * (32 * 36);   // [32 channels][36]: the activation buffers are free now
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) {
        const int n = n0 + wave * WN + nt * 32 + l32;
        const uint32_t ncs = 0u - (uint32_t)za * (uint32_t)colsum[n];
        long long st_s = 0;
        int st_mn = 2147483647, st_mx = -2147483647 - 1;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
            if (g0 + mt * 32 >= g1) continue;   // uniform
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int t0 = mt * 32 + 8 * i + 4 * hk;
                const v4i rs4 = *reinterpret_cast<const v4i *>(&RS[t0]);
                int c[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    c[j] = (int)((uint32_t)acc[mt][nt][i * 4 + j] + (kzz - (uint32_t)zb * (uint32_t)rs4[j]) + ncs);
                const bool full = g0 + t0 + 3 < g1;
                if (STATS) {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (full || g0 + t0 + j < g1) {
                            st_s += c[j];
                            st_mn = min(st_mn, c[j]);
                            st_mx = max(st_mx, c[j]);
                        }
                }
                if (AL) {
                    if (!full && g0 + t0 >= g1) continue;
                    const v4i of4 = *reinterpret_cast<const v4i *>(&OOFF[t0]);
                    if (full) {
                        // 4 positions of one image, 16-byte aligned (plane size and tile start are multiples of 4)
                        const size_t o = (size_t)of4[0] + (size_t)n * PQ;
                        if (acc_out) *reinterpret_cast<int4 *>(acc_out + o) = make_int4(c[0], c[1], c[2], c[3]);
                        if (y) {
                            float4 f;
                            f.x = sc * (float)c[0];
                            f.y = sc * (float)c[1];
                            f.z = sc * (float)c[2];
                            f.w = sc * (float)c[3];
                            *reinterpret_cast<float4 *>(y + o) = f;
                        }
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            if (g0 + t0 + j >= g1) continue;
                            const size_t o = (size_t)of4[j] + (size_t)n * PQ;
                            if (acc_out) acc_out[o] = c[j];
                            if (y) y[o] = sc * (float)c[j];
                        }
                    }
                } else {
                    *reinterpret_cast<v4i *>(&T[l32 * 36 + 8 * i + 4 * hk]) = (v4i){c[0], c[1], c[2], c[3]};
                }
            }
            if (!AL) {
                // lane -> position l32 of the tile; 16 instructions cover the 32 channels two at a time
                const int row = mt * 32 + l32;
                const bool live = g0 + row < g1;
                const size_t obase = (size_t)OOFF[row] + (size_t)(n0 + wave * WN + nt * 32) * PQ;
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    const int col = 2 * k + hk;
                    const int v = T[col * 36 + l32];
                    if (live) {
                        const size_t o = obase + (size_t)col * PQ;
                        if (acc_out) acc_out[o] = v;
                        if (y) y[o] = sc * (float)v;
                    }
                }
            }
        }
        if (STATS) {
            // the two lanes that share a channel
            st_s += __shfl_xor(st_s, 32, 64);
            st_mn = min(st_mn, __shfl_xor(st_mn, 32, 64));
            st_mx = max(st_mx, __shfl_xor(st_mx, 32, 64));
            if (hk == 0) {
                Q8tConvStat r;
                r.sum = st_s;
                r.mn = st_mn;
                r.mx = st_mx;
                bnpart[((size_t)(n >> 6) * g.nbx + bidx) * 64 + (n & 63)] = r;
            }
        }
    }
}

bool make_geom(int which, const q8t_conv_desc *d, WideGeom *g)
{
    if (which > 1 || d->R != 3 || d->S != 3 || d->stride != 1 || d->pad != 1) return false;
    g->N = d->N;
    g->H = d->H;
    g->W = d->W;
    g->PQ = d->H * d->W;
    g->C = which == 0 ? d->C : d->K;
    g->K = which == 0 ? d->K : d->C;
    if (g->C % CH || g->K % 128) return false;
    if (d->W < 4 || d->H < 2 || d->W > 32) return false;
    const int64_t M = (int64_t)d->N * g->PQ;
    if (M * g->C >= ((int64_t)1 << 31) || M * g->K >= ((int64_t)1 << 31)) return false;
    g->M = (int)M;
    g->W1 = d->W + 1;
    g->IMG = (d->H + 1) * g->W1;
    // padded coordinates a tile of BM positions can span, plus the halo rows on either side
    const int row_ends = (BM + d->W - 2) / d->W + 1, img_ends = (BM + g->PQ - 2) / g->PQ + 1;
    g->maxr = BM + row_ends + img_ends * g->W1 + 2 * (g->W1 + 1) + 1;
    if (g->maxr > MAXR) return false;
    g->halo = (d->W + 1 + 3) & ~3;
    g->nbx = (g->M + BM - 1) / BM;
    g->igroups = (g->PQ + 3) / 4;
    g->last_dword = (int)((M * g->C) / 4) - 1;
    int npg;
    if (g->PQ % 4 == 0)
        npg = (BM + 2 * g->halo) / 4;
    else
        npg = ((BM + 2 * g->halo + g->PQ - 2) / g->PQ + 1) * g->igroups;   // whole images that the staged range touches
    g->pg_blocks = (npg + 15) / 16;
    g->nslot = (g->pg_blocks * 4 + kThreads / 64 - 1) / (kThreads / 64);
    if (g->nslot > MAXSLOT) return false;
    return true;
}

size_t lds_bytes(const WideGeom &g)
{
    return (size_t)2 * (g.maxr + 2 * MARG) * ROWB + (size_t)(MAXR + 2 * BM) * sizeof(int);
}

template <bool AL, int NS, bool STATS, int NTW>
int launch(const WideGeom &g, hipStream_t st, const int8_t *a, const int8_t *wpk, const int *colsum, const q8t_qparams *qa,
           const q8t_qparams *qb, float *out_f, int32_t *out_acc, Q8tConvStat *bnpart)
{
    static Q8tLdsOptIn optin;
    const size_t lds = lds_bytes(g);
    if (q8t_allow_lds(optin, (const void *)conv_wide_kernel<AL, NS, STATS, NTW>, 96 * 1024) != Q8T_OK) return Q8T_ERR_HIP;
    const dim3 grid((unsigned)((g.nbx + 7) / 8 * 8), (unsigned)(g.K / (128 * NTW)));
    hipLaunchKernelGGL((conv_wide_kernel<AL, NS, STATS, NTW>), grid, dim3(kThreads), lds, st, a, wpk, colsum, qa, qb, g, out_f,
                       out_acc, bnpart);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

}  // namespace

bool q8t_wide_conv_supported(int which, const q8t_conv_desc *d, const void *a, const void *out_f, const void *out_acc)
{
    WideGeom g;
    if (!make_geom(which, d, &g)) return false;
    // 128-column tiles (layers without a multiple of 256 output channels) read every activation fragment for half
    // the MFMAs: measured slower than the 64-column kernel on 128 -> 128 @28 (67 against 58 us), so they only serve
    // planes that kernel does not take (sizes that are not multiples of 4)
    if (g.K % 256 != 0 && g.PQ % 4 == 0) return false;
    return q8t_aligned(a, 4) && q8t_aligned(out_f, 16) && q8t_aligned(out_acc, 16);
}

int q8t_wide_conv_pack_layout(int which, const q8t_conv_desc *d)
{
    WideGeom g;
    if (!make_geom(which, d, &g)) return Q8T_PACK_NONE;
    if (g.K % 256 != 0 && g.PQ % 4 == 0) return Q8T_PACK_NONE;   // as q8t_wide_conv_supported
    return g.K % 256 == 0 ? Q8T_PACK_WIDE256 : Q8T_PACK_WIDE128;
}

size_t q8t_wide_conv_ws(int which, const q8t_conv_desc *d)
{
    WideGeom g;
    if (!make_geom(which, d, &g)) return 0;
    const size_t wbytes = (size_t)d->K * d->C * 9;
    return ((wbytes + 255) & ~(size_t)255) + (((size_t)g.K * sizeof(int) + 255) & ~(size_t)255) +
           (size_t)g.K * g.nbx * sizeof(Q8tConvStat);
}

int q8t_wide_conv(int which, const q8t_conv_desc *d, const void *a, const q8t_qparams *qa, const void *b,
                  const q8t_qparams *qb, float *out_f, void *out_acc, float *bn_stats, void *ws, hipStream_t st,
                  const void *packed)
{
    WideGeom g;
    if (!make_geom(which, d, &g)) return Q8T_ERR_SHAPE;
    if (!ws || !q8t_aligned(ws, 16)) return Q8T_ERR_WORKSPACE;
    if (packed && !q8t_aligned(packed, 16)) return Q8T_ERR_WORKSPACE;
    if (lds_bytes(g) > 96 * 1024) return Q8T_ERR_SHAPE;
    const size_t wbytes = (size_t)d->K * d->C * 9;
    // the packed filter and its column sums: made here in the workspace, or handed in (q8t_qconv_pack_multi)
    int8_t *wpk = packed ? (int8_t *)packed : (int8_t *)ws;
    int *colsum = (int *)((char *)wpk + ((wbytes + 255) & ~(size_t)255));
    Q8tConvStat *bnpart = bn_stats ? (Q8tConvStat *)((char *)ws + ((wbytes + 255) & ~(size_t)255) +
                                                     (((size_t)g.K * sizeof(int) + 255) & ~(size_t)255))
                                   : (Q8tConvStat *)nullptr;
    const int ntw = g.K % 256 == 0 ? 2 : 1;
    if (!packed) {
        hipLaunchKernelGGL(repack_wide, dim3((unsigned)g.K), dim3(kRepackThreads), 0, st, (const int8_t *)b, d->K, d->C, which,
                           128 * ntw, wpk, colsum);
        Q8T_LAUNCH_CHECK();
    }
    const int8_t *pa = (const int8_t *)a;
    int32_t *pacc = (int32_t *)out_acc;
    const bool al = g.PQ % 4 == 0;
    int rc;
#define Q8T_WIDE2(ALV, NSV, NT)                                                                                     \
    (bnpart ? launch<ALV, NSV, true, NT>(g, st, pa, wpk, colsum, qa, qb, out_f, pacc, bnpart)                       \
            : launch<ALV, NSV, false, NT>(g, st, pa, wpk, colsum, qa, qb, out_f, pacc, bnpart))
#define Q8T_WIDE(ALV, NSV) (ntw == 2 ? Q8T_WIDE2(ALV, NSV, 2) : Q8T_WIDE2(ALV, NSV, 1))
    if (al)
        rc = g.nslot <= 3 ? Q8T_WIDE(true, 3) : Q8T_WIDE(true, 5);
    else
        rc = g.nslot <= 4 ? Q8T_WIDE(false, 4) : Q8T_WIDE(false, 5);
#undef Q8T_WIDE
#undef Q8T_WIDE2
    if (rc) return rc;
    if (bnpart) return q8t_conv_stats_finalize(bnpart, g.K, g.nbx, g.nbx, (double)g.M, qa, qb, bn_stats, st);
    return Q8T_OK;
}
