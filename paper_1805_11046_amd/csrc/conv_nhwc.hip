// General MFMA path for the forward and layer-gradient convolutions (Section 4: both products
// take 8-bit operands and accumulate in 32 bits): any filter size, stride and padding, for
// channel counts that are multiples of 64.  Three launches per call:
//
//  1. to_nhwc      the NCHW int8 operand is rewritten channel-contiguous ([N][H][W][C]) into the
//                  workspace, so that the 64 reduction channels of one filter tap are 64
//                  consecutive bytes; the same pass emits the per-position channel sum that the
//                  zero-point correction needs.
//  2. repack_taps  filter -> [tap][output channel][reduction channel] and the per-output-channel
//                  sums (per stride class).
//  3. igemm_nhwc   implicit GEMM, rows = output positions, columns = output channels, K = taps x
//                  channels in steps of 64, on the shared software-pipelined main loop
//                  (gemm_core.h; 256x256, 128x128 or 128x64 tiles).
//
// Padded taps are staged as the stored zero point, which makes their corrected contribution
// exactly zero; with a = stored code, za/zb = stored zero points:
//    sum (a-za)(b-zb) = sum ab - zb*sum a - za*sum b + Kp*za*zb.
//
// The layer gradient of a strided convolution is split into stride x stride classes of input
// positions (same residue of (h, w) modulo the stride).  Inside a class every position sees the
// same subset of filter taps at stride 1, so each class is a dense problem of its own and no
// multiply is spent on taps that cannot contribute.  All classes run in one launch: the tile index
// selects the class, and the classes of one region, which write interleaved elements of the same
// result lines, are neighbours in the tile order.
#include "q8t_common.h"
#include "q8t_internal.h"
#include "gemm_core.h"

namespace {

using q8t_gemm::v4i;

constexpr int kThreads = 256;
constexpr int PITCH = 80;    // LDS bytes between rows of 64
constexpr int MAXT = 49;     // taps (7x7)
constexpr int MAXCLS = 16;   // stride classes (stride <= 4)

struct TapList {             // per tap: two small signed numbers
    int8_t a[MAXT + 3], b[MAXT + 3];
};
struct ClassOffsets {
    int off[MAXCLS + 1];     // taps of class z are [off[z], off[z+1]) of the TapList
};

struct ClassGeo {            // per stride class: positions enumerated, rows, first tap, taps
    int v[MAXCLS][5];        // OH, OW, M, first tap, number of taps
};
constexpr int CLS_INTS = 8;  // ints per class in the device copy of the table

struct Geo {
    int N, IH, IW, Cp;       // staged operand: [N][IH][IW][Cp]
    int OH, OW;              // output positions enumerated by a class (rows m = (n, oh, ow))
    int ish, isw;            // operand step per output step
    int OC, OHf, OWf;        // NCHW result: channels, full height and width
    int osh, osw, oph, opw;  // result position = (oh*osh + oph, ow*osw + opw)
    int M;                   // N*OH*OW
    int T;                   // taps of a class
    int vec;                 // result pointers are 16-byte aligned
    int ncls, mtiles;        // stride classes in this launch; row tiles of the largest class
    int fill;                // stride 2, even result size, only class (0, 0) has taps: its workgroups
                             // also write the zeros of the three empty classes
};

__device__ __forceinline__ int bytesum4(uint32_t v) { return __builtin_amdgcn_sdot4((int)v, 0x01010101, 0, false); }

// ---- 1. NCHW -> NHWC with channel sums --------------------------------------------------------
template <int VB>   // bytes per global load: 4 needs HW % 4 == 0 and a 4-byte aligned source
__global__ __launch_bounds__(kThreads) void to_nhwc(const int8_t *__restrict__ src, int C, int HW,
                                                    int8_t *__restrict__ dst, int *__restrict__ chansum)
{
    __shared__ __align__(16) int8_t tile[64 * PITCH];
    const int n = blockIdx.y, p0 = blockIdx.x * 64;
    const int tid = threadIdx.x;
    const int rp = tid >> 2, rq = tid & 3;   // read-out role: position rp, 16-byte chunk rq
    int sum = 0;
    for (int c0 = 0; c0 < C; c0 += 64) {
        if (VB == 4) {
            const int ch = tid >> 4, d = tid & 15;
#pragma unroll
            for (int pass = 0; pass < 4; ++pass) {
                const int c = ch + pass * 16, p = p0 + d * 4;
                uint32_t v = 0;
                if (p < HW) v = *reinterpret_cast<const uint32_t *>(src + (size_t)(n * C + c0 + c) * HW + p);
                tile[(d * 4 + 0) * PITCH + c] = (int8_t)(v & 255);
                tile[(d * 4 + 1) * PITCH + c] = (int8_t)((v >> 8) & 255);
                tile[(d * 4 + 2) * PITCH + c] = (int8_t)((v >> 16) & 255);
                tile[(d * 4 + 3) * PITCH + c] = (int8_t)(v >> 24);
            }
        } else {
            const int ch = tid >> 6, d = tid & 63;
#pragma unroll 4
            for (int pass = 0; pass < 16; ++pass) {
                const int c = ch + pass * 4, p = p0 + d;
                tile[d * PITCH + c] = p < HW ? src[(size_t)(n * C + c0 + c) * HW + p] : (int8_t)0;
            }
        }
        __syncthreads();
        if (p0 + rp < HW) {
            const uint4 v = *reinterpret_cast<const uint4 *>(tile + rp * PITCH + rq * 16);
            *reinterpret_cast<uint4 *>(dst + ((size_t)n * HW + p0 + rp) * C + c0 + rq * 16) = v;
            sum += bytesum4(v.x) + bytesum4(v.y) + bytesum4(v.z) + bytesum4(v.w);
        }
        __syncthreads();
    }
    sum += __shfl_xor(sum, 1, Q8T_WAVE);
    sum += __shfl_xor(sum, 2, Q8T_WAVE);
    if (rq == 0 && p0 + rp < HW) chansum[(size_t)n * HW + p0 + rp] = sum;
}

// Small planes (H*W <= 256): the 64 channels x H*W bytes of one image and channel chunk are one
// contiguous stretch of the NCHW tensor; it is copied to LDS with 16-byte loads whatever H*W is,
// and read back transposed.  One workgroup per image walks the channel chunks, so the channel sums
// stay in registers.
__global__ __launch_bounds__(kThreads) void to_nhwc_small(const int8_t *__restrict__ src, int C, int HW,
                                                          int8_t *__restrict__ dst, int *__restrict__ chansum)
{
    extern __shared__ __align__(16) int8_t flat[];   // [64][HW]
    const int n = blockIdx.x, tid = threadIdx.x;
    const int items = HW * 4;                        // (position, 16-channel quarter), quarter fastest
    int sum[4] = {0, 0, 0, 0};
    for (int c0 = 0; c0 < C; c0 += 64) {
        const uint4 *s4 = reinterpret_cast<const uint4 *>(src + ((size_t)n * C + c0) * HW);
        for (int i = tid; i < HW * 4; i += kThreads) reinterpret_cast<uint4 *>(flat)[i] = s4[i];   // 64*HW/16 pieces
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int it = tid + k * kThreads;
            if (it < items) {
                const int p = it >> 2, q = it & 3;
                uint32_t w[4];
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const int8_t *b = flat + (q * 16 + d * 4) * HW + p;
                    w[d] = (uint32_t)(uint8_t)b[0] | ((uint32_t)(uint8_t)b[HW] << 8) | ((uint32_t)(uint8_t)b[2 * HW] << 16) |
                           ((uint32_t)(uint8_t)b[3 * HW] << 24);
                }
                *reinterpret_cast<uint4 *>(dst + ((size_t)n * HW + p) * C + c0 + q * 16) = make_uint4(w[0], w[1], w[2], w[3]);
                sum[k] += bytesum4(w[0]) + bytesum4(w[1]) + bytesum4(w[2]) + bytesum4(w[3]);
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        int v = sum[k];
        v += __shfl_xor(v, 1, Q8T_WAVE);
        v += __shfl_xor(v, 2, Q8T_WAVE);
        const int it = tid + k * kThreads;
        if (it < items && (it & 3) == 0) chansum[(size_t)n * HW + (it >> 2)] = v;
    }
}

// ---- 2. filter -> [tap][output channel][reduction channel], sums per output channel ------------
// grid (OC, classes).  which 0: out = k, reduction = c;  which 1: out = c, reduction = k.
__global__ __launch_bounds__(kThreads) void repack_taps(const int8_t *__restrict__ w, int Kf, int Cf, int R, int S,
                                                        int which, TapList taps, TapList offs, ClassOffsets co,
                                                        ClassGeo cg, int8_t *__restrict__ wt,
                                                        int *__restrict__ colsum, int *__restrict__ tapoff,
                                                        int *__restrict__ clsinfo)
{
    __shared__ int part[kThreads / 64];
    const int j = blockIdx.x, z = blockIdx.y;
    // operand offsets of the taps, packed (dh in the low half), and the class table, for the main kernel
    if (j == 0 && z == 0 && threadIdx.x == 0) {
        for (int tt = 0; tt < co.off[MAXCLS]; ++tt)
            tapoff[tt] = (int)((uint32_t)(uint16_t)(int16_t)offs.a[tt] | ((uint32_t)(uint16_t)(int16_t)offs.b[tt] << 16));
        for (int c = 0; c < (int)gridDim.y; ++c)
            for (int k = 0; k < 5; ++k) clsinfo[c * CLS_INTS + k] = cg.v[c][k];
    }
    const int OC = which == 0 ? Kf : Cf, Cp = which == 0 ? Cf : Kf;
    const int RS = R * S;
    int sum = 0;
    for (int tt = co.off[z]; tt < co.off[z + 1]; ++tt) {
        const int rs = taps.a[tt] * S + taps.b[tt];
        for (int c = threadIdx.x; c < Cp; c += kThreads) {
            const size_t src = which == 0 ? ((size_t)j * Cf + c) * RS + rs : ((size_t)c * Cf + j) * RS + rs;
            const int8_t v = w[src];
            wt[((size_t)tt * OC + j) * Cp + c] = v;
            sum += v;
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, Q8T_WAVE);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) colsum[z * OC + j] = part[0] + part[1] + part[2] + part[3];
}

// ---- 3. implicit GEMM ---------------------------------------------------------------------------
// Staging role of a thread (see gemm_core.h): the 16-byte channel chunk q = tid & 3 of the output
// positions (tile rows) ar = tid >> 2 and ar + RP, and of the filter rows ar and ar + RP.
template <class C>
struct ConvOps {
    const int8_t *xin, *wt;
    const __attribute__((address_space(3))) int *stap;   // tap offsets, in LDS
    int IH, IW, Cp, OC, CC, q, wrow;
    int an0, ih0, iw0, an1, ih1, iw1;   // image and top-left operand position of the two rows
    bool av0, av1;
    uint32_t padw;
    int lt, lc;   // tap and channel chunk of the next load

    __device__ __forceinline__ uint4 row(bool av, int an, int ihb, int iwb, int to, int c) const
    {
        const int ih = ihb + (int)(int16_t)(to & 0xFFFF), iw = iwb + (to >> 16);
        uint4 v = make_uint4(padw, padw, padw, padw);
        if (av && (unsigned)ih < (unsigned)IH && (unsigned)iw < (unsigned)IW)
            v = *reinterpret_cast<const uint4 *>(xin + (size_t)((an * IH + ih) * IW + iw) * Cp + c * 64 + q * 16);
        return v;
    }
    __device__ __forceinline__ void load(q8t_gemm::Regs &r, bool valid)
    {
        const int t = valid ? lt : 0, c = valid ? lc : 0;
        const int to = stap[t];
        r.a0 = row(av0, an0, ih0, iw0, to, c);
        r.a1 = row(av1, an1, ih1, iw1, to, c);
        const int8_t *w = wt + ((size_t)t * OC + wrow) * Cp + c * 64 + q * 16;
        r.b0 = *reinterpret_cast<const uint4 *>(w);
        r.b1 = C::NB == 2 ? *reinterpret_cast<const uint4 *>(w + (size_t)C::RP * Cp) : r.b0;
        const bool wrap = lc + 1 == CC;
        lc = wrap ? 0 : lc + 1;
        lt += wrap ? 1 : 0;
    }
    // a surplus step stages zero filter rows: whatever the operand rows hold, it adds nothing
    __device__ __forceinline__ void prepare(q8t_gemm::Regs &r, bool valid)
    {
        r.b0 = q8t_gemm::sel16(valid, r.b0);
        r.b1 = q8t_gemm::sel16(valid, r.b1);
    }
};

template <class C>
constexpr size_t conv_lds_bytes()
{
    return (size_t)C::LDS_BYTES + C::BM * (sizeof(long long) + sizeof(int)) + (MAXT + 3) * sizeof(int);
}

template <class C>
__global__ __launch_bounds__(C::THREADS, C::MINB) void igemm_nhwc(const int8_t *__restrict__ xin,
                                                                   const int *__restrict__ chansum,
                                                                   const int8_t *__restrict__ wt,
                                                                   const int *__restrict__ colsum,
                                                                   const q8t_qparams *__restrict__ qpa,
                                                                   const q8t_qparams *__restrict__ qpb, Geo g,
                                                                   const int *__restrict__ tapoff,
                                                                   const int *__restrict__ clsinfo,
                                                                   float *__restrict__ out_f, int32_t *__restrict__ out_acc,
                                                                   Q8tConvStat *__restrict__ bnpart)
{
    constexpr int MT = C::MT, NT = C::NT, BM = C::BM, BN = C::BN;
    extern __shared__ __align__(16) int8_t smem[];
    int8_t *sA = smem, *sB = smem + 2 * BM * 64;
    long long *roff = reinterpret_cast<long long *>(smem + C::LDS_BYTES);
    int *rs = reinterpret_cast<int *>(roff + BM);
    int *stap = rs + BM;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, kb = lane >> 4;
    // logical tile order: output-channel tiles fastest (they share the operand rows), then the stride
    // classes of one row tile: they write interleaved elements of the same result lines, and run
    // back to back on one XCD so that its L2 merges them before they go to memory
    const int ny = g.OC / BN, total = g.mtiles * g.ncls * ny;
    const int lg = q8t_gemm::xcd_logical(blockIdx.x, total);
    if (lg >= total) return;
    const int n0 = (lg % ny) * BN, zc = (lg / ny) % g.ncls, m0 = (lg / (ny * g.ncls)) * BM;
    {
        const int *ci = clsinfo + zc * CLS_INTS;
        g.OH = ci[0];
        g.OW = ci[1];
        g.M = ci[2];
        g.T = ci[4];
        g.oph = zc / g.osw;
        g.opw = zc - g.oph * g.osw;
        wt += (size_t)ci[3] * g.OC * g.Cp;
        tapoff += ci[3];
        colsum += (size_t)zc * g.OC;
    }
    if (m0 >= g.M) return;   // a smaller class: the whole workgroup leaves before any barrier
    const int za = qpa->zero_point - (1 << (qpa->bits - 1)), zb = qpb->zero_point - (1 << (qpb->bits - 1));
    const float sc = qpa->scale * qpb->scale;
    const int OHW = g.OH * g.OW;

    if (tid < g.T) stap[tid] = tapoff[tid];
    __syncthreads();
    // per-row bookkeeping: operand sum over the taps (padded taps count Cp zero codes) and the
    // offset of the row's position inside one output channel plane
    if (tid < BM) {
        const int m = m0 + tid;
        int sum = 0;
        long long off = -1;
        if (m < g.M) {
            const int n = m / OHW, rem = m - n * OHW;
            const int oh = rem / g.OW, ow = rem - oh * g.OW;
            for (int t = 0; t < g.T; ++t) {
                const int to = stap[t];
                const int ih = oh * g.ish + (int)(int16_t)(to & 0xFFFF), iw = ow * g.isw + (to >> 16);
                if ((unsigned)ih < (unsigned)g.IH && (unsigned)iw < (unsigned)g.IW)
                    sum += chansum[(n * g.IH + ih) * g.IW + iw];
                else
                    sum += g.Cp * za;
            }
            off = (long long)n * g.OC * g.OHf * g.OWf + (long long)(oh * g.osh + g.oph) * g.OWf + ow * g.osw + g.opw;
        }
        rs[tid] = sum;
        roff[tid] = off;
    }

    ConvOps<C> ops;
    ops.xin = xin;
    ops.wt = wt;
    ops.stap = (const __attribute__((address_space(3))) int *)stap;
    ops.IH = g.IH;
    ops.IW = g.IW;
    ops.Cp = g.Cp;
    ops.OC = g.OC;
    ops.CC = g.Cp >> 6;
    ops.q = tid & 3;
    ops.wrow = n0 + (tid >> 2);
    ops.padw = (uint32_t)(za & 255) * 0x01010101u;
    ops.lt = ops.lc = 0;
    {
        const int am = m0 + (tid >> 2);
        ops.av0 = am < g.M;
        ops.an0 = ops.ih0 = ops.iw0 = 0;
        if (ops.av0) {
            ops.an0 = am / OHW;
            const int rem = am - ops.an0 * OHW;
            const int oh = rem / g.OW;
            ops.ih0 = oh * g.ish;
            ops.iw0 = (rem - oh * g.OW) * g.isw;
        }
        const int bm = am + C::RP;
        ops.av1 = bm < g.M;
        ops.an1 = ops.ih1 = ops.iw1 = 0;
        if (ops.av1) {
            ops.an1 = bm / OHW;
            const int rem = bm - ops.an1 * OHW;
            const int oh = rem / g.OW;
            ops.ih1 = oh * g.ish;
            ops.iw1 = (rem - oh * g.OW) * g.isw;
        }
    }

    const int rowbase = C::rowbase(wave), colbase = C::colbase(wave);
    v4i acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (v4i){0, 0, 0, 0};

    q8t_gemm::pipeline<C>(ops, g.T * ops.CC, sA, sB, acc);
    if (g.T == 0) __syncthreads();   // rs / roff of the other threads

    // ---- epilogue: zero-point correction in wrapping 32-bit arithmetic (the corrected value fits
    // by contract), dequantization; a lane holds 4 consecutive rows of one output channel ----
    const uint32_t kzz = (uint32_t)(g.T * g.Cp) * (uint32_t)za * (uint32_t)zb;
    const long long plane = (long long)g.OHf * g.OWf;
    uint32_t csn[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) csn[nt] = (uint32_t)za * (uint32_t)colsum[n0 + colbase + nt * 16 + l16];
    // statistics of the lane's output channels over its rows, for the Range BN behind a forward product
    long long st_s[NT];
    int st_mn[NT], st_mx[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        st_s[nt] = 0;
        st_mn[nt] = 2147483647;
        st_mx[nt] = -2147483647 - 1;
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int r0 = rowbase + mt * 16 + kb * 4;
        long long o[4];
        uint32_t t[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            o[j] = roff[r0 + j];
            t[j] = kzz - (uint32_t)zb * (uint32_t)rs[r0 + j];
        }
        if (g.fill) {
            // result positions (2*oh, 2*ow): the lane's four rows are 8 consecutive floats of result row
            // 2*oh when they share an image row, and row 2*oh + 1 is all zeros
            const bool run = g.vec && o[0] >= 0 && o[1] == o[0] + 2 && o[2] == o[0] + 4 && o[3] == o[0] + 6;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const long long cb = (long long)(n0 + colbase + nt * 16 + l16) * plane;
                int c[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) c[j] = (int)((uint32_t)acc[mt][nt][j] + t[j] - csn[nt]);
                if (run && (((o[0] + cb) & 3) == 0)) {
                    const long long b0 = o[0] + cb, b1 = b0 + g.OWf;   // OWf is even: b1 is 8-byte aligned
                    if (out_acc) {
                        *reinterpret_cast<int4 *>(out_acc + b0) = make_int4(c[0], 0, c[1], 0);
                        *reinterpret_cast<int4 *>(out_acc + b0 + 4) = make_int4(c[2], 0, c[3], 0);
                        *reinterpret_cast<int2 *>(out_acc + b1) = make_int2(0, 0);
                        *reinterpret_cast<int2 *>(out_acc + b1 + 2) = make_int2(0, 0);
                        *reinterpret_cast<int2 *>(out_acc + b1 + 4) = make_int2(0, 0);
                        *reinterpret_cast<int2 *>(out_acc + b1 + 6) = make_int2(0, 0);
                    }
                    if (out_f) {
                        *reinterpret_cast<float4 *>(out_f + b0) = make_float4(sc * (float)c[0], 0.f, sc * (float)c[1], 0.f);
                        *reinterpret_cast<float4 *>(out_f + b0 + 4) = make_float4(sc * (float)c[2], 0.f, sc * (float)c[3], 0.f);
                        *reinterpret_cast<float2 *>(out_f + b1) = make_float2(0.f, 0.f);
                        *reinterpret_cast<float2 *>(out_f + b1 + 2) = make_float2(0.f, 0.f);
                        *reinterpret_cast<float2 *>(out_f + b1 + 4) = make_float2(0.f, 0.f);
                        *reinterpret_cast<float2 *>(out_f + b1 + 6) = make_float2(0.f, 0.f);
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        if (o[j] < 0) continue;
                        const long long b = o[j] + cb;
                        if (out_acc) {
                            out_acc[b] = c[j];
                            out_acc[b + 1] = 0;
                            out_acc[b + g.OWf] = 0;
                            out_acc[b + g.OWf + 1] = 0;
                        }
                        if (out_f) {
                            out_f[b] = sc * (float)c[j];
                            out_f[b + 1] = 0.f;
                            out_f[b + g.OWf] = 0.f;
                            out_f[b + g.OWf + 1] = 0.f;
                        }
                    }
                }
            }
            continue;
        }
        const bool contig = g.vec && o[0] >= 0 && o[1] == o[0] + 1 && o[2] == o[0] + 2 && o[3] == o[0] + 3;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const long long cb = (long long)(n0 + colbase + nt * 16 + l16) * plane;
            int c[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) c[j] = (int)((uint32_t)acc[mt][nt][j] + t[j] - csn[nt]);
            if (bnpart) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (o[j] >= 0) {
                        st_s[nt] += c[j];
                        st_mn[nt] = min(st_mn[nt], c[j]);
                        st_mx[nt] = max(st_mx[nt], c[j]);
                    }
            }
            if (contig && (((o[0] + cb) & 3) == 0)) {
                if (out_acc) *reinterpret_cast<int4 *>(out_acc + o[0] + cb) = make_int4(c[0], c[1], c[2], c[3]);
                if (out_f) {
                    float4 f;
                    f.x = sc * (float)c[0];
                    f.y = sc * (float)c[1];
                    f.z = sc * (float)c[2];
                    f.w = sc * (float)c[3];
                    *reinterpret_cast<float4 *>(out_f + o[0] + cb) = f;
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (o[j] < 0) continue;
                    if (out_acc) out_acc[o[j] + cb] = c[j];
                    if (out_f) out_f[o[j] + cb] = sc * (float)c[j];
                }
            }
        }
    }
    if (bnpart) {
        // fold the lanes that share a channel through LDS slots (the operand tiles are no longer needed)
        unsigned long long *slot_s = reinterpret_cast<unsigned long long *>(smem);
        int *slot_mn = reinterpret_cast<int *>(slot_s + BN), *slot_mx = slot_mn + BN;
        __syncthreads();
        if (tid < BN) {
            slot_s[tid] = 0;
            slot_mn[tid] = 2147483647;
            slot_mx[tid] = -2147483647 - 1;
        }
        __syncthreads();
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int ch = colbase + nt * 16 + l16;
            atomicAdd(&slot_s[ch], (unsigned long long)st_s[nt]);
            atomicMin(&slot_mn[ch], st_mn[nt]);
            atomicMax(&slot_mx[ch], st_mx[nt]);
        }
        __syncthreads();
        if (tid < BN) {
            const int k = n0 + tid;
            Q8tConvStat r;
            r.sum = (long long)slot_s[tid];
            r.mn = slot_mn[tid];
            r.mx = slot_mx[tid];
            bnpart[((size_t)(k >> 6) * g.mtiles + m0 / BM) * 64 + (k & 63)] = r;
        }
    }
}

// ---- layer gradient at stride 2: the two stride classes (ph, 0) and (ph, 1) in one workgroup -----
// Both classes enumerate the same positions (n, oh, ow) when the result width is even, and their
// results are neighbours in memory: (2*oh + ph, 2*ow) and (2*oh + ph, 2*ow + 1).  A workgroup runs the
// main loop once per class into two accumulator sets and writes 8-byte pairs (32-byte runs where a
// lane's four rows share an image row) instead of isolated 4-byte elements, which is what the L2
// request rate of a stride class on its own is bound by.
template <class C>
constexpr size_t conv_pair_lds_bytes()
{
    return conv_lds_bytes<C>() + C::BM * sizeof(int);
}

template <class C>
__global__ __launch_bounds__(C::THREADS, 2) void igemm_nhwc_pair(const int8_t *__restrict__ xin,
                                                                  const int *__restrict__ chansum,
                                                                  const int8_t *__restrict__ wt,
                                                                  const int *__restrict__ colsum,
                                                                  const q8t_qparams *__restrict__ qpa,
                                                                  const q8t_qparams *__restrict__ qpb, Geo g,
                                                                  const int *__restrict__ tapoff,
                                                                  const int *__restrict__ clsinfo,
                                                                  float *__restrict__ out_f, int32_t *__restrict__ out_acc)
{
    constexpr int MT = C::MT, NT = C::NT, BM = C::BM, BN = C::BN;
    extern __shared__ __align__(16) int8_t smem[];
    int8_t *sA = smem, *sB = smem + 2 * BM * 64;
    long long *roff = reinterpret_cast<long long *>(smem + C::LDS_BYTES);
    int *rsA = reinterpret_cast<int *>(roff + BM);
    int *rsB = rsA + BM;
    int *stap = rsB + BM;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, kb = lane >> 4;
    // logical tile order: output-channel tiles fastest, then the two row parities of one row tile
    const int ny = g.OC / BN, total = g.mtiles * 2 * ny;
    const int lg = q8t_gemm::xcd_logical(blockIdx.x, total);
    if (lg >= total) return;
    const int n0 = (lg % ny) * BN, ph = (lg / ny) & 1, m0 = (lg / (ny * 2)) * BM;
    const int *ciA = clsinfo + (ph * 2) * CLS_INTS, *ciB = ciA + CLS_INTS;
    const int OH = ciA[0], OW = ciA[1], M = ciA[2];
    const int TA = ciA[4], TB = ciB[4];
    if (m0 >= M) return;   // the whole workgroup leaves before any barrier
    const int za = qpa->zero_point - (1 << (qpa->bits - 1)), zb = qpb->zero_point - (1 << (qpb->bits - 1));
    const float sc = qpa->scale * qpb->scale;
    const int OHW = OH * OW;

    // the taps of the two classes are neighbours in the table
    if (tid < TA + TB) stap[tid] = tapoff[ciA[3] + tid];
    __syncthreads();
    if (tid < BM) {
        const int m = m0 + tid;
        int sumA = 0, sumB = 0;
        long long off = -1;
        if (m < M) {
            const int n = m / OHW, rem = m - n * OHW;
            const int oh = rem / OW, ow = rem - oh * OW;
            for (int t = 0; t < TA + TB; ++t) {
                const int to = stap[t];
                const int ih = oh + (int)(int16_t)(to & 0xFFFF), iw = ow + (to >> 16);
                const int v = (unsigned)ih < (unsigned)g.IH && (unsigned)iw < (unsigned)g.IW
                                  ? chansum[(n * g.IH + ih) * g.IW + iw]
                                  : g.Cp * za;
                sumA += t < TA ? v : 0;
                sumB += t < TA ? 0 : v;
            }
            off = (long long)n * g.OC * g.OHf * g.OWf + (long long)(oh * 2 + ph) * g.OWf + ow * 2;
        }
        rsA[tid] = sumA;
        rsB[tid] = sumB;
        roff[tid] = off;
    }
    __syncthreads();

    ConvOps<C> opsA;
    opsA.xin = xin;
    opsA.wt = wt + (size_t)ciA[3] * g.OC * g.Cp;
    opsA.stap = (const __attribute__((address_space(3))) int *)stap;
    opsA.IH = g.IH;
    opsA.IW = g.IW;
    opsA.Cp = g.Cp;
    opsA.OC = g.OC;
    opsA.CC = g.Cp >> 6;
    opsA.q = tid & 3;
    opsA.wrow = n0 + (tid >> 2);
    opsA.padw = (uint32_t)(za & 255) * 0x01010101u;
    opsA.lt = opsA.lc = 0;
    {
        const int am = m0 + (tid >> 2);
        opsA.av0 = am < M;
        opsA.an0 = opsA.ih0 = opsA.iw0 = 0;
        if (opsA.av0) {
            opsA.an0 = am / OHW;
            const int rem = am - opsA.an0 * OHW;
            opsA.ih0 = rem / OW;
            opsA.iw0 = rem - opsA.ih0 * OW;
        }
        const int bm = am + C::RP;
        opsA.av1 = bm < M;
        opsA.an1 = opsA.ih1 = opsA.iw1 = 0;
        if (opsA.av1) {
            opsA.an1 = bm / OHW;
            const int rem = bm - opsA.an1 * OHW;
            opsA.ih1 = rem / OW;
            opsA.iw1 = rem - opsA.ih1 * OW;
        }
    }
    ConvOps<C> opsB = opsA;
    opsB.wt = wt + (size_t)ciB[3] * g.OC * g.Cp;
    opsB.stap = (const __attribute__((address_space(3))) int *)(stap + TA);

    const int rowbase = C::rowbase(wave), colbase = C::colbase(wave);
    v4i accA[MT][NT], accB[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) accA[mt][nt] = accB[mt][nt] = (v4i){0, 0, 0, 0};

    q8t_gemm::pipeline<C>(opsA, TA * opsA.CC, sA, sB, accA);
    q8t_gemm::pipeline<C>(opsB, TB * opsB.CC, sA, sB, accB);

    // ---- epilogue: both classes corrected and dequantized, written as pairs ----
    const uint32_t kzzA = (uint32_t)(TA * g.Cp) * (uint32_t)za * (uint32_t)zb;
    const uint32_t kzzB = (uint32_t)(TB * g.Cp) * (uint32_t)za * (uint32_t)zb;
    const long long plane = (long long)g.OHf * g.OWf;
    const int *colA = colsum + (size_t)(ph * 2) * g.OC, *colB = colA + g.OC;
    uint32_t csA[NT], csB[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        csA[nt] = (uint32_t)za * (uint32_t)colA[n0 + colbase + nt * 16 + l16];
        csB[nt] = (uint32_t)za * (uint32_t)colB[n0 + colbase + nt * 16 + l16];
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int r0 = rowbase + mt * 16 + kb * 4;
        long long o[4];
        uint32_t tA[4], tB[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            o[j] = roff[r0 + j];
            tA[j] = kzzA - (uint32_t)zb * (uint32_t)rsA[r0 + j];
            tB[j] = kzzB - (uint32_t)zb * (uint32_t)rsB[r0 + j];
        }
        const bool run = g.vec && o[0] >= 0 && o[1] == o[0] + 2 && o[2] == o[0] + 4 && o[3] == o[0] + 6;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const long long cb = (long long)(n0 + colbase + nt * 16 + l16) * plane;
            int a[4], b[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                a[j] = (int)((uint32_t)accA[mt][nt][j] + tA[j] - csA[nt]);
                b[j] = (int)((uint32_t)accB[mt][nt][j] + tB[j] - csB[nt]);
            }
            if (run && (((o[0] + cb) & 3) == 0)) {
                if (out_acc) {
                    *reinterpret_cast<int4 *>(out_acc + o[0] + cb) = make_int4(a[0], b[0], a[1], b[1]);
                    *reinterpret_cast<int4 *>(out_acc + o[0] + cb + 4) = make_int4(a[2], b[2], a[3], b[3]);
                }
                if (out_f) {
                    *reinterpret_cast<float4 *>(out_f + o[0] + cb) =
                        make_float4(sc * (float)a[0], sc * (float)b[0], sc * (float)a[1], sc * (float)b[1]);
                    *reinterpret_cast<float4 *>(out_f + o[0] + cb + 4) =
                        make_float4(sc * (float)a[2], sc * (float)b[2], sc * (float)a[3], sc * (float)b[3]);
                }
            } else if (g.vec) {   // even result width and plane: every pair is 8-byte aligned
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (o[j] < 0) continue;
                    if (out_acc) *reinterpret_cast<int2 *>(out_acc + o[j] + cb) = make_int2(a[j], b[j]);
                    if (out_f) *reinterpret_cast<float2 *>(out_f + o[j] + cb) = make_float2(sc * (float)a[j], sc * (float)b[j]);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (o[j] < 0) continue;
                    if (out_acc) {
                        out_acc[o[j] + cb] = a[j];
                        out_acc[o[j] + cb + 1] = b[j];
                    }
                    if (out_f) {
                        out_f[o[j] + cb] = sc * (float)a[j];
                        out_f[o[j] + cb + 1] = sc * (float)b[j];
                    }
                }
            }
        }
    }
}

// Stage the R input rows under output row p of image n, for every channel, into LDS:
// rows[(c*R + r)*pitch + L + w] = x[n][c][p*stride + r - pad][w], the zero code everywhere else
// (padding rows and columns).  L = pad rounded up to a multiple of 4 and pitch a multiple of 4, so
// that aligned dwords of the input are aligned dwords of a staged row.  All loads of a pass are
// issued before the first LDS store: a workgroup's input is a few KB and the pass would otherwise
// be a chain of exposed memory latencies.
__device__ __forceinline__ void stage_rows(const int8_t *__restrict__ x, int n, int C, int H, int W, int R, int stride,
                                           int pad, int p, int L, int pitch, int za, bool vec4, int8_t *rows)
{
    constexpr int U = 6;
    const int CR = C * R, tid = threadIdx.x;
    {
        uint32_t *r32 = reinterpret_cast<uint32_t *>(rows);
        const uint32_t fill = (uint32_t)(za & 255) * 0x01010101u;
        for (int i = tid; i < (CR * pitch) >> 2; i += kThreads) r32[i] = fill;
    }
    __syncthreads();
    if (vec4) {
        const int W4 = W >> 2, items = CR * W4;
        for (int i0 = 0; i0 < items; i0 += kThreads * U) {
            uint32_t v[U];
            int dst[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + u * kThreads + tid;
                dst[u] = -1;
                v[u] = 0;
                if (i < items) {
                    const int cr = i / W4, w4 = i - cr * W4, c = cr / R, r = cr - c * R;
                    const int h = p * stride + r - pad;
                    if ((unsigned)h < (unsigned)H) {
                        v[u] = *reinterpret_cast<const uint32_t *>(x + (((size_t)n * C + c) * H + h) * W + w4 * 4);
                        dst[u] = cr * pitch + L + w4 * 4;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (dst[u] >= 0) *reinterpret_cast<uint32_t *>(rows + dst[u]) = v[u];
        }
    } else {
        const int items = CR * W;
        for (int i0 = 0; i0 < items; i0 += kThreads * U) {
            int8_t v[U];
            int dst[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int i = i0 + u * kThreads + tid;
                dst[u] = -1;
                v[u] = 0;
                if (i < items) {
                    const int cr = i / W, w = i - cr * W, c = cr / R, r = cr - c * R;
                    const int h = p * stride + r - pad;
                    if ((unsigned)h < (unsigned)H) {
                        v[u] = x[(((size_t)n * C + c) * H + h) * W + w];
                        dst[u] = cr * pitch + L + w;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (dst[u] >= 0) rows[dst[u]] = v[u];
        }
    }
}

// ---- forward with few input channels (the network's first layer) --------------------------------
// The reduction (c, r, s) of an output position is laid out explicitly: xn[m][Kc] with
// Kc = C*R*S rounded up to a multiple of 64, entry c*R*S + r*S + s = the input code under that tap
// (zero code in the padding and in the surplus columns), plus the row sum.  With the filter as
// [K][Kc] (zeros in the surplus columns) the product is a 1x1 problem for igemm_nhwc.
// One workgroup per (image, output row): the R input rows of every channel go to LDS once.
__global__ __launch_bounds__(kThreads) void im2col_positions(const int8_t *__restrict__ x, int C, int H, int W, int R, int S,
                                                             int stride, int pad, int P, int Q, int Kc,
                                                             const q8t_qparams *__restrict__ qpx,
                                                             int8_t *__restrict__ xn, int *__restrict__ rowsum, int vec4)
{
    extern __shared__ __align__(16) int8_t lds[];
    const int CRS = C * R * S;
    const int L = (pad + 3) & ~3, Wp = (L + W + pad + 3) & ~3;   // staged row: left margin, pitch
    int8_t *rows = lds;                                   // [C*R][Wp]
    int *lut = reinterpret_cast<int *>(lds + ((C * R * Wp + 15) & ~15));   // [Kc]: offset of column j in `rows`, -1: surplus
    int *rsum = lut + Kc;                                                   // [Q]
    const int n = blockIdx.y, p = blockIdx.x, tid = threadIdx.x;
    const int zsx = qpx->zero_point - (1 << (qpx->bits - 1));
    stage_rows(x, n, C, H, W, R, stride, pad, p, L, Wp, zsx, vec4 != 0, rows);
    for (int q = tid; q < Q; q += kThreads) rsum[q] = 0;
    for (int j = tid; j < Kc; j += kThreads) {
        int off = -1;
        if (j < CRS) {
            const int c = j / (R * S), t = j - c * R * S, r = t / S, s2 = t - r * S;
            off = (c * R + r) * Wp + L - pad + s2;
        }
        lut[j] = off;
    }
    __syncthreads();
    const int chunks = Kc >> 4;
    const size_t m0 = ((size_t)n * P + p) * Q;
    const uint32_t zb = (uint32_t)(zsx & 255);
    for (int it = tid; it < Q * chunks; it += kThreads) {
        const int q = it / chunks, ch = it - q * chunks;
        const int base = q * stride;
        uint32_t w4[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            uint32_t v = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int off = lut[ch * 16 + d * 4 + e];
                const uint32_t b = off >= 0 ? (uint32_t)(uint8_t)rows[off + base] : zb;
                v |= b << (8 * e);
            }
            w4[d] = v;
        }
        *reinterpret_cast<uint4 *>(xn + (m0 + q) * Kc + ch * 16) = make_uint4(w4[0], w4[1], w4[2], w4[3]);
        // row sums: every column of a position, surplus columns included
        atomicAdd(&rsum[q], bytesum4(w4[0]) + bytesum4(w4[1]) + bytesum4(w4[2]) + bytesum4(w4[3]));
    }
    __syncthreads();
    for (int q = tid; q < Q; q += kThreads) rowsum[m0 + q] = rsum[q];
}

// The same forward in one kernel, for reductions of at most 256 columns: the rows of xn never leave
// the compute unit.  One workgroup per (image, output row): the R input rows of every channel are
// staged as above, the (position x Kc) operand tile is built in LDS in the fragment layout of
// gemm_core.h, the [64][Kc] filter block sits beside it, and the four wavefronts multiply 16-row
// tiles of positions against the 64 output channels.  HBM sees the int8 input once and the fp32
// result once, instead of xn written and read back (Kc bytes per output position each way).
// Column order of the fused form: the S taps of one (channel, filter row) are S consecutive bytes of
// a staged row; they become a group of GP = 4 or 8 columns (the surplus ones hold the zero code and
// meet zero filter entries), so that a 16-byte chunk of an operand row is 16 / GP unaligned LDS
// reads of GP bytes instead of 16 single bytes.
constexpr int FUSED_MAXQ = 128;   // positions per pass
template <int GP>
__global__ __launch_bounds__(kThreads) void smallc_fused(const int8_t *__restrict__ x, int C, int H, int W, int R, int S,
                                                         int stride, int pad, int P, int Q, int Kc, int K,
                                                         const int8_t *__restrict__ wt, const int *__restrict__ colsum,
                                                         const q8t_qparams *__restrict__ qpx,
                                                         const q8t_qparams *__restrict__ qpw, float *__restrict__ out_f,
                                                         int32_t *__restrict__ out_acc, int vec, int vec4, int RPB,
                                                         Q8tConvStat *__restrict__ bnpart)
{
    constexpr int U = 6;   // dwords of input a thread carries from one output row to the next
    extern __shared__ __align__(16) int8_t lds[];
    const int KS = Kc >> 6;
    const int L = (pad + 3) & ~3, Wp = (L + W + pad + 3) & ~3;   // staged row: left margin, pitch
    int8_t *sA = lds;                                   // [KS][128][64]
    int8_t *sB = sA + KS * FUSED_MAXQ * 64;             // [KS][64][64]
    int *rsum = reinterpret_cast<int *>(sB + KS * 64 * 64);   // [128]
    int8_t *rows = reinterpret_cast<int8_t *>(rsum + FUSED_MAXQ);   // [C*R][Wp] + 16 bytes of slack
    const int n = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pbeg = blockIdx.x * RPB, pend = min(P, pbeg + RPB);
    const int l16 = lane & 15, kb = lane >> 4;
    const int za = qpx->zero_point - (1 << (qpx->bits - 1)), zb = qpw->zero_point - (1 << (qpw->bits - 1));
    const float sc = qpx->scale * qpw->scale;
    const int CR = C * R;
    const int chunks = Kc >> 4;
    const float rchunks = 1.0f / (float)chunks;
    const uint32_t zbyte = (uint32_t)(za & 255);
    const uint32_t kzz = (uint32_t)Kc * (uint32_t)za * (uint32_t)zb;
    // The workgroup walks RPB output rows.  When the input rows under one output row fit into U dwords
    // per thread, the loads for the next output row are issued before the current one is multiplied
    // and land in LDS afterwards: their latency is off the critical path.  Margins keep the zero code
    // from the one fill below; rows outside the image are rewritten with it every time.
    const int W4 = W >> 2, items = CR * W4;
    const bool carry = vec4 && items <= kThreads * U;
    const bool filter_once = K == 64;
    // statistics of the lane's four output channels (bnpart is only given with one block of 64 channels)
    long long st_s[4] = {0, 0, 0, 0};
    int st_mn[4], st_mx[4];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
        st_mn[nt] = 2147483647;
        st_mx[nt] = -2147483647 - 1;
    }
    uint32_t pv[U];
    int pd[U], prow[U];        // LDS offset of the thread's dword (-1: none); filter row minus padding
    const int8_t *psrc[U];     // its source, at input row 0
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int i = u * kThreads + tid;
        pd[u] = -1;
        prow[u] = 0;
        psrc[u] = x;
        if (carry && i < items) {
            const int cr = i / W4, w4 = i - cr * W4, c = cr / R, r = cr - c * R;
            pd[u] = cr * Wp + L + w4 * 4;
            prow[u] = r - pad;
            psrc[u] = x + ((size_t)n * C + c) * H * W + w4 * 4;
        }
    }
    auto issue = [&](int p) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int h = p * stride + prow[u];
            pv[u] = zbyte * 0x01010101u;
            if (pd[u] >= 0 && (unsigned)h < (unsigned)H) pv[u] = *reinterpret_cast<const uint32_t *>(psrc[u] + (size_t)h * W);
        }
    };
    auto load_filter = [&](int k0) {
        for (int it = tid; it < 64 * chunks; it += kThreads) {
            const int row = it / chunks, ch = it - row * chunks;
            const uint4 v = *reinterpret_cast<const uint4 *>(wt + (size_t)(k0 + row) * Kc + ch * 16);
            *reinterpret_cast<uint4 *>(sB + (ch >> 2) * (64 * 64) + row * 64 + (((ch & 3) ^ q8t_gemm::swz(row)) * 16)) = v;
        }
    };
    if (carry) {
        issue(pbeg);
        uint32_t *r32 = reinterpret_cast<uint32_t *>(rows);
        for (int i = tid; i < (CR * Wp + 16) >> 2; i += kThreads) r32[i] = zbyte * 0x01010101u;
    }
    if (filter_once) load_filter(0);
    // with a single group of 64 output channels the column terms of the epilogue are loaded once
    uint32_t cs_once[4] = {0u, 0u, 0u, 0u};
    if (filter_once) {
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) cs_once[nt] = (uint32_t)za * (uint32_t)colsum[nt * 16 + l16];
    }
    for (int p = pbeg; p < pend; ++p) {
        if (carry) {
            __syncthreads();   // the fill, or the previous output row's operand tile, is done with `rows`
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (pd[u] >= 0) *reinterpret_cast<uint32_t *>(rows + pd[u]) = pv[u];
            if (p + 1 < pend) issue(p + 1);
        } else {
            __syncthreads();
            stage_rows(x, n, C, H, W, R, stride, pad, p, L, Wp, za, vec4 != 0, rows);
        }
        for (int k0 = 0; k0 < K; k0 += 64) {
            for (int q0 = 0; q0 < Q; q0 += FUSED_MAXQ) {
                const int qc = min(FUSED_MAXQ, Q - q0);
                __syncthreads();   // staged rows ready; the previous pass has left sA / sB / rsum
                if (tid < FUSED_MAXQ) rsum[tid] = 0;
                if (!filter_once) load_filter(k0);
                __syncthreads();   // rsum cleared before the sums below
                // operand tile: rows = positions q0 .. q0 + qc (the rest of the last 16-row tile holds the zero code)
                const int qpad = (qc + 15) & ~15;
                for (int it = tid; it < qpad * chunks; it += kThreads) {
                    // q = it / chunks for it < 2^11 * 16 through the float reciprocal, corrected by at most one
                    int q = (int)((float)it * rchunks);
                    q += (it - q * chunks >= chunks) ? 1 : 0;
                    q -= (it - q * chunks < 0) ? 1 : 0;
                    const int ch = it - q * chunks;
                    uint32_t w4[4] = {zbyte * 0x01010101u, zbyte * 0x01010101u, zbyte * 0x01010101u, zbyte * 0x01010101u};
                    if (q < qc) {
                        const int base = (q0 + q) * stride + L - pad;
                        if (GP == 8) {
                            const uint64_t keep = S >= 8 ? ~0ull : ((1ull << (8 * S)) - 1);
                            const uint64_t fill = (uint64_t)zbyte * 0x0101010101010101ull;
#pragma unroll
                            for (int t = 0; t < 2; ++t) {
                                const int g = ch * 2 + t;
                                uint64_t v = fill;
                                if (g < CR) {
                                    __builtin_memcpy(&v, rows + g * Wp + base, 8);
                                    v = (v & keep) | (fill & ~keep);
                                }
                                w4[2 * t] = (uint32_t)v;
                                w4[2 * t + 1] = (uint32_t)(v >> 32);
                            }
                        } else {
                            const uint32_t keep = S >= 4 ? ~0u : ((1u << (8 * S)) - 1);
                            const uint32_t fill = zbyte * 0x01010101u;
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                const int g = ch * 4 + t;
                                uint32_t v = fill;
                                if (g < CR) {
                                    __builtin_memcpy(&v, rows + g * Wp + base, 4);
                                    v = (v & keep) | (fill & ~keep);
                                }
                                w4[t] = v;
                            }
                        }
                        atomicAdd(&rsum[q], bytesum4(w4[0]) + bytesum4(w4[1]) + bytesum4(w4[2]) + bytesum4(w4[3]));
                    }
                    *reinterpret_cast<uint4 *>(sA + (ch >> 2) * (FUSED_MAXQ * 64) + q * 64 +
                                               (((ch & 3) ^ q8t_gemm::swz(q)) * 16)) = make_uint4(w4[0], w4[1], w4[2], w4[3]);
                }
                __syncthreads();
                // wavefront w: 16-row tiles w and w + 4, all four 16-channel tiles
                v4i acc[2][4];
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[i][j] = (v4i){0, 0, 0, 0};
                const int mtiles = qpad >> 4;
                for (int ks = 0; ks < KS; ++ks) {
                    v4i bf[4];
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt) {
                        const int row = nt * 16 + l16;
                        bf[nt] = *reinterpret_cast<const v4i *>(sB + ks * (64 * 64) + row * 64 + ((kb ^ q8t_gemm::swz(row)) * 16));
                    }
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        const int mt = wave + i * 4;
                        if (mt < mtiles) {   // uniform per wavefront
                            const int row = mt * 16 + l16;
                            const v4i af = *reinterpret_cast<const v4i *>(sA + ks * (FUSED_MAXQ * 64) + row * 64 +
                                                                          ((kb ^ q8t_gemm::swz(row)) * 16));
#pragma unroll
                            for (int nt = 0; nt < 4; ++nt)
                                acc[i][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af, bf[nt], acc[i][nt], 0, 0, 0);
                        }
                    }
                }
                // epilogue: a lane holds 4 consecutive positions of one output channel
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int mt = wave + i * 4;
                    if (mt >= mtiles) continue;
                    const int r0 = mt * 16 + kb * 4;
                    uint32_t t[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) t[j] = kzz - (uint32_t)zb * (uint32_t)rsum[r0 + j];
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt) {
                        const int k = k0 + nt * 16 + l16;
                        const uint32_t cs = filter_once ? cs_once[nt] : (uint32_t)za * (uint32_t)colsum[k];
                        int c4[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) c4[j] = (int)((uint32_t)acc[i][nt][j] + t[j] - cs);
                        if (bnpart) {
#pragma unroll
                            for (int j = 0; j < 4; ++j)
                                if (r0 + j < qc) {
                                    st_s[nt] += c4[j];
                                    st_mn[nt] = min(st_mn[nt], c4[j]);
                                    st_mx[nt] = max(st_mx[nt], c4[j]);
                                }
                        }
                        const size_t o = (((size_t)n * K + k) * P + p) * Q + q0 + r0;
                        if (vec && r0 + 3 < qc) {
                            if (out_acc) *reinterpret_cast<int4 *>(out_acc + o) = make_int4(c4[0], c4[1], c4[2], c4[3]);
                            if (out_f)
                                *reinterpret_cast<float4 *>(out_f + o) =
                                    make_float4(sc * (float)c4[0], sc * (float)c4[1], sc * (float)c4[2], sc * (float)c4[3]);
                        } else {
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                if (r0 + j >= qc) continue;
                                if (out_acc) out_acc[o + j] = c4[j];
                                if (out_f) out_f[o + j] = sc * (float)c4[j];
                            }
                        }
                    }
                }
            }
        }
    }
    if (bnpart) {
        // fold the 16 lanes that share a channel through LDS slots (the operand tile is no longer needed)
        unsigned long long *slot_s = reinterpret_cast<unsigned long long *>(lds);
        int *slot_mn = reinterpret_cast<int *>(slot_s + 64), *slot_mx = slot_mn + 64;
        __syncthreads();
        if (tid < 64) {
            slot_s[tid] = 0;
            slot_mn[tid] = 2147483647;
            slot_mx[tid] = -2147483647 - 1;
        }
        __syncthreads();
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            atomicAdd(&slot_s[nt * 16 + l16], (unsigned long long)st_s[nt]);
            atomicMin(&slot_mn[nt * 16 + l16], st_mn[nt]);
            atomicMax(&slot_mx[nt * 16 + l16], st_mx[nt]);
        }
        __syncthreads();
        if (tid < 64) {
            Q8tConvStat r;
            r.sum = (long long)slot_s[tid];
            r.mn = slot_mn[tid];
            r.mx = slot_mx[tid];
            bnpart[((size_t)blockIdx.y * gridDim.x + blockIdx.x) * 64 + tid] = r;
        }
    }
}

// filter [K][C*R*S] -> [K][Kc] in the grouped column order of smallc_fused (column g*GP + s = entry
// (g, s) of the (channel, filter row) group g; zeros elsewhere), sums per output channel
__global__ __launch_bounds__(kThreads) void repack_grouped(const int8_t *__restrict__ w, int CRS, int CR, int S, int GP, int Kc,
                                                           int8_t *__restrict__ wt, int *__restrict__ colsum)
{
    __shared__ int part[kThreads / 64];
    const int k = blockIdx.x;
    int sum = 0;
    for (int j = threadIdx.x; j < Kc; j += kThreads) {
        const int g = j / GP, s2 = j - g * GP;
        const int8_t v = (g < CR && s2 < S) ? w[(size_t)k * CRS + g * S + s2] : (int8_t)0;
        wt[(size_t)k * Kc + j] = v;
        sum += v;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, Q8T_WAVE);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) colsum[k] = part[0] + part[1] + part[2] + part[3];
}

// filter [K][C*R*S] -> [K][Kc] with zero surplus columns, sums per output channel, tap offset 0
__global__ __launch_bounds__(kThreads) void repack_flat(const int8_t *__restrict__ w, int CRS, int Kc, int OH, int OW,
                                                        int M, int8_t *__restrict__ wt, int *__restrict__ colsum,
                                                        int *__restrict__ tapoff, int *__restrict__ clsinfo)
{
    __shared__ int part[kThreads / 64];
    const int k = blockIdx.x;
    int sum = 0;
    for (int j = threadIdx.x; j < Kc; j += kThreads) {
        const int8_t v = j < CRS ? w[(size_t)k * CRS + j] : (int8_t)0;
        wt[(size_t)k * Kc + j] = v;
        sum += v;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, Q8T_WAVE);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        colsum[k] = part[0] + part[1] + part[2] + part[3];
        if (k == 0) {
            tapoff[0] = 0;
            clsinfo[0] = OH;
            clsinfo[1] = OW;
            clsinfo[2] = M;
            clsinfo[3] = 0;
            clsinfo[4] = 1;
        }
    }
}

struct SmallPlan {
    int P, Q, Kc;
    int GP, Kf;   // fused form: columns per (channel, filter row) group (0: not available), padded reduction
    bool fused;   // the fused kernel runs (decided from the shape alone, so the workspace query agrees with the call)
    size_t lds, o_rowsum, o_wt, o_colsum, o_tapoff, total;
};

inline size_t up256s(size_t v) { return (v + 255) & ~(size_t)255; }

// forward only: fewer than 64 input channels, output channels a multiple of 64
bool make_small_plan(int which, const q8t_conv_desc *d, SmallPlan *p)
{
    if (which != 0) return false;
    if (d->N <= 0 || d->C <= 0 || d->C >= 64 || d->K <= 0 || d->K % 64 || d->H <= 0 || d->W <= 0) return false;
    if (d->R <= 0 || d->S <= 0 || d->R > 100 || d->S > 100 || d->stride < 1 || d->pad < 0 || d->pad > 100) return false;
    if (d->H + 2 * d->pad < d->R || d->W + 2 * d->pad < d->S) return false;
    const int64_t crs = (int64_t)d->C * d->R * d->S;
    if (crs > 1024) return false;
    p->Kc = (int)((crs + 63) / 64 * 64);
    p->P = (d->H + 2 * d->pad - d->R) / d->stride + 1;
    p->Q = (d->W + 2 * d->pad - d->S) / d->stride + 1;
    if (d->N > 65535) return false;
    const int64_t M = (int64_t)d->N * p->P * p->Q;
    if (M >= ((int64_t)1 << 31) || (int64_t)d->N * d->C * d->H >= ((int64_t)1 << 31)) return false;
    p->lds = (((size_t)d->C * d->R * ((((d->pad + 3) & ~3) + d->W + d->pad + 3) & ~3) + 15) & ~(size_t)15) +
             ((size_t)p->Kc + p->Q) * sizeof(int);
    if (p->lds > 65536) return false;
    p->GP = d->S <= 4 ? 4 : (d->S <= 8 ? 8 : 0);
    p->Kf = p->GP ? (int)(((int64_t)d->C * d->R * p->GP + 63) / 64 * 64) : 0;
    if (p->Kf > 256) p->GP = p->Kf = 0;
    // the fused kernel (operand tile, filter block, row sums and staged rows in 64 KB of LDS) needs neither the
    // explicit im2col rows nor their row sums in the workspace: for the first layer of a ResNet at batch 256 those
    // would be 630 MB that nothing touches
    {
        const int Ls = (d->pad + 3) & ~3, pitch = (Ls + d->W + d->pad + 3) & ~3;
        const size_t fused_lds = (size_t)(p->Kf >> 6) * (FUSED_MAXQ + 64) * 64 + (size_t)FUSED_MAXQ * sizeof(int) +
                                 (((size_t)d->C * d->R * pitch + 15) & ~(size_t)15) + 16;
        p->fused = p->GP && fused_lds <= 65536;
    }
    p->o_rowsum = p->fused ? 0 : up256s((size_t)M * p->Kc);
    p->o_wt = p->o_rowsum + (p->fused ? 0 : up256s((size_t)M * sizeof(int)));
    p->o_colsum = p->o_wt + up256s((size_t)d->K * (p->Kc > p->Kf ? p->Kc : p->Kf));
    p->o_tapoff = p->o_colsum + up256s((size_t)d->K * sizeof(int));
    p->total = p->o_tapoff + 256;
    return true;
}

struct Plan {
    int red, oc;          // reduction and output channels
    int IH, IW;           // operand spatial size
    int OHf, OWf;         // result spatial size
    int ncls;             // stride classes
    size_t o_chansum, o_wt, o_colsum, o_tapoff, o_cls, total;
};

inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

bool make_plan(int which, const q8t_conv_desc *d, Plan *p)
{
    if (which < 0 || which > 1) return false;
    if (d->N <= 0 || d->C <= 0 || d->K <= 0 || d->H <= 0 || d->W <= 0 || d->R <= 0 || d->S <= 0) return false;
    if (d->stride < 1 || d->stride > 4 || d->pad < 0 || d->pad > 100) return false;
    if (d->R * d->S > MAXT || d->R > 100 || d->S > 100) return false;
    if (d->H + 2 * d->pad < d->R || d->W + 2 * d->pad < d->S) return false;
    const int P = (d->H + 2 * d->pad - d->R) / d->stride + 1, Q = (d->W + 2 * d->pad - d->S) / d->stride + 1;
    p->red = which == 0 ? d->C : d->K;
    p->oc = which == 0 ? d->K : d->C;
    if (p->red % 64 || p->oc % 64) return false;
    p->IH = which == 0 ? d->H : P;
    p->IW = which == 0 ? d->W : Q;
    p->OHf = which == 0 ? P : d->H;
    p->OWf = which == 0 ? Q : d->W;
    p->ncls = which == 0 ? 1 : d->stride * d->stride;
    const int64_t ipos = (int64_t)d->N * p->IH * p->IW, opos = (int64_t)d->N * p->OHf * p->OWf;
    if (ipos >= ((int64_t)1 << 31) || opos >= ((int64_t)1 << 31)) return false;
    if ((int64_t)d->N * (which == 0 ? d->C : d->K) >= ((int64_t)1 << 31)) return false;
    const size_t xn = up256((size_t)ipos * p->red);
    p->o_chansum = xn;
    p->o_wt = p->o_chansum + up256((size_t)ipos * sizeof(int));
    p->o_colsum = p->o_wt + up256((size_t)d->K * d->C * d->R * d->S);
    p->o_tapoff = p->o_colsum + up256((size_t)p->ncls * p->oc * sizeof(int));
    p->o_cls = p->o_tapoff + up256((MAXT + 3) * sizeof(int));
    p->total = p->o_cls + up256((size_t)MAXCLS * CLS_INTS * sizeof(int));
    return true;
}

}  // namespace

bool q8t_smallc_conv_supported(int which, const q8t_conv_desc *d)
{
    SmallPlan p;
    return make_small_plan(which, d, &p);
}

size_t q8t_smallc_conv_ws(int which, const q8t_conv_desc *d)
{
    SmallPlan p;
    return make_small_plan(which, d, &p) ? p.total : 0;
}

namespace {
// the fused kernel runs (operand tile, filter block, row sums and staged rows fit into 64 KB of LDS)
bool smallc_is_fused(const q8t_conv_desc *d, const SmallPlan &p)
{
    (void)d;
    return p.fused;
}
constexpr int kSmallRPB = 4;   // output rows per workgroup of the fused kernel
}  // namespace

size_t q8t_smallc_conv_stats_ws(const q8t_conv_desc *d)
{
    SmallPlan p;
    if (!make_small_plan(0, d, &p) || d->K != 64 || !smallc_is_fused(d, p)) return 0;
    return (size_t)((p.P + kSmallRPB - 1) / kSmallRPB) * d->N * 64 * sizeof(Q8tConvStat);
}

int q8t_smallc_conv(const q8t_conv_desc *d, const void *a, const q8t_qparams *qa, const void *b, const q8t_qparams *qb,
                    float *out_f, void *out_acc, float *bn_stats, void *stats_ws, void *ws, hipStream_t st)
{
    SmallPlan p;
    if (!make_small_plan(0, d, &p)) return Q8T_ERR_SHAPE;
    if (!ws || !q8t_aligned(ws, 16)) return Q8T_ERR_WORKSPACE;
    if (bn_stats && (!q8t_smallc_conv_stats_ws(d) || !stats_ws || !q8t_aligned(stats_ws, 16))) return Q8T_ERR_WORKSPACE;
    Q8tConvStat *bnp = bn_stats ? (Q8tConvStat *)stats_ws : (Q8tConvStat *)nullptr;
    int8_t *xn = (int8_t *)ws;
    int *rowsum = (int *)((char *)ws + p.o_rowsum);
    int8_t *wt = (int8_t *)ws + p.o_wt;
    int *colsum = (int *)((char *)ws + p.o_colsum);
    int *tapoff = (int *)((char *)ws + p.o_tapoff);
    // fused form: operand tile, filter block, row sums and staged rows all in LDS
    const int Ls = (d->pad + 3) & ~3, pitch = (Ls + d->W + d->pad + 3) & ~3;
    const int vec4 = d->W % 4 == 0 && q8t_aligned(a, 4);
    const size_t fused_lds = (size_t)(p.Kf >> 6) * (FUSED_MAXQ + 64) * 64 + (size_t)FUSED_MAXQ * sizeof(int) +
                             (((size_t)d->C * d->R * pitch + 15) & ~(size_t)15) + 16;
    if (p.fused) {
        hipLaunchKernelGGL(repack_grouped, dim3((unsigned)d->K), dim3(kThreads), 0, st, (const int8_t *)b,
                           d->C * d->R * d->S, d->C * d->R, d->S, p.GP, p.Kf, wt, colsum);
        Q8T_LAUNCH_CHECK();
        // 16-byte stores need rows of the result that start on 16 bytes
        const int vec = p.Q % 4 == 0 && q8t_aligned(out_f, 16) && q8t_aligned(out_acc, 16);
        const int RPB = kSmallRPB;
        const dim3 grid((unsigned)((p.P + RPB - 1) / RPB), (unsigned)d->N);
        if (p.GP == 8)
            hipLaunchKernelGGL(smallc_fused<8>, grid, dim3(kThreads), fused_lds, st, (const int8_t *)a, d->C, d->H, d->W, d->R,
                               d->S, d->stride, d->pad, p.P, p.Q, p.Kf, d->K, wt, colsum, qa, qb, out_f, (int32_t *)out_acc,
                               vec, vec4, RPB, bnp);
        else
            hipLaunchKernelGGL(smallc_fused<4>, grid, dim3(kThreads), fused_lds, st, (const int8_t *)a, d->C, d->H, d->W, d->R,
                               d->S, d->stride, d->pad, p.P, p.Q, p.Kf, d->K, wt, colsum, qa, qb, out_f, (int32_t *)out_acc,
                               vec, vec4, RPB, bnp);
        Q8T_LAUNCH_CHECK();
        if (bnp) {
            const int nwg = (int)(grid.x * grid.y);
            return q8t_conv_stats_finalize(bnp, 64, nwg, nwg, (double)d->N * p.P * p.Q, qa, qb, bn_stats, st);
        }
        return Q8T_OK;
    }
    int *clsinfo = tapoff + 8;   // the tap table of this path has one entry
    hipLaunchKernelGGL(repack_flat, dim3((unsigned)d->K), dim3(kThreads), 0, st, (const int8_t *)b, d->C * d->R * d->S, p.Kc,
                       p.P, p.Q, d->N * p.P * p.Q, wt, colsum, tapoff, clsinfo);
    Q8T_LAUNCH_CHECK();
    hipLaunchKernelGGL(im2col_positions, dim3((unsigned)p.P, (unsigned)d->N), dim3(kThreads), p.lds, st, (const int8_t *)a,
                       d->C, d->H, d->W, d->R, d->S, d->stride, d->pad, p.P, p.Q, p.Kc, qa, xn, rowsum, vec4);
    Q8T_LAUNCH_CHECK();
    Geo g;
    g.N = d->N;
    g.IH = p.P;
    g.IW = p.Q;
    g.Cp = p.Kc;
    g.OH = p.P;
    g.OW = p.Q;
    g.ish = g.isw = 1;
    g.OC = d->K;
    g.OHf = p.P;
    g.OWf = p.Q;
    g.osh = g.osw = 1;
    g.oph = g.opw = 0;
    g.M = d->N * p.P * p.Q;
    g.T = 1;
    g.vec = q8t_aligned(out_f, 16) && q8t_aligned(out_acc, 16);
    g.ncls = 1;
    g.fill = 0;
#define Q8T_GO(CFG)                                                                                                   \
    {                                                                                                                 \
        g.mtiles = (g.M + CFG::BM - 1) / CFG::BM;                                                                     \
        const int64_t tiles = (int64_t)g.mtiles * (d->K / CFG::BN);                                                   \
        hipLaunchKernelGGL(igemm_nhwc<CFG>, dim3(q8t_gemm::xcd_grid(tiles)), dim3(CFG::THREADS), conv_lds_bytes<CFG>(), \
                           st, xn, rowsum, wt, colsum, qa, qb, g, tapoff, clsinfo, out_f, (int32_t *)out_acc,         \
                           (Q8tConvStat *)nullptr);                                                                \
    }
    if (d->K % 128 == 0) Q8T_GO(q8t_gemm::Mid)
    else Q8T_GO(q8t_gemm::Small)
#undef Q8T_GO
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

bool q8t_nhwc_conv_supported(int which, const q8t_conv_desc *d)
{
    Plan p;
    return make_plan(which, d, &p);
}

size_t q8t_nhwc_conv_ws(int which, const q8t_conv_desc *d)
{
    Plan p;
    return make_plan(which, d, &p) ? p.total : 0;
}

size_t q8t_nhwc_conv_stats_ws(const q8t_conv_desc *d)
{
    Plan p;
    if (!make_plan(0, d, &p)) return 0;
    // one partial per (128-row tile, output channel); larger tiles need fewer
    const int64_t M = (int64_t)d->N * p.OHf * p.OWf;
    return (size_t)((M + 127) / 128) * p.oc * sizeof(Q8tConvStat);
}

int q8t_nhwc_conv(int which, const q8t_conv_desc *d, const void *a, const q8t_qparams *qa, const void *b,
                  const q8t_qparams *qb, float *out_f, void *out_acc, float *bn_stats, void *stats_ws, void *ws,
                  hipStream_t st)
{
    Plan p;
    if (!make_plan(which, d, &p)) return Q8T_ERR_SHAPE;
    if (!ws || !q8t_aligned(ws, 16)) return Q8T_ERR_WORKSPACE;
    if (bn_stats && (which != 0 || !stats_ws || !q8t_aligned(stats_ws, 16))) return Q8T_ERR_WORKSPACE;
    Q8tConvStat *bnp = bn_stats ? (Q8tConvStat *)stats_ws : (Q8tConvStat *)nullptr;
    int8_t *xn = (int8_t *)ws;
    int *chansum = (int *)((char *)ws + p.o_chansum);
    int8_t *wt = (int8_t *)ws + p.o_wt;
    int *colsum = (int *)((char *)ws + p.o_colsum);
    int *tapoff = (int *)((char *)ws + p.o_tapoff);

    // 1. operand relayout
    {
        const int HW = p.IH * p.IW;
        const dim3 grid((unsigned)((HW + 63) / 64), (unsigned)d->N);
        if (HW <= 256 && q8t_aligned(a, 16))
            hipLaunchKernelGGL(to_nhwc_small, dim3((unsigned)d->N), dim3(kThreads), (size_t)64 * HW, st, (const int8_t *)a,
                               p.red, HW, xn, chansum);
        else if (HW % 4 == 0 && q8t_aligned(a, 4))
            hipLaunchKernelGGL(to_nhwc<4>, grid, dim3(kThreads), 0, st, (const int8_t *)a, p.red, HW, xn, chansum);
        else
            hipLaunchKernelGGL(to_nhwc<1>, grid, dim3(kThreads), 0, st, (const int8_t *)a, p.red, HW, xn, chansum);
        Q8T_LAUNCH_CHECK();
    }

    // 2. taps of every class.  forward: one class with all taps, operand offset (r - pad, s - pad).
    // layer gradient: class (ph, pw) keeps the taps with (ph + pad - r) and (pw + pad - s) divisible
    // by the stride; the operand (output-gradient) offset is that quotient.
    TapList rs_list = {}, off_list = {};
    ClassOffsets co = {};
    const int stv = d->stride;
    int nt = 0;
    for (int z = 0; z < p.ncls; ++z) {
        co.off[z] = nt;
        const int ph = z / stv, pw = z % stv;
        for (int r = 0; r < d->R; ++r)
            for (int s = 0; s < d->S; ++s) {
                int dh, dw;
                if (which == 0) {
                    dh = r - d->pad;
                    dw = s - d->pad;
                } else {
                    const int eh = ph + d->pad - r, ew = pw + d->pad - s;
                    if (eh % stv || ew % stv) continue;
                    dh = eh / stv;
                    dw = ew / stv;
                }
                rs_list.a[nt] = (int8_t)r;
                rs_list.b[nt] = (int8_t)s;
                off_list.a[nt] = (int8_t)dh;
                off_list.b[nt] = (int8_t)dw;
                ++nt;
            }
    }
    for (int z = p.ncls; z <= MAXCLS; ++z) co.off[z] = nt;
    // positions of every class
    ClassGeo cg = {};
    int maxM = 0;
    for (int z = 0; z < p.ncls; ++z) {
        int oh = p.OHf, ow = p.OWf;
        if (which == 1) {
            const int ph = z / stv, pw = z % stv;
            oh = (p.OHf - ph + stv - 1) / stv;
            ow = (p.OWf - pw + stv - 1) / stv;
        }
        const int m = oh > 0 && ow > 0 ? d->N * oh * ow : 0;
        cg.v[z][0] = oh;
        cg.v[z][1] = ow;
        cg.v[z][2] = m;
        cg.v[z][3] = co.off[z];
        cg.v[z][4] = co.off[z + 1] - co.off[z];
        if (m > maxM) maxM = m;
    }
    // stride 2 with taps in class (0, 0) only (a 1x1 filter without padding) and an even result size:
    // that class's workgroups write the zeros of the other three as well
    bool fill = which == 1 && stv == 2 && p.OHf % 2 == 0 && p.OWf % 2 == 0 && cg.v[0][4] > 0;
    for (int z = 1; z < p.ncls; ++z) fill = fill && cg.v[z][4] == 0;
    const int ncls = fill ? 1 : p.ncls;
    if (fill) maxM = cg.v[0][2];
    int *clsinfo = (int *)((char *)ws + p.o_cls);
    hipLaunchKernelGGL(repack_taps, dim3((unsigned)p.oc, (unsigned)p.ncls), dim3(kThreads), 0, st, (const int8_t *)b,
                       d->K, d->C, d->R, d->S, which, rs_list, off_list, co, cg, wt, colsum, tapoff, clsinfo);
    Q8T_LAUNCH_CHECK();

    // 3. one launch over all classes (the kernel picks its class from the tile index)
    Geo g;
    g.N = d->N;
    g.IH = p.IH;
    g.IW = p.IW;
    g.Cp = p.red;
    g.OC = p.oc;
    g.OHf = p.OHf;
    g.OWf = p.OWf;
    g.ish = g.isw = which == 0 ? stv : 1;
    g.osh = g.osw = which == 0 ? 1 : stv;
    g.OH = g.OW = g.M = g.T = g.oph = g.opw = 0;   // per class, read by the kernel from the class table
    g.vec = q8t_aligned(out_f, 16) && q8t_aligned(out_acc, 16);
    g.ncls = ncls;
    g.fill = fill ? 1 : 0;
    // stride 2 with an even result width: the classes (ph, 0) and (ph, 1) share their positions and are
    // computed by one workgroup, which writes their interleaved results as pairs
    if (which == 1 && stv == 2 && !fill && p.OWf % 2 == 0 && cg.v[0][2] > 0) {
        const int pairM = cg.v[0][2];   // class (0, 0) is the larger row parity
#define Q8T_GOP(CFG)                                                                                                 \
    {                                                                                                                \
        static Q8tLdsOptIn optin;                                                                                    \
        if (conv_pair_lds_bytes<CFG>() > 65536 && q8t_allow_lds(optin, (const void *)igemm_nhwc_pair<CFG>, conv_pair_lds_bytes<CFG>()) != Q8T_OK)      \
            return Q8T_ERR_HIP;                                                                                      \
        g.mtiles = (pairM + CFG::BM - 1) / CFG::BM;                                                                  \
        const int64_t tiles = (int64_t)g.mtiles * 2 * (p.oc / CFG::BN);                                              \
        hipLaunchKernelGGL(igemm_nhwc_pair<CFG>, dim3(q8t_gemm::xcd_grid(tiles)), dim3(CFG::THREADS),                \
                           conv_pair_lds_bytes<CFG>(), st, xn, chansum, wt, colsum, qa, qb, g, tapoff, clsinfo, out_f, \
                           (int32_t *)out_acc);                                                                      \
    }
        if (p.oc % 128 == 0) Q8T_GOP(q8t_gemm::Mid)
        else Q8T_GOP(q8t_gemm::Small)
#undef Q8T_GOP
        Q8T_LAUNCH_CHECK();
        return Q8T_OK;
    }
    // tile: 256 x 256 where the output channels allow it and the launch still fills the chip,
    // else 128 x 128, else 128 x 64
#define Q8T_GO(CFG)                                                                                                  \
    {                                                                                                                \
        static Q8tLdsOptIn optin;                                                                                    \
        if (conv_lds_bytes<CFG>() > 65536 && q8t_allow_lds(optin, (const void *)igemm_nhwc<CFG>, conv_lds_bytes<CFG>()) != Q8T_OK)      \
            return Q8T_ERR_HIP;                                                                                      \
        g.mtiles = (maxM + CFG::BM - 1) / CFG::BM;                                                                   \
        const int64_t tiles = (int64_t)g.mtiles * ncls * (p.oc / CFG::BN);                                         \
        if (tiles > 0)                                                                                               \
            hipLaunchKernelGGL(igemm_nhwc<CFG>, dim3(q8t_gemm::xcd_grid(tiles)), dim3(CFG::THREADS),                 \
                               conv_lds_bytes<CFG>(), st, xn, chansum, wt, colsum, qa, qb, g, tapoff, clsinfo, out_f, \
                               (int32_t *)out_acc, bnp);                                                             \
    }
    if (p.oc % 256 == 0 && (int64_t)((maxM + 255) / 256) * ncls * (p.oc / 256) >= 128) Q8T_GO(q8t_gemm::Big)
    else if (p.oc % 128 == 0) Q8T_GO(q8t_gemm::Mid)
    else Q8T_GO(q8t_gemm::Small)
#undef Q8T_GO
    Q8T_LAUNCH_CHECK();
    if (bnp)   // forward: one class, every row tile wrote its partial
        return q8t_conv_stats_finalize(bnp, p.oc, g.mtiles, g.mtiles, (double)maxM, qa, qb, bn_stats, st);
    return Q8T_OK;
}
