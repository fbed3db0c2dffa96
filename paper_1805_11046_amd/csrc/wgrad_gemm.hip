// General MFMA path for the convolution weight gradient g_W = g_l * I^T with the 16-bit copy of
// the gradient (Sections 1 and 4, "gradient bifurcation"): any filter size, stride, padding and
// channel count.  The reduction runs over every output position (n, p, q), which is the
// contiguous index of both NCHW operands, so the product is a GEMM of two matrices that are both
// stored "reduction index fastest":
//
//   A'[2K][Mp]   rows k      : high bytes of the stored 16-bit gradient codes of output channel k
//                rows K + k  : their low bytes, re-centred ( s = 256*hi + lo + 128, hi and lo signed bytes )
//   B'[CRS][Mp]  row (c,r,s) : the input code that meets gradient position m under filter tap (r,s)
//                              (stored zero point where the tap falls into the padding)
//   m = (n*P + p)*Q + q, padded with zero codes up to Mp (a multiple of 64).
//
// Launches: split16 (builds A'), im2col_rows (builds B'), gemm_nt (int8 MFMA, 128x128 or 128x64
// tiles, the reduction split over blockIdx.z into slices of at most 65536 products so that the
// 32-bit accumulators cannot overflow), wgrad_finish (sums the slices in 64 bits, recombines the
// two byte planes, applies the zero-point correction, dequantizes).  Exact for any reduction
// length: every partial sum is an integer below 2^31 and the recombination is done in int64.
#include "q8t_common.h"
#include "q8t_internal.h"
#include "gemm_core.h"

namespace {

using q8t_gemm::v4i;

constexpr int kThreads = 256;
constexpr int BM = 128;
constexpr int kMaxSlice = 65536;

__device__ __forceinline__ int bytesum4(uint32_t v) { return __builtin_amdgcn_sdot4((int)v, 0x01010101, 0, false); }
__device__ __forceinline__ int bytesum16(const uint4 &v)
{
    return bytesum4(v.x) + bytesum4(v.y) + bytesum4(v.z) + bytesum4(v.w);
}

// quotient x / d for 0 <= x < 2^24 through the float reciprocal, corrected by at most one
__device__ __forceinline__ int fdiv(int x, int d, float rd)
{
    int q = (int)((float)x * rd);
    const int r = x - q * d;
    if (r < 0) --q;
    else if (r >= d) ++q;
    return q;
}

// ---- A': byte planes of the 16-bit gradient, [2K][Mp] -----------------------------------------
// G = codes per global load: 16 (planes of a multiple of 16 positions, 32-byte aligned rows),
// 4 (multiple of 4, 8-byte aligned) or 1.  A group of G positions never straddles two images.
template <int G>
__global__ __launch_bounds__(kThreads) void split16(const int16_t *__restrict__ g16, int K, int PQ, int64_t Mtot,
                                                    int64_t Mp, const q8t_qparams *__restrict__ qpg,
                                                    int8_t *__restrict__ A)
{
    const int64_t chunks = Mp >> 4;
    const int64_t id = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (id >= chunks * K) return;
    const int k = (int)(id / chunks);
    const int64_t m0 = (id - (int64_t)k * chunks) << 4;
    const int zsg = qpg->zero_point - (1 << (qpg->bits - 1));
    const uint32_t zz = (uint32_t)(zsg & 0xFFFF) * 0x00010001u;
    int n = (int)(m0 / PQ), pq = (int)(m0 - (int64_t)n * PQ);
    uint32_t d[8];   // 16 codes, two per dword
#pragma unroll
    for (int i = 0; i < 8; ++i) d[i] = zz;
    if (G == 16) {
        if (m0 < Mtot) {
            const uint4 *src = reinterpret_cast<const uint4 *>(g16 + ((size_t)n * K + k) * PQ + pq);
            const uint4 u = src[0], v = src[1];
            d[0] = u.x; d[1] = u.y; d[2] = u.z; d[3] = u.w;
            d[4] = v.x; d[5] = v.y; d[6] = v.z; d[7] = v.w;
        }
    } else if (G == 4) {
#pragma unroll
        for (int grp = 0; grp < 4; ++grp) {
            if (m0 + grp * 4 < Mtot) {
                const uint2 u = *reinterpret_cast<const uint2 *>(g16 + ((size_t)n * K + k) * PQ + pq);
                d[grp * 2] = u.x;
                d[grp * 2 + 1] = u.y;
            }
            pq += 4;
            if (pq == PQ) {
                pq = 0;
                ++n;
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if (m0 + i < Mtot) {
                const uint32_t s = (uint16_t)g16[((size_t)n * K + k) * PQ + pq];
                d[i >> 1] = (i & 1) ? (d[i >> 1] & 0x0000FFFFu) | (s << 16) : (d[i >> 1] & 0xFFFF0000u) | s;
            }
            if (++pq == PQ) {
                pq = 0;
                ++n;
            }
        }
    }
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        hi[i] = __builtin_amdgcn_perm(d[2 * i + 1], d[2 * i], 0x07050301u);
        lo[i] = __builtin_amdgcn_perm(d[2 * i + 1], d[2 * i], 0x06040200u) ^ 0x80808080u;
    }
    *reinterpret_cast<uint4 *>(A + (size_t)k * Mp + m0) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
    *reinterpret_cast<uint4 *>(A + (size_t)(K + k) * Mp + m0) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
}

// ---- B': one row per (c, r, s), [CRS][Mp] ------------------------------------------------------
struct ConvG {
    int N, C, H, W, K, R, S, stride, pad, P, Q;
};

__global__ __launch_bounds__(kThreads) void im2col_rows(const int8_t *__restrict__ x, ConvG g, int64_t Mtot, int64_t Mp,
                                                        const q8t_qparams *__restrict__ qpx, int8_t *__restrict__ B)
{
    const int64_t chunks = Mp >> 4;
    const int64_t id = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int CRS = g.C * g.R * g.S;
    if (id >= chunks * CRS) return;
    const int col = (int)(id / chunks);
    const int64_t m0 = (id - (int64_t)col * chunks) << 4;
    const int RS = g.R * g.S;
    const int c = col / RS, t = col - c * RS, r = t / g.S, s = t - r * g.S;
    const int zsx = qpx->zero_point - (1 << (qpx->bits - 1));
    const int PQ = g.P * g.Q;
    int n = (int)(m0 / PQ);
    const int rem = (int)(m0 - (int64_t)n * PQ);
    int p = rem / g.Q, q = rem - p * g.Q;
    uint32_t o[4] = {0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        int v = zsx;
        if (m0 + i < Mtot) {
            const int h = p * g.stride + r - g.pad, w = q * g.stride + s - g.pad;
            if ((unsigned)h < (unsigned)g.H && (unsigned)w < (unsigned)g.W)
                v = x[(((size_t)n * g.C + c) * g.H + h) * g.W + w];
        }
        o[i >> 2] |= (uint32_t)(v & 255) << (8 * (i & 3));
        if (++q == g.Q) {
            q = 0;
            if (++p == g.P) {
                p = 0;
                ++n;
            }
        }
    }
    *reinterpret_cast<uint4 *>(B + (size_t)col * Mp + m0) = make_uint4(o[0], o[1], o[2], o[3]);
}

// Same result through LDS: a workgroup stages the zero-padded planes of CG channels for a group of
// NI images (NI*P*Q a multiple of 4, so that its stretch of every row starts on a dword), then
// every thread builds, for one channel, one dword (4 consecutive positions) for each of the R*S
// taps.  The input is read once instead of R*S times and every store is a full dword.
// A staged plane has (H + 2*pad) rows of `pitch` bytes; the image starts at column L = pad rounded
// up to a multiple of 4 and the pitch is a multiple of 4, so that an aligned dword of the input
// (W % 4 == 0) is an aligned dword of the plane.
struct PlaneG {
    int L, pitch, PB;   // left margin, row pitch, bytes per plane (a multiple of 4)
    int vec;            // bytes per aligned input load: 4, 2 or 1
};

__global__ __launch_bounds__(kThreads) void im2col_planes(const int8_t *__restrict__ x, ConvG g, PlaneG pg, int NI, int CG,
                                                          int64_t Mtot, int64_t Mp, const q8t_qparams *__restrict__ qpx,
                                                          int8_t *__restrict__ B)
{
    extern __shared__ __align__(16) int8_t planes[];
    const int c0 = blockIdx.y * CG, n0 = blockIdx.x * NI;
    const int ni = min(NI, g.N - n0), cg = min(CG, g.C - c0);
    const int PB = pg.PB, pitch = pg.pitch;
    const int PQ = g.P * g.Q, HW = g.H * g.W;
    const int zsx = qpx->zero_point - (1 << (qpx->bits - 1));
    const uint32_t zb = (uint32_t)(zsx & 255);
    {
        uint32_t *pw = reinterpret_cast<uint32_t *>(planes);
        for (int i = threadIdx.x; i < (cg * NI * PB) >> 2; i += kThreads) pw[i] = zb * 0x01010101u;
    }
    __syncthreads();
    // plane (cl, nl) sits at (cl*NI + nl)*PB
    if (pg.vec == 4) {
        const int HW4 = HW >> 2, W4 = g.W >> 2;
        const float rHW4 = 1.0f / (float)HW4, rW4 = 1.0f / (float)W4;
        for (int i = threadIdx.x; i < cg * ni * HW4; i += kThreads) {
            const int pl = fdiv(i, HW4, rHW4), t = i - pl * HW4, h = fdiv(t, W4, rW4), w4 = t - h * W4;
            const int cl = pl / ni, nl = pl - cl * ni;
            const uint32_t v = *reinterpret_cast<const uint32_t *>(x + ((size_t)(n0 + nl) * g.C + c0 + cl) * HW + (size_t)t * 4);
            *reinterpret_cast<uint32_t *>(planes + (cl * NI + nl) * PB + (h + g.pad) * pitch + pg.L + w4 * 4) = v;
        }
    } else if (pg.vec == 2) {
        const int HW2 = HW >> 1, W2 = g.W >> 1;
        const float rHW2 = 1.0f / (float)HW2, rW2 = 1.0f / (float)W2;
        for (int i = threadIdx.x; i < cg * ni * HW2; i += kThreads) {
            const int pl = fdiv(i, HW2, rHW2), t = i - pl * HW2, h = fdiv(t, W2, rW2), w2 = t - h * W2;
            const int cl = pl / ni, nl = pl - cl * ni;
            const uint16_t v = *reinterpret_cast<const uint16_t *>(x + ((size_t)(n0 + nl) * g.C + c0 + cl) * HW + (size_t)t * 2);
            *reinterpret_cast<uint16_t *>(planes + (cl * NI + nl) * PB + (h + g.pad) * pitch + pg.L + w2 * 2) = v;
        }
    } else {
        const float rHW = 1.0f / (float)HW, rW = 1.0f / (float)g.W;
        for (int i = threadIdx.x; i < cg * ni * HW; i += kThreads) {
            const int pl = fdiv(i, HW, rHW), t = i - pl * HW, h = fdiv(t, g.W, rW), w = t - h * g.W;
            const int cl = pl / ni, nl = pl - cl * ni;
            planes[(cl * NI + nl) * PB + (h + g.pad) * pitch + pg.L + w] = x[((size_t)(n0 + nl) * g.C + c0 + cl) * HW + t];
        }
    }
    __syncthreads();
    const float rPQ = 1.0f / (float)PQ, rQ = 1.0f / (float)g.Q;
    const int64_t mbase = (int64_t)n0 * PQ;
    const bool last = n0 + NI >= g.N;
    const int64_t mend = last ? Mp : mbase + (int64_t)NI * PQ;   // the last group also writes the padding
    const int ndw = (int)((mend - mbase) >> 2);
    const float rndw = 1.0f / (float)ndw;
    const int RS = g.R * g.S;
    const int col0 = pg.L - g.pad;   // plane column of input column -pad
    for (int it = threadIdx.x; it < cg * ndw; it += kThreads) {
        const int cl = fdiv(it, ndw, rndw), dp = it - cl * ndw;
        int off[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int e = dp * 4 + j;
            off[j] = -1;
            if (mbase + e < Mtot) {
                const int nl = fdiv(e, PQ, rPQ), t = e - nl * PQ, pp = fdiv(t, g.Q, rQ), qq = t - pp * g.Q;
                off[j] = (cl * NI + nl) * PB + pp * g.stride * pitch + qq * g.stride + col0;
            }
        }
        int8_t *dst = B + ((size_t)(c0 + cl) * RS) * Mp + mbase + (int64_t)dp * 4;
        for (int r = 0; r < g.R; ++r)
            for (int s = 0; s < g.S; ++s) {
                const int o = r * pitch + s;
                uint32_t v = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t b = off[j] >= 0 ? (uint32_t)(uint8_t)planes[off[j] + o] : zb;
                    v |= b << (8 * j);
                }
                *reinterpret_cast<uint32_t *>(dst) = v;
                dst += Mp;
            }
    }
}

// ---- C[z][i][j] = sum over slice z of A'[i][m] * B'[j][m] ---------------------------------------
// Also leaves the sums of the staged bytes per row (of A') and per column (row of B') and slice.
// Staging role of a thread (see gemm_core.h): chunk q = tid & 3 of tile rows ar = tid >> 2 and ar + RP.
template <class C>
struct NtOps {
    const int8_t *pa, *pb, *pa0, *pb0;   // next chunk; first chunk (always readable)
    size_t skip;                         // RP rows further
    bool need_a, need_b;                 // this workgroup reports the row / column sums of its tiles
    int sa0, sa1, sb0, sb1;
    __device__ __forceinline__ void load(q8t_gemm::Regs &r, bool valid)
    {
        const int8_t *qa = valid ? pa : pa0, *qb = valid ? pb : pb0;
        r.a0 = *reinterpret_cast<const uint4 *>(qa);
        r.a1 = *reinterpret_cast<const uint4 *>(qa + skip);
        r.b0 = *reinterpret_cast<const uint4 *>(qb);
        r.b1 = C::NB == 2 ? *reinterpret_cast<const uint4 *>(qb + skip) : r.b0;
        pa += 64;
        pb += 64;
    }
    __device__ __forceinline__ void prepare(q8t_gemm::Regs &r, bool valid)
    {
        // a surplus step stages zero B' rows, so whatever A' holds adds nothing to the products
        r.b0 = q8t_gemm::sel16(valid, r.b0);
        r.b1 = q8t_gemm::sel16(valid, r.b1);
        if (need_a) {   // uniform over the workgroup
            sa0 += valid ? bytesum16(r.a0) : 0;
            sa1 += valid ? bytesum16(r.a1) : 0;
        }
        if (need_b) {
            sb0 += bytesum16(r.b0);
            if (C::NB == 2) sb1 += bytesum16(r.b1);
        }
    }
};

__device__ __forceinline__ int quad_sum(int v)
{
    v += __shfl_xor(v, 1, Q8T_WAVE);
    v += __shfl_xor(v, 2, Q8T_WAVE);
    return v;
}

template <class C>
__device__ __forceinline__ void write_partials(int32_t *__restrict__ dst, int Rbp, int r0, int c0,
                                               const v4i (&acc)[C::MT][C::NT])
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, kb = lane >> 4;
    const int rowbase = C::rowbase(wave), colbase = C::colbase(wave);
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < C::NT; ++nt)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                dst[(size_t)(r0 + rowbase + mt * 16 + kb * 4 + j) * Rbp + c0 + colbase + nt * 16 + l16] = acc[mt][nt][j];
}

template <class C>
__global__ __launch_bounds__(C::THREADS, C::MINB) void gemm_nt(const int8_t *__restrict__ A, const int8_t *__restrict__ B,
                                                                int64_t Mp, int slice, int Rap, int Rbp, int nz,
                                                                int32_t *__restrict__ part, int *__restrict__ rsum,
                                                                int *__restrict__ csum)
{
    __shared__ __align__(16) int8_t sA[2 * C::BM * 64];
    __shared__ __align__(16) int8_t sB[2 * C::BN * 64];

    // logical tile order: row tiles fastest (they share the B' tile), then column tiles (same A' slice)
    const int nx = Rap / C::BM, ny = Rbp / C::BN;
    const int lg = q8t_gemm::xcd_logical(blockIdx.x, nx * ny * nz);
    if (lg >= nx * ny * nz) return;
    const int bx = lg % nx, by = (lg / nx) % ny, z = lg / (nx * ny);
    const int tid = threadIdx.x, ar = tid >> 2, q = tid & 3;
    const int r0 = bx * C::BM, c0 = by * C::BN;
    const int64_t mb = (int64_t)z * slice;
    const int64_t me = mb + slice < Mp ? mb + slice : Mp;
    const int steps = (int)((me - mb) >> 6);

    NtOps<C> ops;
    ops.pa = ops.pa0 = A + (size_t)(r0 + ar) * Mp + mb + q * 16;
    ops.pb = ops.pb0 = B + (size_t)(c0 + ar) * Mp + mb + q * 16;
    ops.skip = (size_t)C::RP * Mp;
    ops.need_a = by == 0;
    ops.need_b = bx == 0;
    ops.sa0 = ops.sa1 = ops.sb0 = ops.sb1 = 0;

    v4i acc[C::MT][C::NT];
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < C::NT; ++nt) acc[mt][nt] = (v4i){0, 0, 0, 0};
    q8t_gemm::pipeline<C>(ops, steps, sA, sB, acc);

    // byte sums of this slice: the four threads of a row hold its pieces
    const int sa0 = quad_sum(ops.sa0), sa1 = quad_sum(ops.sa1), sb0 = quad_sum(ops.sb0), sb1 = quad_sum(ops.sb1);
    if (by == 0 && q == 0) {
        rsum[(size_t)z * Rap + r0 + ar] = sa0;
        rsum[(size_t)z * Rap + r0 + ar + C::RP] = sa1;
    }
    if (bx == 0 && q == 0) {
        csum[(size_t)z * Rbp + c0 + ar] = sb0;
        if (C::NB == 2) csum[(size_t)z * Rbp + c0 + ar + C::RP] = sb1;
    }
    write_partials<C>(part + (size_t)z * Rap * Rbp, Rbp, r0, c0, acc);
}

// ---- 1x1, stride 1, no padding, planes of a multiple of 64 positions ---------------------------
// Both operands are read in place: a step is 64 consecutive positions of one image, where row k
// of the gradient and row c of the input are contiguous in NCHW.  The 16-bit codes are split into
// their byte planes in registers.  A row tile holds RP output channels: its first RP rows are the
// high bytes, the next RP rows the low bytes, and the slice results keep that tiled row order.
template <class C>
struct DirectOps {
    const int16_t *g16;
    const int8_t *x;
    int K, Cin, PQ, cpi, krow, crow, q;
    int n, ch, n_first, ch_first;
    bool need_a, need_b;
    int shi, slo, sb0, sb1;
    __device__ __forceinline__ void load(q8t_gemm::Regs &r, bool valid)
    {
        const int nn = valid ? n : n_first, cc = valid ? ch : ch_first;
        const int16_t *pa = g16 + ((size_t)nn * K + krow) * PQ + cc * 64 + q * 16;
        const int8_t *pb = x + ((size_t)nn * Cin + crow) * PQ + cc * 64 + q * 16;
        r.a0 = *reinterpret_cast<const uint4 *>(pa);
        r.a1 = *reinterpret_cast<const uint4 *>(pa + 8);
        r.b0 = *reinterpret_cast<const uint4 *>(pb);
        r.b1 = C::NB == 2 ? *reinterpret_cast<const uint4 *>(pb + (size_t)C::RP * PQ) : r.b0;
        const bool wrap = ch + 1 == cpi;
        ch = wrap ? 0 : ch + 1;
        n += wrap ? 1 : 0;
    }
    __device__ __forceinline__ void prepare(q8t_gemm::Regs &r, bool valid)
    {
        uint4 hi, lo;
        hi.x = __builtin_amdgcn_perm(r.a0.y, r.a0.x, 0x07050301u);
        hi.y = __builtin_amdgcn_perm(r.a0.w, r.a0.z, 0x07050301u);
        hi.z = __builtin_amdgcn_perm(r.a1.y, r.a1.x, 0x07050301u);
        hi.w = __builtin_amdgcn_perm(r.a1.w, r.a1.z, 0x07050301u);
        lo.x = __builtin_amdgcn_perm(r.a0.y, r.a0.x, 0x06040200u) ^ 0x80808080u;
        lo.y = __builtin_amdgcn_perm(r.a0.w, r.a0.z, 0x06040200u) ^ 0x80808080u;
        lo.z = __builtin_amdgcn_perm(r.a1.y, r.a1.x, 0x06040200u) ^ 0x80808080u;
        lo.w = __builtin_amdgcn_perm(r.a1.w, r.a1.z, 0x06040200u) ^ 0x80808080u;
        r.a0 = hi;
        r.a1 = lo;
        r.b0 = q8t_gemm::sel16(valid, r.b0);   // a surplus step stages zero input rows
        r.b1 = q8t_gemm::sel16(valid, r.b1);
        if (need_a) {   // uniform over the workgroup
            shi += valid ? bytesum16(hi) : 0;
            slo += valid ? bytesum16(lo) : 0;
        }
        if (need_b) {
            sb0 += bytesum16(r.b0);
            if (C::NB == 2) sb1 += bytesum16(r.b1);
        }
    }
};

template <class C>
__global__ __launch_bounds__(C::THREADS, C::MINB) void gemm_direct(const int16_t *__restrict__ g16, const int8_t *__restrict__ x,
                                                                    int K, int Cin, int PQ, int steps_total, int steps_slice,
                                                                    int Rap, int Rbp, int nz, int32_t *__restrict__ part,
                                                                    int *__restrict__ rsum, int *__restrict__ csum)
{
    __shared__ __align__(16) int8_t sA[2 * C::BM * 64];
    __shared__ __align__(16) int8_t sB[2 * C::BN * 64];

    const int nx = K / C::RP, ny = Rbp / C::BN;
    const int lg = q8t_gemm::xcd_logical(blockIdx.x, nx * ny * nz);
    if (lg >= nx * ny * nz) return;
    const int bx = lg % nx, by = (lg / nx) % ny, z = lg / (nx * ny);
    const int tid = threadIdx.x, ar = tid >> 2, q = tid & 3;
    const int r0 = bx * C::BM, c0 = by * C::BN;
    const int t0 = z * steps_slice;
    const int steps = min(steps_slice, steps_total - t0);

    DirectOps<C> ops;
    ops.g16 = g16;
    ops.x = x;
    ops.K = K;
    ops.Cin = Cin;
    ops.PQ = PQ;
    ops.cpi = PQ >> 6;   // steps per image
    ops.q = q;
    ops.krow = bx * C::RP + ar;
    ops.crow = c0 + ar;
    ops.n = ops.n_first = t0 / ops.cpi;
    ops.ch = ops.ch_first = t0 - ops.n * ops.cpi;
    ops.need_a = by == 0;
    ops.need_b = bx == 0;
    ops.shi = ops.slo = ops.sb0 = ops.sb1 = 0;

    v4i acc[C::MT][C::NT];
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < C::NT; ++nt) acc[mt][nt] = (v4i){0, 0, 0, 0};
    q8t_gemm::pipeline<C>(ops, steps, sA, sB, acc);

    const int shi = quad_sum(ops.shi), slo = quad_sum(ops.slo), sb0 = quad_sum(ops.sb0), sb1 = quad_sum(ops.sb1);
    if (by == 0 && q == 0) {
        rsum[(size_t)z * Rap + r0 + ar] = shi;
        rsum[(size_t)z * Rap + r0 + C::RP + ar] = slo;
    }
    if (bx == 0 && q == 0) {
        csum[(size_t)z * Rbp + c0 + ar] = sb0;
        if (C::NB == 2) csum[(size_t)z * Rbp + c0 + ar + C::RP] = sb1;
    }
    write_partials<C>(part + (size_t)z * Rap * Rbp, Rbp, r0, c0, acc);
}

// ---- slices -> exact 64-bit sums -> outputs ------------------------------------------------------
// acc(k,col) = sum (g - zg)(x - zx),  g = 256*hi + lo + 128 :
//   256*S_hi + S_lo + (128 - zg)*colsum - zx*(256*rowsum_hi + rowsum_lo + (128 - zg)*Mp)
// A workgroup owns 256/zgn consecutive outputs; its zgn groups of lanes share the slices.
__global__ __launch_bounds__(kThreads) void wgrad_finish(const int32_t *__restrict__ part, const int *__restrict__ rsum,
                                                         const int *__restrict__ csum, int nz, int K, int CRS, int Rap,
                                                         int Rbp, int64_t Mp, const q8t_qparams *__restrict__ qpg,
                                                         const q8t_qparams *__restrict__ qpx, float *__restrict__ dw,
                                                         int64_t *__restrict__ acc_out, int zgn, int tiled, int S, int GP)
{
    __shared__ long long red[5][kThreads];
    const int per = kThreads / zgn;
    const int o = threadIdx.x % per, zg = threadIdx.x / per;
    const int64_t id = (int64_t)blockIdx.x * per + o;
    const bool ok = id < (int64_t)K * CRS;
    long long shi = 0, slo = 0, rhi = 0, rlo = 0, cs = 0;
    int k = 0, col = 0;
    if (ok) {
        k = (int)(id / CRS);
        col = (int)(id - (int64_t)k * CRS);
        // GP > 0: the partial sums keep the taps of one (channel, filter row) in groups of GP columns
        if (GP) col = (col / S) * GP + col % S;
        // rows of the two byte planes: [all high | all low], or per `tiled` channels [high | low]
        const int rh = tiled ? (k / tiled) * 2 * tiled + (k % tiled) : k, rl = tiled ? rh + tiled : K + k;
        for (int z = zg; z < nz; z += zgn) {
            shi += part[((size_t)z * Rap + rh) * Rbp + col];
            slo += part[((size_t)z * Rap + rl) * Rbp + col];
            rhi += rsum[(size_t)z * Rap + rh];
            rlo += rsum[(size_t)z * Rap + rl];
            cs += csum[(size_t)z * Rbp + col];
        }
    }
    if (zgn > 1) {
        red[0][threadIdx.x] = shi;
        red[1][threadIdx.x] = slo;
        red[2][threadIdx.x] = rhi;
        red[3][threadIdx.x] = rlo;
        red[4][threadIdx.x] = cs;
        __syncthreads();
        if (zg != 0 || !ok) return;
        shi = slo = rhi = rlo = cs = 0;
        for (int g = 0; g < zgn; ++g) {
            shi += red[0][g * per + o];
            slo += red[1][g * per + o];
            rhi += red[2][g * per + o];
            rlo += red[3][g * per + o];
            cs += red[4][g * per + o];
        }
    }
    if (!ok) return;
    const int zsg = qpg->zero_point - (1 << (qpg->bits - 1)), zsx = qpx->zero_point - (1 << (qpx->bits - 1));
    const int64_t ca = 128 - zsg;
    const int64_t v = 256 * shi + slo + ca * cs - (int64_t)zsx * (256 * rhi + rlo + ca * Mp);
    if (acc_out) acc_out[id] = v;
    if (dw) dw[id] = (float)((double)v * (double)(qpg->scale * qpx->scale));
}

struct Plan {
    int P, Q, CRS, Rap, Rbp, nz, slice, direct;
    int cfg;   // 2: 256x256 tiles, 1: 128x128, 0: 128x64
    int64_t Mtot, Mp;
    size_t o_B, o_part, o_rsum, o_csum, total;
};

inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

// ---- weight gradient of a layer with few input channels (the network's first layer), one kernel ----
// GEMM view as above (rows = byte planes of g16 for 64 output channels, columns = (channel, filter
// row) groups of GP taps, reduction = positions), but neither operand is laid out in HBM: a
// workgroup walks output rows (n, p); for each it splits the 64 x Q gradient values into the two
// byte planes straight into the LDS operand tile, stages the R input rows of every channel and
// cuts the column operand out of them (16 consecutive positions of one tap = 16 bytes `stride`
// apart in a staged row), multiplies, and keeps the 128 x Kf accumulator tile in registers until its
// share of the rows is done.  Positions Q..127 of a row hold (0, zero code): they add nothing and
// are counted in the reduction length handed to wgrad_finish.  The loads for the next output row
// are issued before the current one is multiplied.
// Needs: C*R*GP <= 256, stride 1 or 2, Q <= 128 and Q % 16 == 0, W % 4 == 0, 16-byte aligned g16
// rows (Q % 8 == 0), at most UX dwords of input and UA / UB operand pieces per thread and row.
template <int GP, int NT>
__global__ __launch_bounds__(kThreads) void wgrad_smallc(const int16_t *__restrict__ g16, const int8_t *__restrict__ x, int C,
                                                         int H, int W, int R, int S, int stride, int pad, int P, int Q, int K,
                                                         int RB, int rows_total, const q8t_qparams *__restrict__ qpx,
                                                         int32_t *__restrict__ part, int *__restrict__ rsum,
                                                         int *__restrict__ csum)
{
    constexpr int Kf = NT * 16, UX = 6, UA = 4, UB = 5;
    extern __shared__ __align__(16) int8_t lds[];
    int8_t *sA = lds;                                    // [2][128][64]
    int8_t *sB = sA + 2 * 128 * 64;                      // [2][Kf][64]
    int *sums = reinterpret_cast<int *>(sB + 2 * Kf * 64);   // [128] rows of A', [Kf] rows of B'
    int8_t *rows = reinterpret_cast<int8_t *>(sums + 128 + Kf);   // [C*R][Wp] + 16
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, kq = lane >> 4;
    const int z = blockIdx.x, kblk = blockIdx.y;
    const int row0 = z * RB, row1 = min(rows_total, row0 + RB);
    const int zx = qpx->zero_point - (1 << (qpx->bits - 1));
    const uint32_t zfill = (uint32_t)(zx & 255) * 0x01010101u;
    const int CR = C * R, L = (pad + 3) & ~3, Wp = (L + W + pad + 3) & ~3;
    const int W4 = W >> 2, Q8 = Q >> 3, Q16 = Q >> 4;

    // ---- fixed roles of the thread ----
    int xd[UX], xr[UX], xo[UX];          // input dwords: LDS offset (-1: none), filter row - pad, offset inside an image
    int ag[UA], ad[UA];                  // gradient pieces of 8 values: offset inside an image, LDS offset (-1: none)
    int bs[UB], bd[UB], bj[UB];          // column pieces of 16 positions: byte offset in `rows`, LDS offset (-1), column
#pragma unroll
    for (int u = 0; u < UX; ++u) {
        const int i = u * kThreads + tid;
        xd[u] = -1;
        xr[u] = xo[u] = 0;
        if (i < CR * W4) {
            const int cr = i / W4, w4 = i - cr * W4, c = cr / R, r = cr - c * R;
            xd[u] = cr * Wp + L + w4 * 4;
            xr[u] = r - pad;
            xo[u] = c * H * W + w4 * 4;
        }
    }
#pragma unroll
    for (int u = 0; u < UA; ++u) {
        const int i = u * kThreads + tid;
        ad[u] = -1;
        ag[u] = 0;
        if (i < 64 * Q8) {
            const int k = i / Q8, ch = i - k * Q8, m = ch * 8;
            ag[u] = (kblk * 64 + k) * P * Q + m;
            ad[u] = (m >> 6) * (128 * 64) + k * 64 + ((((m & 63) >> 4) ^ q8t_gemm::swz(k)) * 16) + ((m >> 3) & 1) * 8;
        }
    }
#pragma unroll
    for (int u = 0; u < UB; ++u) {
        const int i = u * kThreads + tid;
        bd[u] = -1;
        bs[u] = bj[u] = 0;
        if (i < CR * S * Q16) {
            const int t = i / Q16, c = i - t * Q16, gg = t / S, s2 = t - gg * S, j = gg * GP + s2;
            bj[u] = j;
            bs[u] = gg * Wp + L - pad + s2 + stride * 16 * c;
            bd[u] = (c >> 2) * (Kf * 64) + j * 64 + (((c & 3) ^ q8t_gemm::swz(j)) * 16);
        }
    }
    // ---- LDS: A' zero, B' and the staged rows at the zero code ----
    {
        uint32_t *w = reinterpret_cast<uint32_t *>(sA);
        for (int i = tid; i < (2 * 128 * 64) >> 2; i += kThreads) w[i] = 0;
        w = reinterpret_cast<uint32_t *>(sB);
        for (int i = tid; i < (2 * Kf * 64) >> 2; i += kThreads) w[i] = zfill;
        w = reinterpret_cast<uint32_t *>(rows);
        for (int i = tid; i < (CR * Wp + 16) >> 2; i += kThreads) w[i] = zfill;
        for (int i = tid; i < 128 + Kf; i += kThreads) sums[i] = 0;
    }
    v4i acc[2][NT];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) acc[i][j] = (v4i){0, 0, 0, 0};
    int sah[UA], sal[UA], sbs[UB];
#pragma unroll
    for (int u = 0; u < UA; ++u) sah[u] = sal[u] = 0;
#pragma unroll
    for (int u = 0; u < UB; ++u) sbs[u] = 0;

    uint32_t xv[UX];
    uint4 av[UA];
    auto issue = [&](int row) {
        const int n = row / P, p = row - n * P;
        const int8_t *xb = x + (size_t)n * C * H * W;
        const int16_t *gb = g16 + (size_t)n * K * P * Q + (size_t)p * Q;
#pragma unroll
        for (int u = 0; u < UX; ++u) {
            const int h = p * stride + xr[u];
            xv[u] = zfill;
            if (xd[u] >= 0 && (unsigned)h < (unsigned)H) xv[u] = *reinterpret_cast<const uint32_t *>(xb + xo[u] + (size_t)h * W);
        }
#pragma unroll
        for (int u = 0; u < UA; ++u) {
            av[u] = make_uint4(0, 0, 0, 0);
            if (ad[u] >= 0) av[u] = *reinterpret_cast<const uint4 *>(gb + ag[u]);
        }
    };
    if (row0 < row1) issue(row0);
    for (int row = row0; row < row1; ++row) {
        __syncthreads();   // the fill, or the previous row's multiply, is done with sA / sB / rows
#pragma unroll
        for (int u = 0; u < UX; ++u)
            if (xd[u] >= 0) *reinterpret_cast<uint32_t *>(rows + xd[u]) = xv[u];
#pragma unroll
        for (int u = 0; u < UA; ++u) {
            if (ad[u] < 0) continue;
            const uint32_t h0 = __builtin_amdgcn_perm(av[u].y, av[u].x, 0x07050301u);
            const uint32_t h1 = __builtin_amdgcn_perm(av[u].w, av[u].z, 0x07050301u);
            const uint32_t l0 = __builtin_amdgcn_perm(av[u].y, av[u].x, 0x06040200u) ^ 0x80808080u;
            const uint32_t l1 = __builtin_amdgcn_perm(av[u].w, av[u].z, 0x06040200u) ^ 0x80808080u;
            *reinterpret_cast<uint2 *>(sA + ad[u]) = make_uint2(h0, h1);
            *reinterpret_cast<uint2 *>(sA + ad[u] + 64 * 64) = make_uint2(l0, l1);
            sah[u] += bytesum4(h0) + bytesum4(h1);
            sal[u] += bytesum4(l0) + bytesum4(l1);
        }
        if (row + 1 < row1) issue(row + 1);
        __syncthreads();   // staged rows complete
        // column operand: 16 positions of one tap are 16 bytes `stride` apart; read the aligned dwords
        // that contain them, shift to the first byte, keep every stride-th byte
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            if (bd[u] < 0) continue;
            const int a0 = bs[u] & ~3;
            const uint32_t sh = (uint32_t)(bs[u] & 3);
            uint32_t o[4];
            if (stride == 1) {
                uint32_t d[5];
#pragma unroll
                for (int i = 0; i < 5; ++i) d[i] = *reinterpret_cast<const uint32_t *>(rows + a0 + 4 * i);
#pragma unroll
                for (int i = 0; i < 4; ++i) o[i] = __builtin_amdgcn_alignbyte(d[i + 1], d[i], sh);
            } else {
                uint32_t d[9];
#pragma unroll
                for (int i = 0; i < 9; ++i) d[i] = *reinterpret_cast<const uint32_t *>(rows + a0 + 4 * i);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t e0 = __builtin_amdgcn_alignbyte(d[2 * i + 1], d[2 * i], sh);
                    const uint32_t e1 = __builtin_amdgcn_alignbyte(d[2 * i + 2], d[2 * i + 1], sh);
                    o[i] = __builtin_amdgcn_perm(e1, e0, 0x06040200u);   // bytes 0, 2, 4, 6 of the 8
                }
            }
            *reinterpret_cast<uint4 *>(sB + bd[u]) = make_uint4(o[0], o[1], o[2], o[3]);
            sbs[u] += bytesum4(o[0]) + bytesum4(o[1]) + bytesum4(o[2]) + bytesum4(o[3]);
        }
        __syncthreads();
        // wavefront w multiplies rows [32w, 32w + 32) of A' (w < 2: high plane) against every column tile
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v4i af[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int r = wave * 32 + i * 16 + l16;
                af[i] = *reinterpret_cast<const v4i *>(sA + ks * (128 * 64) + r * 64 + ((kq ^ q8t_gemm::swz(r)) * 16));
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int r = nt * 16 + l16;
                const v4i bf = *reinterpret_cast<const v4i *>(sB + ks * (Kf * 64) + r * 64 + ((kq ^ q8t_gemm::swz(r)) * 16));
                acc[0][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[0], bf, acc[0][nt], 0, 0, 0);
                acc[1][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af[1], bf, acc[1][nt], 0, 0, 0);
            }
        }
    }
    // ---- byte sums of the rows of A' and B' (zero-point correction), then the partial tile ----
    __syncthreads();
#pragma unroll
    for (int u = 0; u < UA; ++u) {
        if (ad[u] < 0) continue;
        const int k = (u * kThreads + tid) / Q8;
        atomicAdd(&sums[k], sah[u]);
        atomicAdd(&sums[64 + k], sal[u]);
    }
#pragma unroll
    for (int u = 0; u < UB; ++u)
        if (bd[u] >= 0) atomicAdd(&sums[128 + bj[u]], sbs[u]);
    __syncthreads();
    const int Rap = 2 * K;
    if (tid < 128) rsum[(size_t)z * Rap + (tid < 64 ? kblk * 64 + tid : K + kblk * 64 + tid - 64)] = sums[tid];
    // positions Q..127 of every row hold the zero code
    if (kblk == 0 && tid < Kf) csum[(size_t)z * Kf + tid] = sums[128 + tid] + (row1 > row0 ? (row1 - row0) * (128 - Q) * zx : 0);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int lr = wave * 32 + i * 16 + kq * 4 + jj;
            const int gr = lr < 64 ? kblk * 64 + lr : K + kblk * 64 + lr - 64;
            int32_t *dst = part + ((size_t)z * Rap + gr) * Kf + l16;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) dst[nt * 16] = acc[i][nt][jj];
        }
}

struct FusedPlan {
    int P, Q, GP, Kf, nz, RB, rows;
    size_t lds, o_rsum, o_csum, total;
};

bool make_fused_plan(const q8t_conv_desc *d, FusedPlan *p)
{
    if (d->N <= 0 || d->C <= 0 || d->C >= 64 || d->K <= 0 || d->K % 64 || d->H <= 0 || d->W <= 0) return false;
    if (d->R <= 0 || d->S <= 0 || d->S > 8 || d->R > 100 || d->stride < 1 || d->stride > 2 || d->pad < 0 || d->pad > 100)
        return false;
    if (d->H + 2 * d->pad < d->R || d->W + 2 * d->pad < d->S || d->W % 4) return false;
    p->P = (d->H + 2 * d->pad - d->R) / d->stride + 1;
    p->Q = (d->W + 2 * d->pad - d->S) / d->stride + 1;
    if (p->Q > 128 || p->Q % 16) return false;
    p->GP = d->S <= 4 ? 4 : 8;
    p->Kf = (d->C * d->R * p->GP + 63) / 64 * 64;
    if (p->Kf > 256) return false;
    const int CR = d->C * d->R, L = (d->pad + 3) & ~3, Wp = (L + d->W + d->pad + 3) & ~3;
    // pieces per thread and output row
    if (CR * (d->W / 4) > kThreads * 6 || 64 * (p->Q / 8) > kThreads * 4 || CR * d->S * (p->Q / 16) > kThreads * 5) return false;
    const int64_t rows = (int64_t)d->N * p->P;
    if (rows >= ((int64_t)1 << 30) || (int64_t)d->N * d->K * p->P * p->Q >= ((int64_t)1 << 31) ||
        (int64_t)d->N * d->C * d->H * d->W >= ((int64_t)1 << 31))
        return false;
    p->rows = (int)rows;
    // two workgroups per compute unit; a workgroup's accumulators take at most 512 rows of 128 products
    int64_t nz = rows < 512 ? rows : 512;
    if ((rows + nz - 1) / nz > 512) nz = (rows + 511) / 512;
    if (nz > 65535) return false;
    p->RB = (int)((rows + nz - 1) / nz);
    p->nz = (int)((rows + p->RB - 1) / p->RB);
    p->lds = (size_t)2 * 128 * 64 + (size_t)2 * p->Kf * 64 + (size_t)(128 + p->Kf) * sizeof(int) + (((size_t)CR * Wp + 15) & ~(size_t)15) + 16;
    if (p->lds > 65536) return false;
    p->o_rsum = up256((size_t)p->nz * 2 * d->K * p->Kf * sizeof(int32_t));
    p->o_csum = p->o_rsum + up256((size_t)p->nz * 2 * d->K * sizeof(int));
    p->total = p->o_csum + up256((size_t)p->nz * p->Kf * sizeof(int));
    return true;
}


bool make_plan(const q8t_conv_desc *d, Plan *p)
{
    if (d->N <= 0 || d->C <= 0 || d->K <= 0 || d->H <= 0 || d->W <= 0 || d->R <= 0 || d->S <= 0) return false;
    if (d->stride < 1 || d->pad < 0) return false;
    if (d->H + 2 * d->pad < d->R || d->W + 2 * d->pad < d->S) return false;
    p->P = (d->H + 2 * d->pad - d->R) / d->stride + 1;
    p->Q = (d->W + 2 * d->pad - d->S) / d->stride + 1;
    const int64_t crs = (int64_t)d->C * d->R * d->S;
    if (crs > (1 << 24) || d->K > (1 << 22)) return false;
    p->CRS = (int)crs;
    p->Mtot = (int64_t)d->N * p->P * p->Q;
    if (p->Mtot >= ((int64_t)1 << 36)) return false;
    if ((int64_t)d->N * d->C >= ((int64_t)1 << 31) || (int64_t)d->N * d->K >= ((int64_t)1 << 31)) return false;
    p->Mp = (p->Mtot + 63) & ~(int64_t)63;
    const int64_t widest = crs > d->K ? crs : d->K;
    if ((p->Mp >> 4) * widest / kThreads >= ((int64_t)1 << 31)) return false;   // grid of the relayout kernels
    p->Rap = (2 * d->K + BM - 1) / BM * BM;
    p->Rbp = (p->CRS + 63) / 64 * 64;
    // 1x1 / stride 1 / no padding on planes of a multiple of 64 positions: operands are used in place
    p->direct = d->R == 1 && d->S == 1 && d->stride == 1 && d->pad == 0 && (p->P * p->Q) % 64 == 0 && d->K % 64 == 0 &&
                d->C % 64 == 0;
    p->cfg = (p->Rap % 256 == 0 && p->Rbp % 256 == 0 && (!p->direct || d->K % 128 == 0)) ? 2 : (p->Rbp % 128 == 0 ? 1 : 0);
    const int bm = p->cfg == 2 ? 256 : 128, bn = p->cfg == 2 ? 256 : (p->cfg == 1 ? 128 : 64);
    const int64_t tiles = (int64_t)(p->Rap / bm) * (p->Rbp / bn);
    // slices: the big tile runs one workgroup per compute unit, so aim at (just under) a multiple of
    // 256 workgroups; the small tiles at three per compute unit
    int64_t nz = p->cfg == 2 ? (tiles >= 256 ? 1 : 256 / tiles) : (768 + tiles - 1) / tiles;
    const int64_t most = (p->Mp + 1023) / 1024;              // but at least 16 steps per slice
    if (nz > most) nz = most;
    const int64_t ovf = (p->Mp + kMaxSlice - 1) / kMaxSlice;  // 32-bit accumulator bound
    if (nz < ovf) nz = ovf;
    int64_t slice = ((p->Mp + nz - 1) / nz + 63) & ~(int64_t)63;
    if (slice > kMaxSlice) slice = kMaxSlice;
    nz = (p->Mp + slice - 1) / slice;
    if (nz > 65535 || tiles * nz >= ((int64_t)1 << 30)) return false;
    p->nz = (int)nz;
    p->slice = (int)slice;
    const size_t a_bytes = up256((size_t)p->Rap * p->Mp);
    p->o_B = a_bytes;
    p->o_part = p->o_B + up256((size_t)p->Rbp * p->Mp);
    p->o_rsum = p->o_part + up256((size_t)p->nz * p->Rap * p->Rbp * sizeof(int32_t));
    p->o_csum = p->o_rsum + up256((size_t)p->nz * p->Rap * sizeof(int));
    p->total = p->o_csum + up256((size_t)p->nz * p->Rbp * sizeof(int));
    return true;
}

}  // namespace

bool q8t_gemm_wgrad_supported(const q8t_conv_desc *d)
{
    Plan p;
    FusedPlan f;
    return make_plan(d, &p) || make_fused_plan(d, &f);
}

size_t q8t_gemm_wgrad_ws(const q8t_conv_desc *d)
{
    Plan p;
    FusedPlan f;
    const size_t a = make_plan(d, &p) ? p.total : 0, b = make_fused_plan(d, &f) ? f.total : 0;
    return a > b ? a : b;
}

int q8t_gemm_wgrad(const q8t_conv_desc *d, const int16_t *g16, const q8t_qparams *qg, const int8_t *x,
                   const q8t_qparams *qx, float *dw, int64_t *acc_out, void *ws, hipStream_t st)
{
    FusedPlan f;
    if (make_fused_plan(d, &f) && q8t_aligned(g16, 16) && q8t_aligned(x, 4)) {
        if (!ws || !q8t_aligned(ws, 16)) return Q8T_ERR_WORKSPACE;
        int32_t *part = (int32_t *)ws;
        int *rsum = (int *)((char *)ws + f.o_rsum);
        int *csum = (int *)((char *)ws + f.o_csum);
        const dim3 grid((unsigned)f.nz, (unsigned)(d->K / 64));
#define Q8T_GO(GPV, NTV)                                                                                              \
    hipLaunchKernelGGL((wgrad_smallc<GPV, NTV>), grid, dim3(kThreads), f.lds, st, g16, x, d->C, d->H, d->W, d->R, d->S, \
                       d->stride, d->pad, f.P, f.Q, d->K, f.RB, f.rows, qx, part, rsum, csum)
        const int nt = f.Kf / 16;
        if (f.GP == 8) {
            if (nt == 4) Q8T_GO(8, 4); else if (nt == 8) Q8T_GO(8, 8); else if (nt == 12) Q8T_GO(8, 12); else Q8T_GO(8, 16);
        } else {
            if (nt == 4) Q8T_GO(4, 4); else if (nt == 8) Q8T_GO(4, 8); else if (nt == 12) Q8T_GO(4, 12); else Q8T_GO(4, 16);
        }
#undef Q8T_GO
        Q8T_LAUNCH_CHECK();
        const int CRS = d->C * d->R * d->S;
        const int64_t count = (int64_t)d->K * CRS;
        const int zgn = f.nz >= 64 ? 16 : (f.nz >= 8 ? 4 : 1);
        const int per = kThreads / zgn;
        hipLaunchKernelGGL(wgrad_finish, dim3((unsigned)((count + per - 1) / per)), dim3(kThreads), 0, st, part, rsum, csum,
                           f.nz, d->K, CRS, 2 * d->K, f.Kf, (int64_t)f.rows * 128, qg, qx, dw, acc_out, zgn, 0, d->S, f.GP);
        Q8T_LAUNCH_CHECK();
        return Q8T_OK;
    }
    Plan p;
    if (!make_plan(d, &p)) return Q8T_ERR_SHAPE;
    if (!ws || !q8t_aligned(ws, 16)) return Q8T_ERR_WORKSPACE;
    int8_t *A = (int8_t *)ws;
    int8_t *B = (int8_t *)ws + p.o_B;
    int32_t *part = (int32_t *)((char *)ws + p.o_part);
    int *rsum = (int *)((char *)ws + p.o_rsum);
    int *csum = (int *)((char *)ws + p.o_csum);
    const int64_t chunks = p.Mp >> 4;
    const int direct = p.direct && q8t_aligned(g16, 16) && q8t_aligned(x, 16);
    if (direct) {
        const int steps_total = (int)(p.Mtot >> 6), steps_slice = p.slice >> 6;
#define Q8T_GO(CFG)                                                                                                       \
    hipLaunchKernelGGL(gemm_direct<CFG>, dim3(q8t_gemm::xcd_grid((int64_t)(d->K / CFG::RP) * (p.Rbp / CFG::BN) * p.nz)), \
                       dim3(CFG::THREADS), 0, st, g16, x, d->K, d->C, p.P * p.Q, steps_total, steps_slice, p.Rap, p.Rbp, \
                       p.nz, part, rsum, csum)
        if (p.cfg == 2) Q8T_GO(q8t_gemm::Big);
        else if (p.cfg == 1) Q8T_GO(q8t_gemm::Mid);
        else Q8T_GO(q8t_gemm::Small);
#undef Q8T_GO
        Q8T_LAUNCH_CHECK();
    } else {
    {
        const int64_t blocks = (chunks * d->K + kThreads - 1) / kThreads;
        const int PQ = p.P * p.Q;
        if (PQ % 16 == 0 && q8t_aligned(g16, 16))
            hipLaunchKernelGGL(split16<16>, dim3((unsigned)blocks), dim3(kThreads), 0, st, g16, d->K, PQ, p.Mtot, p.Mp, qg, A);
        else if (PQ % 4 == 0 && q8t_aligned(g16, 8))
            hipLaunchKernelGGL(split16<4>, dim3((unsigned)blocks), dim3(kThreads), 0, st, g16, d->K, PQ, p.Mtot, p.Mp, qg, A);
        else
            hipLaunchKernelGGL(split16<1>, dim3((unsigned)blocks), dim3(kThreads), 0, st, g16, d->K, PQ, p.Mtot, p.Mp, qg, A);
        Q8T_LAUNCH_CHECK();
    }
    {
        ConvG g = {d->N, d->C, d->H, d->W, d->K, d->R, d->S, d->stride, d->pad, p.P, p.Q};
        const int64_t blocks = (chunks * p.CRS + kThreads - 1) / kThreads;
        const int PQ = p.P * p.Q;
        const int NI = PQ % 4 == 0 ? 1 : (PQ % 2 == 0 ? 2 : 4);
        PlaneG pg;
        pg.L = (d->pad + 3) & ~3;
        pg.pitch = (pg.L + d->W + d->pad + 3) & ~3;
        pg.PB = (d->H + 2 * d->pad) * pg.pitch;
        pg.vec = d->W % 4 == 0 && q8t_aligned(x, 4) ? 4 : (d->W % 2 == 0 && q8t_aligned(x, 2) ? 2 : 1);
        const size_t lds1 = (size_t)NI * pg.PB;
        // channels per workgroup: about 1024 dwords of work per tap, within 32 KB of LDS
        int CG = (int)(4096 / ((int64_t)NI * PQ) > 0 ? 4096 / ((int64_t)NI * PQ) : 1);
        if (lds1 * CG > 32768) CG = (int)(32768 / lds1 > 0 ? 32768 / lds1 : 1);
        if (CG > d->C) CG = d->C;
        const size_t lds = lds1 * CG;
        if (lds <= 65536 && (int64_t)CG * (NI * (int64_t)PQ + 64) < (1 << 24) && (int64_t)CG * NI * d->H * d->W < (1 << 24) &&
            (d->C + CG - 1) / CG <= 65535)
            hipLaunchKernelGGL(im2col_planes, dim3((unsigned)((d->N + NI - 1) / NI), (unsigned)((d->C + CG - 1) / CG)),
                               dim3(kThreads), lds, st, x, g, pg, NI, CG, p.Mtot, p.Mp, qx, B);
        else
            hipLaunchKernelGGL(im2col_rows, dim3((unsigned)blocks), dim3(kThreads), 0, st, x, g, p.Mtot, p.Mp, qx, B);
        Q8T_LAUNCH_CHECK();
    }
#define Q8T_GO(CFG)                                                                                                   \
    hipLaunchKernelGGL(gemm_nt<CFG>, dim3(q8t_gemm::xcd_grid((int64_t)(p.Rap / CFG::BM) * (p.Rbp / CFG::BN) * p.nz)), \
                       dim3(CFG::THREADS), 0, st, A, B, p.Mp, p.slice, p.Rap, p.Rbp, p.nz, part, rsum, csum)
    if (p.cfg == 2) Q8T_GO(q8t_gemm::Big);
    else if (p.cfg == 1) Q8T_GO(q8t_gemm::Mid);
    else Q8T_GO(q8t_gemm::Small);
#undef Q8T_GO
    Q8T_LAUNCH_CHECK();
    }
    {
        const int64_t count = (int64_t)d->K * p.CRS;
        const int zgn = p.nz >= 64 ? 16 : (p.nz >= 8 ? 4 : 1);   // lanes sharing the slices of one output
        const int per = kThreads / zgn;
        hipLaunchKernelGGL(wgrad_finish, dim3((unsigned)((count + per - 1) / per)), dim3(kThreads), 0, st,
                           part, rsum, csum, p.nz, d->K, p.CRS, p.Rap, p.Rbp, p.Mp, qg, qx, dw, acc_out, zgn,
                           direct ? (p.cfg == 2 ? 128 : 64) : 0, 1, 0);
        Q8T_LAUNCH_CHECK();
    }
    return Q8T_OK;
}
