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

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int BM = 128;
constexpr int PITCH = 80;
constexpr int kMaxSlice = 65536;

__device__ __forceinline__ int bytesum4(uint32_t v) { return __builtin_amdgcn_sdot4((int)v, 0x01010101, 0, false); }
__device__ __forceinline__ int bytesum16(const uint4 &v)
{
    return bytesum4(v.x) + bytesum4(v.y) + bytesum4(v.z) + bytesum4(v.w);
}

// ---- A': byte planes of the 16-bit gradient, [2K][Mp] -----------------------------------------
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
    int n = (int)(m0 / PQ), pq = (int)(m0 - (int64_t)n * PQ);
    uint32_t hi[4] = {0, 0, 0, 0}, lo[4] = {0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        int s = zsg;
        if (m0 + i < Mtot) s = g16[((size_t)n * K + k) * PQ + pq];
        hi[i >> 2] |= (uint32_t)((s >> 8) & 255) << (8 * (i & 3));
        lo[i >> 2] |= (uint32_t)(((s & 255) - 128) & 255) << (8 * (i & 3));
        if (++pq == PQ) {
            pq = 0;
            ++n;
        }
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

// ---- C[z][i][j] = sum over slice z of A'[i][m] * B'[j][m] ---------------------------------------
// Also leaves the sums of the staged bytes per row (of A') and per column (row of B') and slice.
template <int BN>
__global__ __launch_bounds__(kThreads) void gemm_nt(const int8_t *__restrict__ A, const int8_t *__restrict__ B, int64_t Mp,
                                                    int slice, int Rap, int Rbp, int32_t *__restrict__ part,
                                                    int *__restrict__ rsum, int *__restrict__ csum)
{
    constexpr int WM = BN == 128 ? 2 : 4;
    constexpr int MT = BM / WM / 16;
    constexpr int NT = 4;
    constexpr int NB = BN / 64;

    __shared__ __align__(16) int8_t sA[2][BM * PITCH];
    __shared__ __align__(16) int8_t sB[2][BN * PITCH];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, kb = lane >> 4;
    const int r0 = blockIdx.x * BM, c0 = blockIdx.y * BN, z = blockIdx.z;
    const int64_t mb = (int64_t)z * slice;
    const int64_t me = mb + slice < Mp ? mb + slice : Mp;
    const int steps = (int)((me - mb) >> 6);

    const int ar = tid >> 1, ao = (tid & 1) * 32;
    const int br = NB == 2 ? tid >> 1 : tid >> 2;
    const int bo = NB == 2 ? (tid & 1) * 32 : (tid & 3) * 16;
    const int8_t *pa = A + (size_t)(r0 + ar) * Mp + mb + ao;
    const int8_t *pb = B + (size_t)(c0 + br) * Mp + mb + bo;

    uint4 a0, a1, b0, b1;
    a0 = a1 = b0 = b1 = make_uint4(0, 0, 0, 0);
    int sa = 0, sb = 0;
    auto load = [&]() {
        a0 = *reinterpret_cast<const uint4 *>(pa);
        a1 = *reinterpret_cast<const uint4 *>(pa + 16);
        b0 = *reinterpret_cast<const uint4 *>(pb);
        if (NB == 2) b1 = *reinterpret_cast<const uint4 *>(pb + 16);
        pa += 64;
        pb += 64;
    };
    auto store = [&](int buf) {
        *reinterpret_cast<uint4 *>(&sA[buf][ar * PITCH + ao]) = a0;
        *reinterpret_cast<uint4 *>(&sA[buf][ar * PITCH + ao + 16]) = a1;
        *reinterpret_cast<uint4 *>(&sB[buf][br * PITCH + bo]) = b0;
        if (NB == 2) *reinterpret_cast<uint4 *>(&sB[buf][br * PITCH + bo + 16]) = b1;
        sa += bytesum16(a0) + bytesum16(a1);
        sb += bytesum16(b0);
        if (NB == 2) sb += bytesum16(b1);
    };

    const int rowbase = BN == 128 ? (wave & 1) * 64 : wave * 32;
    const int colbase = BN == 128 ? (wave >> 1) * 64 : 0;
    v4i acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = (v4i){0, 0, 0, 0};

    if (steps > 0) {
        load();
        store(0);
    }
    __syncthreads();
    for (int s = 0; s < steps; ++s) {
        const int buf = s & 1;
        if (s + 1 < steps) load();
        v4i bf[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            bf[nt] = *reinterpret_cast<const v4i *>(&sB[buf][(colbase + nt * 16 + l16) * PITCH + kb * 16]);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const v4i a = *reinterpret_cast<const v4i *>(&sA[buf][(rowbase + mt * 16 + l16) * PITCH + kb * 16]);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, bf[nt], acc[mt][nt], 0, 0, 0);
        }
        if (s + 1 < steps) store(buf ^ 1);
        __syncthreads();
    }

    // byte sums of this slice: the two (or four) threads of a row hold its pieces
    sa += __shfl_xor(sa, 1, Q8T_WAVE);
    sb += __shfl_xor(sb, 1, Q8T_WAVE);
    if (NB == 1) sb += __shfl_xor(sb, 2, Q8T_WAVE);
    if (blockIdx.y == 0 && (tid & 1) == 0) rsum[(size_t)z * Rap + r0 + ar] = sa;
    if (blockIdx.x == 0 && (NB == 2 ? (tid & 1) == 0 : (tid & 3) == 0)) csum[(size_t)z * Rbp + c0 + br] = sb;

    int32_t *dst = part + (size_t)z * Rap * Rbp;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                dst[(size_t)(r0 + rowbase + mt * 16 + kb * 4 + j) * Rbp + c0 + colbase + nt * 16 + l16] = acc[mt][nt][j];
}

// ---- slices -> exact 64-bit sums -> outputs ------------------------------------------------------
// acc(k,col) = sum (g - zg)(x - zx),  g = 256*hi + lo + 128 :
//   256*S_hi + S_lo + (128 - zg)*colsum - zx*(256*rowsum_hi + rowsum_lo + (128 - zg)*Mp)
__global__ __launch_bounds__(kThreads) void wgrad_finish(const int32_t *__restrict__ part, const int *__restrict__ rsum,
                                                         const int *__restrict__ csum, int nz, int K, int CRS, int Rap,
                                                         int Rbp, int64_t Mp, const q8t_qparams *__restrict__ qpg,
                                                         const q8t_qparams *__restrict__ qpx, float *__restrict__ dw,
                                                         int64_t *__restrict__ acc_out)
{
    const int64_t id = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (id >= (int64_t)K * CRS) return;
    const int k = (int)(id / CRS), col = (int)(id - (int64_t)k * CRS);
    const int zg = qpg->zero_point - (1 << (qpg->bits - 1)), zx = qpx->zero_point - (1 << (qpx->bits - 1));
    int64_t shi = 0, slo = 0, rhi = 0, rlo = 0, cs = 0;
    for (int z = 0; z < nz; ++z) {
        shi += part[((size_t)z * Rap + k) * Rbp + col];
        slo += part[((size_t)z * Rap + K + k) * Rbp + col];
        rhi += rsum[(size_t)z * Rap + k];
        rlo += rsum[(size_t)z * Rap + K + k];
        cs += csum[(size_t)z * Rbp + col];
    }
    const int64_t ca = 128 - zg;
    const int64_t v = 256 * shi + slo + ca * cs - (int64_t)zx * (256 * rhi + rlo + ca * Mp);
    if (acc_out) acc_out[id] = v;
    if (dw) dw[id] = (float)((double)v * (double)(qpg->scale * qpx->scale));
}

struct Plan {
    int P, Q, CRS, Rap, Rbp, nz, slice;
    int64_t Mtot, Mp;
    size_t o_B, o_part, o_rsum, o_csum, total;
};

inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

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
    if (p->Mtot >= ((int64_t)1 << 40)) return false;
    if ((int64_t)d->N * d->C >= ((int64_t)1 << 31) || (int64_t)d->N * d->K >= ((int64_t)1 << 31)) return false;
    p->Mp = (p->Mtot + 63) & ~(int64_t)63;
    const int64_t widest = crs > d->K ? crs : d->K;
    if ((p->Mp >> 4) * widest / kThreads >= ((int64_t)1 << 31)) return false;   // grid of the relayout kernels
    p->Rap = (2 * d->K + BM - 1) / BM * BM;
    p->Rbp = (p->CRS + 63) / 64 * 64;
    const int64_t tiles = (int64_t)(p->Rap / BM) * (p->Rbp % 128 == 0 ? p->Rbp / 128 : p->Rbp / 64);
    int64_t nz = (1024 + tiles - 1) / tiles;                 // enough workgroups to fill the chip
    const int64_t most = (p->Mp + 1023) / 1024;              // but at least 16 steps per slice
    if (nz > most) nz = most;
    const int64_t ovf = (p->Mp + kMaxSlice - 1) / kMaxSlice;  // 32-bit accumulator bound
    if (nz < ovf) nz = ovf;
    int64_t slice = ((p->Mp + nz - 1) / nz + 63) & ~(int64_t)63;
    if (slice > kMaxSlice) slice = kMaxSlice;
    nz = (p->Mp + slice - 1) / slice;
    if (nz > 65535) return false;
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
    return make_plan(d, &p);
}

size_t q8t_gemm_wgrad_ws(const q8t_conv_desc *d)
{
    Plan p;
    return make_plan(d, &p) ? p.total : 0;
}

int q8t_gemm_wgrad(const q8t_conv_desc *d, const int16_t *g16, const q8t_qparams *qg, const int8_t *x,
                   const q8t_qparams *qx, float *dw, int64_t *acc_out, void *ws, hipStream_t st)
{
    Plan p;
    if (!make_plan(d, &p)) return Q8T_ERR_SHAPE;
    if (!ws || !q8t_aligned(ws, 16)) return Q8T_ERR_WORKSPACE;
    int8_t *A = (int8_t *)ws;
    int8_t *B = (int8_t *)ws + p.o_B;
    int32_t *part = (int32_t *)((char *)ws + p.o_part);
    int *rsum = (int *)((char *)ws + p.o_rsum);
    int *csum = (int *)((char *)ws + p.o_csum);
    const int64_t chunks = p.Mp >> 4;
    {
        const int64_t blocks = (chunks * d->K + kThreads - 1) / kThreads;
        hipLaunchKernelGGL(split16, dim3((unsigned)blocks), dim3(kThreads), 0, st, g16, d->K, p.P * p.Q, p.Mtot, p.Mp, qg, A);
        Q8T_LAUNCH_CHECK();
    }
    {
        ConvG g = {d->N, d->C, d->H, d->W, d->K, d->R, d->S, d->stride, d->pad, p.P, p.Q};
        const int64_t blocks = (chunks * p.CRS + kThreads - 1) / kThreads;
        hipLaunchKernelGGL(im2col_rows, dim3((unsigned)blocks), dim3(kThreads), 0, st, x, g, p.Mtot, p.Mp, qx, B);
        Q8T_LAUNCH_CHECK();
    }
    if (p.Rbp % 128 == 0)
        hipLaunchKernelGGL(gemm_nt<128>, dim3((unsigned)(p.Rap / BM), (unsigned)(p.Rbp / 128), (unsigned)p.nz),
                           dim3(kThreads), 0, st, A, B, p.Mp, p.slice, p.Rap, p.Rbp, part, rsum, csum);
    else
        hipLaunchKernelGGL(gemm_nt<64>, dim3((unsigned)(p.Rap / BM), (unsigned)(p.Rbp / 64), (unsigned)p.nz),
                           dim3(kThreads), 0, st, A, B, p.Mp, p.slice, p.Rap, p.Rbp, part, rsum, csum);
    Q8T_LAUNCH_CHECK();
    {
        const int64_t count = (int64_t)d->K * p.CRS;
        hipLaunchKernelGGL(wgrad_finish, dim3((unsigned)((count + kThreads - 1) / kThreads)), dim3(kThreads), 0, st,
                           part, rsum, csum, p.nz, d->K, p.CRS, p.Rap, p.Rbp, p.Mp, qg, qx, dw, acc_out);
        Q8T_LAUNCH_CHECK();
    }
    return Q8T_OK;
}
