// Forward convolution of a layer with very few input channels and 64 output channels (the first layer of a
// ResNet: 3 -> 64, 7x7, stride 2), 8-bit operands with 32-bit accumulation (Section 4).
//
// GEMM view: rows = output positions, columns = the 64 output channels, reduction = (channel, filter row) groups of
// 8 columns each: the S <= 8 taps of one filter row, the surplus columns meeting filter entries that hold the
// filter's zero code, so whatever input byte sits under them contributes nothing once the zero points are taken out:
//    sum (a - za)(b - zb) = sum ab - zb * sum a - za * sum b + Kc * za * zb       (all sums over the Kc columns).
// The operand rows are never built.  A workgroup stages the band of input rows under RPB output rows once (every
// channel, zero code in the padding); the 8 bytes of a group for output column q are then 8 consecutive bytes of a
// staged row, starting at q * stride, and a lane reads its MFMA fragment (16 bytes = two groups) straight from the
// band with two unaligned 8-byte LDS reads.  The whole [64][Kc] filter lives in registers (v_mfma_i32_16x16x64_i8
// fragments, loaded once per workgroup).  Row sums: v_dot4 on the fragments, folded over the four lanes that share
// a position.  HBM sees the int8 input once (plus the overlap of neighbouring bands) and the fp32 result once.
#include "q8t_common.h"
#include "q8t_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kRPB = 8;       // output rows per workgroup
constexpr int kStageU = 8;    // dwords a thread has in flight while staging
constexpr int kTP = 36;       // ints per channel row of a wavefront's result tile in LDS (32 positions + 4: 144 bytes)

struct FirstGeom {
    int N, C, H, W, R, S, stride, pad, P, Q;
    int CR;        // (channel, filter row) groups
    int NR;        // staged input rows per channel: (kRPB - 1) * stride + R
    int L, Wp;     // left margin and pitch of a staged row (multiples of 4)
    int mtiles;    // 16-position tiles per output row
    int band_bytes;   // LDS bytes of the band (a multiple of 16); the wavefronts' result tiles follow
    int vec;       // 16-byte stores allowed
};

// filter [64][C*R*S] -> [64][Kc], column g * 8 + s = entry (g, s) of group g, the filter's zero code elsewhere;
// sums per output channel over all Kc columns
__global__ __launch_bounds__(64) void repack_first(const int8_t *__restrict__ w, int CRS, int CR, int S, int Kc,
                                                   const q8t_qparams *__restrict__ qpw, int8_t *__restrict__ wt,
                                                   int *__restrict__ colsum)
{
    const int k = blockIdx.x;
    const int zb = qpw->zero_point - (1 << (qpw->bits - 1));
    int sum = 0;
    for (int j = threadIdx.x; j < Kc; j += 64) {
        const int g = j >> 3, s = j & 7;
        const int v = (g < CR && s < S) ? (int)w[(size_t)k * CRS + g * S + s] : zb;
        wt[(size_t)k * Kc + j] = (int8_t)v;
        sum += v;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, Q8T_WAVE);
    if (threadIdx.x == 0) colsum[k] = sum;
}

template <int KS>
__global__ __launch_bounds__(kThreads) void first_conv(const int8_t *__restrict__ x, const FirstGeom g,
                                                       const int8_t *__restrict__ wt, const int *__restrict__ colsum,
                                                       const q8t_qparams *__restrict__ qpx,
                                                       const q8t_qparams *__restrict__ qpw, float *__restrict__ out_f,
                                                       int32_t *__restrict__ out_acc, Q8tConvStat *__restrict__ bnpart)
{
    extern __shared__ __align__(16) int8_t band[];   // [C * NR][Wp] + slack
    constexpr int Kc = 64 * KS;
    const int n = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, kb = lane >> 4;
    const int pbeg = blockIdx.x * kRPB, nrows = min(kRPB, g.P - pbeg);
    const int za = qpx->zero_point - (1 << (qpx->bits - 1)), zb = qpw->zero_point - (1 << (qpw->bits - 1));
    const float sc = qpx->scale * qpw->scale;
    const uint32_t zfill = (uint32_t)(za & 255) * 0x01010101u;
    const uint32_t kzz = (uint32_t)Kc * (uint32_t)za * (uint32_t)zb;

    // ---- stage the band: a wavefront per staged row and round (no per-lane index arithmetic), lanes over the dwords
    // of the row; the loads of the first round are in flight while the zero code is filled in ----
    const int W4 = g.W >> 2, nstaged = g.C * g.NR;
    const int h0 = pbeg * g.stride - g.pad;
    const int band_dwords = (g.C * g.NR * g.Wp + 16 * g.stride + 32) >> 2;
    for (int r0 = 0; r0 < nstaged; r0 += (kThreads / 64) * kStageU) {
        for (int w0 = 0; w0 < W4; w0 += 64) {
            uint32_t v[kStageU];
            int dst[kStageU];
            const int w4 = w0 + lane;
#pragma unroll
            for (int u = 0; u < kStageU; ++u) {
                const int cr = r0 + u * (kThreads / 64) + wave;      // uniform in the wavefront
                const int c = cr / g.NR, h = h0 + cr - c * g.NR;
                dst[u] = -1;
                v[u] = 0;
                if (cr < nstaged && (unsigned)h < (unsigned)g.H && w4 < W4) {
                    dst[u] = cr * g.Wp + g.L + 4 * w4;
                    v[u] = *reinterpret_cast<const uint32_t *>(x + (((size_t)n * g.C + c) * g.H + h) * g.W + 4 * w4);
                }
            }
            if (r0 == 0 && w0 == 0) {
                uint32_t *b32 = reinterpret_cast<uint32_t *>(band);
                for (int i = tid; i < band_dwords; i += kThreads) b32[i] = zfill;
                __syncthreads();
            }
#pragma unroll
            for (int u = 0; u < kStageU; ++u)
                if (dst[u] >= 0) *reinterpret_cast<uint32_t *>(band + dst[u]) = v[u];
        }
    }

    // ---- the filter, in registers: bf[ks][nt] = columns ks*64 + kb*16 .. +15 of output channel nt*16 + l16 ----
    v4i bf[KS][4];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
            bf[ks][nt] = *reinterpret_cast<const v4i *>(wt + (size_t)(nt * 16 + l16) * Kc + ks * 64 + kb * 16);
    int ncs[4];   // minus the column term of the zero-point correction
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) ncs[nt] = (int)(0u - (uint32_t)za * (uint32_t)colsum[nt * 16 + l16]);
    // band offsets of the lane's two groups per K-step (a surplus group reads group 0: its filter entries are zero codes)
    int goff[KS][2];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int grp = ks * 8 + kb * 2 + t;
            const int c = grp / g.R, r = grp - c * g.R;
            goff[ks][t] = (grp < g.CR ? (c * g.NR + r) * g.Wp : 0) + g.L - g.pad;
        }

    long long st_s[4] = {0, 0, 0, 0};
    int st_mn[4], st_mx[4];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
        st_mn[nt] = 2147483647;
        st_mx[nt] = -2147483647 - 1;
    }
    __syncthreads();   // the band is complete

    // A task = one output row x two neighbouring 16-position tiles.  The corrected sums go through a wavefront-private
    // LDS tile [64 channels][32 positions] and leave as 16-byte pieces with the eight lanes of a channel side by side:
    // every store instruction writes whole 128-byte lines (straight from the accumulators, neighbouring lanes hold
    // different channels, and the 16-byte requests of 64 different lines bound the kernel at 60% of this rate).
    int *T = reinterpret_cast<int *>(band + g.band_bytes) + wave * (64 * kTP);
    const int pairs = (g.mtiles + 1) >> 1, tasks = nrows * pairs;
    for (int t = wave; t < tasks; t += kThreads / 64) {
        const int pl = t / pairs, mp = t - pl * pairs;
        const int p = pbeg + pl;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int mt = 2 * mp + i;
            if (mt >= g.mtiles) break;   // uniform
            const int abase = pl * g.stride * g.Wp + (mt * 16 + l16) * g.stride;
            v4i acc[4];
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) acc[nt] = (v4i){ncs[nt], ncs[nt], ncs[nt], ncs[nt]};   // the column term rides along
            int rs = 0;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                uint64_t lo, hi;
                __builtin_memcpy(&lo, band + goff[ks][0] + abase, 8);
                __builtin_memcpy(&hi, band + goff[ks][1] + abase, 8);
                const v4i af = {(int)(uint32_t)lo, (int)(uint32_t)(lo >> 32), (int)(uint32_t)hi, (int)(uint32_t)(hi >> 32)};
#pragma unroll
                for (int q = 0; q < 4; ++q) rs = __builtin_amdgcn_sdot4(af[q], 0x01010101, rs, false);
#pragma unroll
                for (int nt = 0; nt < 4; ++nt)
                    acc[nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af, bf[ks][nt], acc[nt], 0, 0, 0);
            }
            // row sum of position l16: fold the four lanes (kb) that hold its columns; then fetch those of the lane's
            // own four result positions kb * 4 + j
            rs += __shfl_xor(rs, 16, Q8T_WAVE);
            rs += __shfl_xor(rs, 32, Q8T_WAVE);
            uint32_t tj[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) tj[j] = kzz - (uint32_t)zb * (uint32_t)__shfl(rs, kb * 4 + j, Q8T_WAVE);
            const int r0 = mt * 16 + kb * 4;
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                v4i c4;
#pragma unroll
                for (int j = 0; j < 4; ++j) c4[j] = (int)((uint32_t)acc[nt][j] + tj[j]);
                if (bnpart) {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (r0 + j < g.Q) {
                            st_s[nt] += c4[j];
                            st_mn[nt] = min(st_mn[nt], c4[j]);
                            st_mx[nt] = max(st_mx[nt], c4[j]);
                        }
                }
                *reinterpret_cast<v4i *>(&T[(nt * 16 + l16) * kTP + i * 16 + kb * 4]) = c4;
            }
        }
        __builtin_amdgcn_wave_barrier();
        // lane -> piece lane % 8 (4 positions) of channels lane / 8 + 8 * it
        const int piece = lane & 7, pos = mp * 32 + piece * 4;
        const bool live = pos < g.Q;
        const size_t obase = (((size_t)n * 64 + (lane >> 3)) * g.P + p) * g.Q + pos;
        const size_t ostep = (size_t)8 * g.P * g.Q;
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const v4i c4 = *reinterpret_cast<const v4i *>(&T[(it * 8 + (lane >> 3)) * kTP + piece * 4]);
            const size_t o = obase + it * ostep;
            if (!live) continue;
            if (g.vec && pos + 3 < g.Q) {
                if (out_acc) *reinterpret_cast<int4 *>(out_acc + o) = make_int4(c4[0], c4[1], c4[2], c4[3]);
                if (out_f)
                    *reinterpret_cast<float4 *>(out_f + o) =
                        make_float4(sc * (float)c4[0], sc * (float)c4[1], sc * (float)c4[2], sc * (float)c4[3]);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (pos + j >= g.Q) continue;
                    if (out_acc) out_acc[o + j] = c4[j];
                    if (out_f) out_f[o + j] = sc * (float)c4[j];
                }
            }
        }
        __builtin_amdgcn_wave_barrier();   // the tile is rewritten by the next task
    }

    if (bnpart) {
        // fold the 16 lanes x 4 wavefronts that share a channel through LDS slots (the band is no longer needed)
        unsigned long long *slot_s = reinterpret_cast<unsigned long long *>(band);
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

// the last tile of an output row may reach up to 15 positions past the row: its (discarded) fragments are read from
// the bytes behind the band
// (at least the 1 KB of slots that fold the statistics at the end)
int band_bytes(const FirstGeom &g)
{
    const int band = (g.C * g.NR * g.Wp + 16 * g.stride + 32 + 15) & ~15;
    return band < 1024 ? 1024 : band;
}
size_t lds_bytes(const FirstGeom &g) { return (size_t)band_bytes(g) + (kThreads / 64) * 64 * kTP * sizeof(int); }

bool make_geom(const q8t_conv_desc *d, FirstGeom *g)
{
    if (d->N <= 0 || d->N > 65535 || d->C <= 0 || d->C >= 64 || d->K != 64 || d->H <= 0 || d->W <= 0) return false;
    if (d->R <= 0 || d->R > 32 || d->S <= 0 || d->S > 8 || d->stride < 1 || d->stride > 4 || d->pad < 0 || d->pad > 16) return false;
    if (d->H + 2 * d->pad < d->R || d->W + 2 * d->pad < d->S || d->W % 4) return false;
    g->N = d->N; g->C = d->C; g->H = d->H; g->W = d->W; g->R = d->R; g->S = d->S; g->stride = d->stride; g->pad = d->pad;
    g->P = (d->H + 2 * d->pad - d->R) / d->stride + 1;
    g->Q = (d->W + 2 * d->pad - d->S) / d->stride + 1;
    g->CR = d->C * d->R;
    if (g->CR > 32) return false;
    g->NR = (kRPB - 1) * d->stride + d->R;
    g->L = (d->pad + 3) & ~3;
    g->Wp = (g->L + d->W + d->pad + 3) & ~3;
    g->mtiles = (g->Q + 15) / 16;
    if ((int64_t)g->C * g->NR * g->Wp > 60 * 1024) return false;
    g->band_bytes = band_bytes(*g);
    if ((int64_t)d->N * 64 * g->P * g->Q >= ((int64_t)1 << 40) || (int64_t)d->N * d->C * d->H * d->W >= ((int64_t)1 << 40)) return false;
    return true;
}

int ksteps(const FirstGeom &g) { return (g.CR + 7) / 8; }

}  // namespace

bool q8t_first_conv_supported(const q8t_conv_desc *d, const void *a, const void *out_f, const void *out_acc)
{
    FirstGeom g;
    if (!make_geom(d, &g)) return false;
    if (lds_bytes(g) > 64 * 1024) return false;
    return q8t_aligned(a, 4) && q8t_aligned(out_f, 4) && q8t_aligned(out_acc, 4);
}

size_t q8t_first_conv_ws(const q8t_conv_desc *d)
{
    FirstGeom g;
    if (!make_geom(d, &g)) return 0;
    return (size_t)64 * 64 * ksteps(g) + 256 + 64 * sizeof(int);
}

size_t q8t_first_conv_stats_ws(const q8t_conv_desc *d)
{
    FirstGeom g;
    if (!make_geom(d, &g)) return 0;
    return (size_t)((g.P + kRPB - 1) / kRPB) * d->N * 64 * sizeof(Q8tConvStat);
}

int q8t_first_conv(const q8t_conv_desc *d, const void *a, const q8t_qparams *qa, const void *b, const q8t_qparams *qb,
                   float *out_f, void *out_acc, float *bn_stats, void *stats_ws, void *ws, hipStream_t st)
{
    FirstGeom g;
    if (!make_geom(d, &g)) return Q8T_ERR_SHAPE;
    if (!ws || !q8t_aligned(ws, 16)) return Q8T_ERR_WORKSPACE;
    if (bn_stats && (!stats_ws || !q8t_aligned(stats_ws, 16))) return Q8T_ERR_WORKSPACE;
    const int KS = ksteps(g), Kc = 64 * KS;
    int8_t *wt = (int8_t *)ws;
    int *colsum = (int *)((char *)ws + (((size_t)64 * Kc + 255) & ~(size_t)255));
    Q8tConvStat *bnp = bn_stats ? (Q8tConvStat *)stats_ws : (Q8tConvStat *)nullptr;
    g.vec = g.Q % 4 == 0 && q8t_aligned(out_f, 16) && q8t_aligned(out_acc, 16);
    hipLaunchKernelGGL(repack_first, dim3(64), dim3(64), 0, st, (const int8_t *)b, d->C * d->R * d->S, g.CR, d->S, Kc, qb, wt,
                       colsum);
    Q8T_LAUNCH_CHECK();
    const dim3 grid((unsigned)((g.P + kRPB - 1) / kRPB), (unsigned)d->N);
    const size_t lds = lds_bytes(g);
#define Q8T_FIRST(KSV)                                                                                                    \
    {                                                                                                                     \
        static Q8tLdsOptIn optin;                                                                                         \
        if (q8t_allow_lds(optin, (const void *)first_conv<KSV>, 64 * 1024) != Q8T_OK) return Q8T_ERR_HIP;                \
        hipLaunchKernelGGL(first_conv<KSV>, grid, dim3(kThreads), lds, st, (const int8_t *)a, g, wt, colsum, qa, qb, out_f, \
                           (int32_t *)out_acc, bnp);                                                                      \
    }
    switch (KS) {
    case 1: Q8T_FIRST(1) break;
    case 2: Q8T_FIRST(2) break;
    case 3: Q8T_FIRST(3) break;
    default: Q8T_FIRST(4) break;
    }
#undef Q8T_FIRST
    Q8T_LAUNCH_CHECK();
    if (bnp) {
        const int nwg = (int)(grid.x * grid.y);
        return q8t_conv_stats_finalize(bnp, 64, nwg, nwg, (double)d->N * g.P * g.Q, qa, qb, bn_stats, st);
    }
    return Q8T_OK;
}
