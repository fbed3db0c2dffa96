// Specialised int8 implicit-GEMM convolution for the ResNet hot shapes: stride 1, 3x3 pad 1 or
// 1x1 pad 0, channel counts that are multiples of 64 (forward, and the layer gradient, which for
// stride 1 is the same convolution with the filter flipped and its channel roles swapped;
// Section 4, eq. (grad_layer)).
//
// GEMM view: rows = flattened (image, y, x) output positions, cols = output channels,
// reduction = (tap, input channel).  Per workgroup: 256 consecutive rows x 64 output channels,
// 4 wavefronts of 64x64 (4x4 v_mfma_i32_16x16x64_i8 tiles); one MFMA K-step = one filter tap over
// 64 input channels.
//
// Data movement (the kernel is HBM-bound for 64-channel layers: 1 byte in, 4 bytes out per element):
//  * activations are NCHW int8, but MFMA wants the reduction index contiguous per lane, so the
//    tile (with its halo of W+1 positions on either side) is transposed on the way into LDS:
//    each lane loads 4 positions x 4 channels as 4 dwords, transposes 4x4 bytes with v_perm and
//    writes [position][channel] rows of 80 bytes (64 + 16 pad: 16-byte aligned, conflict-free
//    ds_read_b128 for the A fragments);
//  * a tap is a row offset into that tile; taps that fall outside the image are replaced by the
//    operand's zero point per lane (border predicates), so padding contributes exactly nothing;
//  * weights are repacked once per call into [tap][out-channel][in-channel] (and their per-channel
//    sums taken) by a small pre-pass; row sums of A come from v_dot4 on the fragments already in
//    registers.  Epilogue: zero-point correction, dequantization, float4 stores (4 consecutive
//    positions of one output channel per lane).
#include "q8t_common.h"
#include "q8t_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int BM = 256;          // rows per workgroup
constexpr int CH = 64;           // channels per reduction chunk / output channels per workgroup
constexpr int ROWB = 80;         // LDS bytes per staged row
constexpr int MAX_W = 64;        // widest image row the 3x3 variant stages
constexpr int MAX_STAGE_ROWS = BM + 2 * (MAX_W + 1) + 8;

struct FastGeom {
    int N, C, K;      // images, reduction channels, output channels
    int H, W, PQ;     // plane
    int64_t M;        // N * PQ
    int tiles;        // ceil(M / BM)
};

// ---- weight pre-pass: repack + per-output-channel sums -----------------------------------------
// out[(oc/64)][cc][tap][oc%64][ch%64] = W'(oc, ch, tap);  forward: W'(oc,ch,r,s) = W[oc][ch][r][s];
// layer gradient: W'(oc,ch,r,s) = W[ch][oc][R-1-r][S-1-s]  (oc = input channel of the layer).
__global__ __launch_bounds__(kThreads) void repack_weights(const int8_t *__restrict__ w, int Kf, int Cf, int R,
                                                           int S, int dgrad, int8_t *__restrict__ out,
                                                           int *__restrict__ colsum)
{
    __shared__ int red[kThreads / 64];
    const int OC = dgrad ? Cf : Kf, CHN = dgrad ? Kf : Cf;
    const int oc = blockIdx.x;
    const int taps = R * S, CC = CHN / CH;
    int sum = 0;
    for (int e = threadIdx.x; e < taps * CHN; e += kThreads) {
        const int tap = e / CHN, ch = e - tap * CHN;
        const int r = tap / S, s = tap - r * S;
        int v;
        if (!dgrad)
            v = w[(((int64_t)oc * Cf + ch) * R + r) * S + s];
        else
            v = w[(((int64_t)ch * Cf + oc) * R + (R - 1 - r)) * S + (S - 1 - s)];
        sum += v;
        const int64_t o = ((((int64_t)(oc / CH) * CC + ch / CH) * taps + tap) * CH + (oc % CH)) * CH + (ch % CH);
        out[o] = (int8_t)v;
    }
    sum = wave_reduce(sum, [](int a, int b) { return a + b; });
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) colsum[oc] = red[0] + red[1] + red[2] + red[3];
    (void)OC;
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

// XCD-aware order: consecutive workgroup ids go round-robin over the 8 XCDs; give each XCD one
// contiguous run of tiles so that neighbouring tiles (which share halo rows) share an L2.
__device__ __forceinline__ int xcd_tile(int bid, int tiles)
{
    const int per = (tiles + 7) / 8;
    const int t = (bid & 7) * per + (bid >> 3);
    return t;
}

template <int TAPS>
__global__ __launch_bounds__(kThreads, 2) void conv_s1_kernel(const int8_t *__restrict__ x,
                                                              const int8_t *__restrict__ wpk,
                                                              const int *__restrict__ colsum,
                                                              const q8t_qparams *__restrict__ qpa,
                                                              const q8t_qparams *__restrict__ qpb, FastGeom g,
                                                              float *__restrict__ y, int32_t *__restrict__ acc_out)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    constexpr int A_BYTES = (TAPS == 9 ? MAX_STAGE_ROWS : BM + 8) * ROWB;
    uint8_t *As = smem;
    uint8_t *Bs = smem + A_BYTES;
    int *rs = reinterpret_cast<int *>(smem + A_BYTES + TAPS * CH * ROWB);

    const int tile = xcd_tile(blockIdx.x, g.tiles);
    if (tile >= g.tiles) return;
    const int occ = blockIdx.y;  // output-channel chunk
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, kb = lane >> 4;

    const int za = qpa->zero_point - 128, zb = qpb->zero_point - 128;
    const float sc = qpa->scale * qpb->scale;
    const uint32_t zavec = (uint32_t)(za & 255) * 0x01010101u;

    const int64_t g0 = (int64_t)tile * BM;
    const int halo = (TAPS == 9) ? g.W + 1 : 0;
    const int64_t stage_start = (g0 - halo) & ~(int64_t)3;  // arithmetic: also right for negatives
    const int stage_rows = (int)(((g0 + BM + halo + 3) & ~(int64_t)3) - stage_start);
    const int row_base = (int)(g0 - stage_start) + wave * 64;  // LDS row of this wave's first output row

    // border predicates of this lane's A rows (one row per m-tile: row l16 of the 16)
    bool ok_up[4], ok_dn[4], ok_lf[4], ok_rt[4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
        const int64_t gr = g0 + wave * 64 + mt * 16 + l16;
        const int pos = (int)(gr % g.PQ);
        const int p = pos / g.W, q = pos - p * g.W;
        ok_up[mt] = p > 0;
        ok_dn[mt] = p < g.H - 1;
        ok_lf[mt] = q > 0;
        ok_rt[mt] = q < g.W - 1;
    }

    v4i acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = (v4i){0, 0, 0, 0};
    int rsum[4] = {0, 0, 0, 0};

    const int CC = g.C / CH;
    for (int cc = 0; cc < CC; ++cc) {
        __syncthreads();
        // ---- stage A: [position][64 channels], transposing 4x4 bytes per lane ----
        {
            const int npg = stage_rows >> 2;        // groups of 4 positions
            const int pg_blocks = (npg + 15) >> 4;  // blocks of 16 position groups
            // one wavefront instruction = 16 position groups x 4 channel groups: 64-byte global
            // segments per channel, 16 distinct LDS banks per store
            for (int slab = wave; slab < pg_blocks * 4; slab += kThreads / 64) {
                const int pgb = slab % pg_blocks, cgb = slab / pg_blocks;
                const int pg = pgb * 16 + (lane & 15), cg = cgb * 4 + (lane >> 4);
                if (pg < npg) {
                    const int64_t gr = stage_start + (int64_t)pg * 4;
                    uint32_t in[4] = {0, 0, 0, 0}, out[4];
                    if (gr >= 0 && gr < g.M) {
                        const int b = (int)(gr / g.PQ);
                        const int pos = (int)(gr - (int64_t)b * g.PQ);
                        const int8_t *src = x + ((int64_t)b * g.C + cc * CH + cg * 4) * g.PQ + pos;
#pragma unroll
                        for (int j = 0; j < 4; ++j) in[j] = *reinterpret_cast<const uint32_t *>(src + (int64_t)j * g.PQ);
                    }
                    transpose4x4(in, out);
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        *reinterpret_cast<uint32_t *>(&As[(pg * 4 + i) * ROWB + cg * 4]) = out[i];
                }
            }
        }
        // ---- stage B: packed weights of (occ, cc): [tap][64 oc][64 ch] -> rows of 80 bytes ----
        {
            const int8_t *src = wpk + ((int64_t)occ * CC + cc) * TAPS * CH * CH;
            for (int e = tid; e < TAPS * CH * 4; e += kThreads) {
                const int row = e >> 2, part = e & 3;
                const uint4 v = *reinterpret_cast<const uint4 *>(src + (int64_t)row * CH + part * 16);
                *reinterpret_cast<uint4 *>(&Bs[row * ROWB + part * 16]) = v;
            }
        }
        __syncthreads();
        // ---- MFMA: one K-step per tap ----
#pragma unroll
        for (int tap = 0; tap < TAPS; ++tap) {
            const int dr = (TAPS == 9) ? tap / 3 - 1 : 0, ds = (TAPS == 9) ? tap % 3 - 1 : 0;
            const int off = dr * g.W + ds;
            v4i bf[4];
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
                bf[nt] = *reinterpret_cast<const v4i *>(&Bs[(tap * CH + nt * 16 + l16) * ROWB + kb * 16]);
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
                v4i a = *reinterpret_cast<const v4i *>(&As[(row_base + mt * 16 + l16 + off) * ROWB + kb * 16]);
                if (TAPS == 9) {
                    bool ok = true;
                    if (dr < 0) ok = ok && ok_up[mt];
                    if (dr > 0) ok = ok && ok_dn[mt];
                    if (ds < 0) ok = ok && ok_lf[mt];
                    if (ds > 0) ok = ok && ok_rt[mt];
                    if (!ok) a = (v4i){(int)zavec, (int)zavec, (int)zavec, (int)zavec};
                }
                rsum[mt] = dot4_ones(a[0], dot4_ones(a[1], dot4_ones(a[2], dot4_ones(a[3], rsum[mt]))));
#pragma unroll
                for (int nt = 0; nt < 4; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, bf[nt], acc[mt][nt], 0, 0, 0);
            }
        }
    }

    // ---- row sums: fold the 4 k-blocks, hand them to the lanes that own the rows in the C layout ----
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
        int v = rsum[mt];
        v += __shfl_xor(v, 16, 64);
        v += __shfl_xor(v, 32, 64);
        if (kb == 0) rs[wave * 64 + mt * 16 + l16] = v;
    }
    __syncthreads();

    // zero-point correction in wrapping 32-bit arithmetic: the corrected value fits by contract
    const uint32_t Kp = (uint32_t)(g.C * TAPS);
    const uint32_t kzz = Kp * (uint32_t)za * (uint32_t)zb;
    const uint32_t uzb = (uint32_t)zb;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt) {
        const int lr = wave * 64 + mt * 16 + kb * 4;
        const int64_t gr = g0 + lr;
        if (gr >= g.M) continue;
        const int b = (int)(gr / g.PQ);
        const int pos = (int)(gr - (int64_t)b * g.PQ);
        const int4 r4 = *reinterpret_cast<const int4 *>(&rs[lr]);
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            const int oc = occ * CH + nt * 16 + l16;
            const uint32_t cs = (uint32_t)za * (uint32_t)colsum[oc];
            const int64_t o = ((int64_t)b * g.K + oc) * g.PQ + pos;
            const int c0 = (int)((uint32_t)acc[mt][nt][0] - uzb * (uint32_t)r4.x - cs + kzz);
            const int c1 = (int)((uint32_t)acc[mt][nt][1] - uzb * (uint32_t)r4.y - cs + kzz);
            const int c2 = (int)((uint32_t)acc[mt][nt][2] - uzb * (uint32_t)r4.z - cs + kzz);
            const int c3 = (int)((uint32_t)acc[mt][nt][3] - uzb * (uint32_t)r4.w - cs + kzz);
            if (acc_out) *reinterpret_cast<int4 *>(acc_out + o) = make_int4(c0, c1, c2, c3);
            if (y) {
                float4 f;
                f.x = sc * (float)c0;
                f.y = sc * (float)c1;
                f.z = sc * (float)c2;
                f.w = sc * (float)c3;
                *reinterpret_cast<float4 *>(y + o) = f;
            }
        }
    }
}

template <int TAPS>
constexpr size_t smem_bytes()
{
    return (size_t)(TAPS == 9 ? MAX_STAGE_ROWS : BM + 8) * ROWB + (size_t)TAPS * CH * ROWB + BM * sizeof(int);
}

bool shape_ok(int which, const q8t_conv_desc *d)
{
    if (which > 1) return false;
    if (d->stride != 1 || d->R != d->S) return false;
    if (!((d->R == 3 && d->pad == 1) || (d->R == 1 && d->pad == 0))) return false;
    if (d->C % CH || d->K % CH) return false;
    if ((d->H * d->W) % 4) return false;
    if (d->R == 3 && d->W > MAX_W) return false;
    if (d->H < 2 || d->W < 2) return false;
    return true;
}

}  // namespace

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
    return ((wbytes + 255) & ~(size_t)255) + (size_t)oc * sizeof(int);
}

int q8t_fast_conv(int which, const q8t_conv_desc *d, const void *a, const q8t_qparams *qa, const void *b,
                  const q8t_qparams *qb, float *out_f, void *out_acc, void *ws, hipStream_t st)
{
    if (!ws || !q8t_aligned(ws, 16)) return Q8T_ERR_WORKSPACE;
    const int taps = d->R * d->S;
    const size_t wbytes = (size_t)d->K * d->C * taps;
    int8_t *wpk = (int8_t *)ws;
    int *colsum = (int *)((char *)ws + ((wbytes + 255) & ~(size_t)255));
    FastGeom g;
    g.N = d->N;
    g.H = d->H;
    g.W = d->W;
    g.PQ = d->H * d->W;
    g.C = which == 0 ? d->C : d->K;   // reduction channels
    g.K = which == 0 ? d->K : d->C;   // output channels
    g.M = (int64_t)g.N * g.PQ;
    g.tiles = (int)((g.M + BM - 1) / BM);
    hipLaunchKernelGGL(repack_weights, dim3(g.K), dim3(kThreads), 0, st, (const int8_t *)b, d->K, d->C, d->R, d->S,
                       which, wpk, colsum);
    Q8T_LAUNCH_CHECK();
    const dim3 grid((unsigned)(((g.tiles + 7) / 8) * 8), (unsigned)(g.K / CH));
    if (taps == 9) {
        static bool attr9 = false;
        if (!attr9) {
            if (hipFuncSetAttribute((const void *)conv_s1_kernel<9>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)smem_bytes<9>()) != hipSuccess)
                return Q8T_ERR_HIP;
            attr9 = true;
        }
        hipLaunchKernelGGL(conv_s1_kernel<9>, grid, dim3(kThreads), smem_bytes<9>(), st, (const int8_t *)a, wpk,
                           colsum, qa, qb, g, out_f, (int32_t *)out_acc);
    } else {
        hipLaunchKernelGGL(conv_s1_kernel<1>, grid, dim3(kThreads), smem_bytes<1>(), st, (const int8_t *)a, wpk,
                           colsum, qa, qb, g, out_f, (int32_t *)out_acc);
    }
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}
