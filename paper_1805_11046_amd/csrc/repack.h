// Weight pre-pass of the specialised forward / layer-gradient kernels: the filter in the order their MFMA operands are
// read, plus the sum of every output channel's codes (the zero-point correction of Section 4's products).  The bodies
// live here so that one kernel can serve a single layer (conv_fast.hip, conv_wide.hip) or the filters of a whole
// network in one launch (repack_multi.hip).
#pragma once
#include "q8t_common.h"

constexpr int kRepackThreads = 256;

// 64-column register-tile kernel (conv_fast.hip):
// out[(oc/64)][cc][tap][oc%64][ch%64] = W'(oc, ch, tap);  forward: W'(oc,ch,r,s) = W[oc][ch][r][s];
// layer gradient: W'(oc,ch,r,s) = W[ch][oc][R-1-r][S-1-s]  (oc = input channel of the layer).
// One workgroup of kRepackThreads per output channel oc; red: kRepackThreads / 64 ints of LDS.
__device__ __forceinline__ void q8t_repack_tile64(const int8_t *__restrict__ w, int Kf, int Cf, int R, int S, int dgrad,
                                                  int8_t *__restrict__ out, int *__restrict__ colsum, int oc, int *red)
{
    constexpr int CH = 64;
    const int CHN = dgrad ? Kf : Cf;
    const int taps = R * S, CC = CHN / CH;
    int sum = 0;
    for (int e = threadIdx.x; e < taps * CHN; e += kRepackThreads) {
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
}

// Wide-tile kernel (conv_wide.hip), BN = 256 or 128 columns per workgroup: block (oc / BN, chunk, tap) of BN x 64 bytes =
// [32-column tile = oc % BN / 32 (a wavefront owns BN / 128 consecutive ones)][K half = ch % 64 / 32]
// [lane = (ch % 32 / 16) * 32 + oc % 32][16 bytes = ch % 16]: every MFMA operand of a wavefront is one 16-byte
// load per lane, 1 KB contiguous per instruction.  3x3 filters; W' as above; colsum[oc] = sum of W'(oc,.,.)
__device__ __forceinline__ void q8t_repack_wide(const int8_t *__restrict__ w, int Kf, int Cf, int dgrad, int BN,
                                                int8_t *__restrict__ out, int *__restrict__ colsum, int oc, int *red)
{
    constexpr int CH = 64;
    const int CHN = dgrad ? Kf : Cf;
    const int CC = CHN / CH;
    const int o256 = oc % BN;
    int sum = 0;
    // a thread gathers the 16 reduction channels of one (tap, 16-channel group) and writes them as one piece
    for (int e = threadIdx.x; e < 9 * (CHN / 16); e += kRepackThreads) {
        const int tap = e / (CHN / 16), c16 = e - tap * (CHN / 16);
        const int r = tap / 3, t = tap - r * 3;
        const int ch0 = c16 * 16, c64 = ch0 % CH;
        uint32_t pk[4] = {0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int ch = ch0 + i;
            int v;
            if (!dgrad)
                v = w[(((int64_t)oc * Cf + ch) * 3 + r) * 3 + t];
            else
                v = w[(((int64_t)ch * Cf + oc) * 3 + (2 - r)) * 3 + (2 - t)];
            sum += v;
            pk[i >> 2] |= (uint32_t)(v & 255) << (8 * (i & 3));
        }
        const int64_t blk = ((int64_t)(oc / BN) * CC + ch0 / CH) * 9 + tap;
        const int frag = (o256 / 32) * 2 + c64 / 32;   // (wavefront, column tile) = o256 / (BN / 4), (o256 % (BN / 4)) / 32 in one index
        *reinterpret_cast<uint4 *>(out + blk * (BN * CH) + frag * 1024 + (((c64 % 32) / 16) * 32 + oc % 32) * 16) =
            make_uint4(pk[0], pk[1], pk[2], pk[3]);
    }
    sum = wave_reduce(sum, [](int a, int b) { return a + b; });
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) colsum[oc] = red[0] + red[1] + red[2] + red[3];
}

// Filters packed ahead of the products (q8t_qconv_pack): which layout a (shape, product) pair takes
enum { Q8T_PACK_NONE = 0, Q8T_PACK_TILE64 = 1, Q8T_PACK_WIDE256 = 2, Q8T_PACK_WIDE128 = 3 };

// a packed filter: [codes, K*C*R*S bytes rounded up to 256][column sums, one int per output channel of the product]
inline size_t q8t_pack_colsum_offset(const q8t_conv_desc *d) { return ((size_t)d->K * d->C * d->R * d->S + 255) & ~(size_t)255; }
inline size_t q8t_pack_bytes(int which, const q8t_conv_desc *d)
{
    return q8t_pack_colsum_offset(d) + (((size_t)(which == 0 ? d->K : d->C) * sizeof(int) + 255) & ~(size_t)255);
}

struct Q8tPackJob {
    const int8_t *w;
    int8_t *out;
    int *colsum;
    int Kf, Cf, R, S;
    int dgrad, layout;   // layout: Q8T_PACK_*
    int first_block;     // its output channels are blocks first_block .. of the launch
};
constexpr int kPackMaxJobs = 48;
// one launch for all jobs (repack_multi.hip); jobs is a host array
int q8t_pack_launch(const Q8tPackJob *jobs, int n, hipStream_t st);
