// Specialised weight-gradient kernel for stride-1 3x3 (pad 1) convolutions:
//   dW[k,c,r,s] = sum_{n,p,q} g16[n,k,p,q] * x8[n,c,p+r-1,q+s-1]        (Section 4, eq. (grad_weight))
// with the 16-bit copy of the gradient (Sections 1, 7) and the 8-bit layer input, exact in integers.
//
// GEMM view: rows = output channel k, cols = (input channel c, tap), reduction = (image, position).
// Both operands are contiguous along the reduction in NCHW, so nothing is transposed.  The 16-bit
// operand is split into two signed bytes (s = 256*hi + lo + 128) and run as two int8 MFMA products.
//
// Padding without masks: inside LDS every image row is given a pitch of W+4 bytes; the 4 spare
// bytes hold the operand's zero point.  In that "padded-pitch" index space a tap is a pure byte
// offset ((r-1)*pitch + (s-1)), a pad column serves as right border of one row and left border
// of the next, and positions before/after the image are zero-point rows.  The gradient operand is
// staged with the same pitch (zero code in the pad columns), so pad positions contribute nothing.
// The three horizontal taps of a row come from one 24-byte aligned read, shifted with
// v_alignbyte.
//
// Work split: the output is tiny (K*C*9) and the reduction huge (N*H*W), so the reduction is split
// three ways: across workgroups (k-ranges of whole images), across the 4 wavefront pairs of a
// workgroup (interleaved 64-position K-steps, summed through LDS at the end) and in time.  A
// workgroup owns 64 rows x 16 channels x 9 taps x 2 byte planes = 72 MFMA tiles; wavefront
// (plane, lane-of-K) holds 36 of them.  Per-slice int32 partials (each slice is far below the
// 32-bit bound) are combined in int64 by wgrad_reduce, which also applies the zero-point
// correction from the row / column sums (columns with v_dot4 beside the MFMAs, rows with one more
// MFMA per row tile against an all-ones operand).
//
// The loop is bound by the number of instructions a wavefront issues (two wavefronts per SIMD
// reach about one vector instruction per 5-6 cycles, whatever its kind), not by the matrix pipe:
// everything that is not an MFMA is kept off the per-chunk path where it can be (scalar bases +
// per-thread constant offsets when the padded pitch divides the chunk, carried unit state).
#include <type_traits>

#include "q8t_common.h"
#include "q8t_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kThreads = 512;
constexpr int KC = 256;               // padded positions per staged chunk (4 K-steps of 64)
constexpr int APITCH = KC + 16;       // LDS bytes per gradient row and byte plane
constexpr int HALO = 72;              // staged halo on either side of the input chunk (>= pitch+1, mult. of 8)
constexpr int BROW = KC + 2 * HALO;   // staged input bytes per channel
constexpr int BPITCH = BROW + 4;      // 404 bytes = 101 dwords: at most 2-way bank conflicts for the
                                      // (16 channels x 4 k-blocks) dword reads of one wavefront
constexpr int A_BYTES = 2 * 64 * APITCH;
constexpr int B_BYTES = 16 * BPITCH;
constexpr int TILE_INTS = 2 * 4 * 9 * 4 * 64;          // [plane][mt][tap][j][lane]
constexpr int PART_INTS = TILE_INTS + 9 * 16 + 2 * 64; // + column sums [tap][ch] + row sums [plane][row]
constexpr int SLOT_INTS = 36 * 4 * 64 + 25 * 64;       // one wavefront's accumulators + its 9 + 16 sums
constexpr int BUF_BYTES = A_BYTES + B_BYTES;           // one staging buffer (two are used)
constexpr int SMEM_BYTES = 2 * BUF_BYTES > 2 * SLOT_INTS * 4 ? 2 * BUF_BYTES : 2 * SLOT_INTS * 4;

struct WGeom {
    int N, C, K, H, W, PQ;
    int pitch, Lp;        // padded row pitch, padded positions per image (H*pitch)
    float rpitch;         // 1/pitch
    int chunks;           // chunks per image
    int ncg, nrg;         // channel groups (C/16), row groups (K/64)
    int S, ipr;           // k-ranges, images per k-range
};

__device__ __forceinline__ int dot4_ones(int v, int acc) { return __builtin_amdgcn_sdot4(v, 0x01010101, acc, false); }

// WC > 0 fixes the image width at compile time (constant-divisor index arithmetic)
template <int WC>
__global__ __launch_bounds__(kThreads) void wgrad_s1_3x3(const int16_t *__restrict__ g16,
                                                          const int8_t *__restrict__ x,
                                                          const q8t_qparams *__restrict__ qpg,
                                                          const q8t_qparams *__restrict__ qpx, WGeom g,
                                                          int *__restrict__ partial)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    constexpr bool WIDE = WC > 0 && WC % 8 == 0;          // rows are 16-byte aligned: wide staging
    constexpr int PITCHC = WIDE ? WC + 8 : WC + 4;
    const int Wd = WC ? WC : g.W, pitch = WC ? PITCHC : g.pitch;

    // XCD-aware decode: workgroups that share a k-range (same gradient rows) sit on one XCD
    const int bid = blockIdx.x;
    const int xcd = bid & 7, jj = bid >> 3;
    const int per = g.ncg * g.nrg;
    const int sub = jj % per, kr = (jj / per) * 8 + xcd;
    if (kr >= g.S) return;
    const int cg = sub % g.ncg, rg = sub / g.ncg;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int plane = wave & 1, kl = wave >> 1;
    const int l16 = lane & 15, kb = lane >> 4;

    const int zsg = qpg->zero_point - (1 << (qpg->bits - 1)), zsx = qpx->zero_point - (1 << (qpx->bits - 1));
    const uint32_t a_pad = (uint32_t)(zsg & 0xFFFF) * 0x00010001u;   // two zero codes
    const uint32_t b_pad = (uint32_t)(zsx & 255) * 0x01010101u;

    const int img0 = kr * g.ipr, img1 = min(g.N, img0 + g.ipr);
    const int units = (img1 - img0) * g.chunks;

    v4i acc[4][9];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int t = 0; t < 9; ++t) acc[i][t] = (v4i){0, 0, 0, 0};
    int cs[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
    // Row sums of the gradient bytes: one more MFMA per row tile against an all-ones operand puts
    // them into accumulator layout (element j of lane (col, kb) = sum of row 4*kb + j, any col);
    // the matrix pipe has room for it, the vector ALU does not.
    v4i rs[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) rs[i] = (v4i){0, 0, 0, 0};
    const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};

    // staging registers: one chunk (64 gradient rows x 256 positions, 16 input channels x BROW)
    uint4 regA[4];
    uint2 regB[WIDE ? 2 : 4];
#pragma unroll
    for (int i = 0; i < 4; ++i) regA[i] = make_uint4(a_pad, a_pad, a_pad, a_pad);

    // When the padded pitch divides the chunk (pitch 64 or 32), a chunk is a whole number of image
    // rows: a thread's pieces keep their column and their row inside the chunk for the whole run,
    // and only the chunk's first image row (uniform) changes.  Global offsets then split into a
    // scalar base and a per-thread constant, and pad columns belong to the same lanes every time.
    constexpr bool SEP = WC > 0 && KC % PITCHC == 0;
    constexpr int RPC = SEP ? KC / PITCHC : 1;                    // image rows per chunk
    constexpr int PIECE = WIDE ? 8 : 4, NB = WIDE ? 2 : 4;
    constexpr int BPC = BROW / PIECE;                             // pieces per staged input channel
    constexpr int RB = SEP ? (HALO + PITCHC - 1) / PITCHC : 0;    // image rows covered by the halo
    constexpr int kNever = 1 << 24;                               // row offset of a lane that only ever stages padding
    int a_dp = kNever, b_dp[NB];
    uint32_t a_off = 0, b_off[NB];                                // byte offsets from the scalar bases
    if (SEP) {
        const int ta = PIECE * (WIDE ? (tid & 31) : lane), ra = ta / PITCHC, qa = ta - ra * PITCHC;
        if (qa < WC) a_dp = ra;
        a_off = (uint32_t)((WIDE ? (tid >> 5) * g.PQ : 0) + ra * WC + qa) * 2u;
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int e = tid + kThreads * i, c = e / BPC, pi = e - c * BPC;
            const int t = PIECE * pi - HALO + RB * PITCHC, rb = t / PITCHC, qb = t - rb * PITCHC;
            b_dp[i] = (e < 16 * BPC && qb < WC) ? rb - RB : kNever;
            b_off[i] = (uint32_t)(c * g.PQ + rb * WC + qb);
        }
    }
    // position / pitch: quotients are image rows (< 2^15), a float estimate with fix-up is exact
    auto pdiv = [&](uint32_t n) -> uint32_t {
        if (WC) return n / (uint32_t)(WC ? PITCHC : 1);
        uint32_t q = (uint32_t)((float)n * g.rpitch);
        const int rem = (int)(n - q * (uint32_t)pitch);
        if (rem < 0) --q;
        else if (rem >= pitch) ++q;
        return q;
    };

    // Units are staged in order, so the (image, chunk) of the next one and its scalar base
    // addresses are carried along instead of being derived from the unit index.
    int l_b = img0, l_ck = 0;
    const char *l_ga = reinterpret_cast<const char *>(g16 + ((int64_t)img0 * g.K + rg * 64) * g.PQ);
    // the input offsets are counted from RB image rows above the chunk (never dereferenced there)
    const char *l_xb = reinterpret_cast<const char *>(x) + ((int64_t)img0 * g.C + cg * 16) * g.PQ - RB * WC;
    const int64_t wrap_ga = ((int64_t)g.K * g.PQ - (int64_t)g.chunks * RPC * WC) * 2;
    const int64_t wrap_xb = (int64_t)g.C * g.PQ - (int64_t)g.chunks * RPC * WC;
    auto load_regs = [&]() {
        const int b = l_b, kp0 = l_ck * KC;
        if (SEP) {
            const int P0 = l_ck * RPC;
            const char *ga = l_ga, *xb = l_xb;
            if ((uint32_t)(P0 + a_dp) < (uint32_t)g.H) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (WIDE) {
                        regA[i] = *reinterpret_cast<const uint4 *>(ga + (int64_t)i * 32 * g.PQ + a_off);
                    } else {
                        const uint2 v0 = *reinterpret_cast<const uint2 *>(ga + (int64_t)(wave + 16 * i) * 2 * g.PQ + a_off);
                        const uint2 v1 = *reinterpret_cast<const uint2 *>(ga + (int64_t)(wave + 16 * i + 8) * 2 * g.PQ + a_off);
                        regA[i] = make_uint4(v0.x, v0.y, v1.x, v1.y);
                    }
                }
            } else if (a_dp != kNever) {   // rows past the image in a ragged last chunk
#pragma unroll
                for (int i = 0; i < 4; ++i) regA[i] = make_uint4(a_pad, a_pad, a_pad, a_pad);
            }
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                const bool ld = (uint32_t)(P0 + b_dp[i]) < (uint32_t)g.H;
                regB[i] = make_uint2(b_pad, b_pad);
                if (WIDE) {
                    if (ld) regB[i] = *reinterpret_cast<const uint2 *>(xb + b_off[i]);
                } else {
                    if (ld) regB[i].x = *reinterpret_cast<const uint32_t *>(xb + b_off[i]);
                }
            }
        } else if (WIDE) {
            // pieces of 8 positions: 16-byte gradient loads, 8-byte input loads (the vector memory
            // pipeline is paid per instruction, not per byte)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = tid + kThreads * i, row = e >> 5, pi = e & 31;
                const int kp = kp0 + 8 * pi;
                const int p = (int)pdiv((uint32_t)kp), qq = kp - p * pitch;
                regA[i] = make_uint4(a_pad, a_pad, a_pad, a_pad);
                if (kp < g.Lp && qq < Wd)
                    regA[i] = *reinterpret_cast<const uint4 *>(g16 + ((int64_t)b * g.K + rg * 64 + row) * g.PQ + p * Wd + qq);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int e = tid + kThreads * i, c = e / (BROW / 8), pi = e - c * (BROW / 8);
                const int kp = kp0 - HALO + 8 * pi;
                bool valid = e < 16 * (BROW / 8) && kp >= 0 && kp < g.Lp;
                const int kpc = valid ? kp : 0;
                const int p = (int)pdiv((uint32_t)kpc), qq = kpc - p * pitch;
                valid = valid && qq < Wd;
                regB[i] = make_uint2(b_pad, b_pad);
                if (valid)
                    regB[i] = *reinterpret_cast<const uint2 *>(x + ((int64_t)b * g.C + cg * 16 + c) * g.PQ + p * Wd + qq);
            }
        } else {
            // pieces of 4 positions; wavefront w stages gradient rows w, w+8, ..., lane = piece
            const int kp = kp0 + 4 * lane;
            const int p = (int)pdiv((uint32_t)kp), qq = kp - p * pitch;
            const bool valid = kp < g.Lp && qq < Wd;
            const int16_t *src = g16 + ((int64_t)b * g.K + rg * 64 + wave) * g.PQ + p * Wd + qq;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint2 v0 = make_uint2(a_pad, a_pad), v1 = v0;
                if (valid) {
                    v0 = *reinterpret_cast<const uint2 *>(src + (int64_t)(2 * i) * 8 * g.PQ);
                    v1 = *reinterpret_cast<const uint2 *>(src + (int64_t)(2 * i + 1) * 8 * g.PQ);
                }
                regA[i] = make_uint4(v0.x, v0.y, v1.x, v1.y);   // rows wave+16i and wave+16i+8
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = tid + kThreads * i, c = e / (BROW / 4), gi = e - c * (BROW / 4);
                const int kp = kp0 - HALO + 4 * gi;
                bool valid = e < 16 * (BROW / 4) && kp >= 0 && kp < g.Lp;
                const int kpc = valid ? kp : 0;
                const int p = (int)pdiv((uint32_t)kpc), qq = kpc - p * pitch;
                valid = valid && qq < Wd;
                regB[i].x = b_pad;
                if (valid)
                    regB[i].x = *reinterpret_cast<const uint32_t *>(x + ((int64_t)b * g.C + cg * 16 + c) * g.PQ + p * Wd + qq);
            }
        }
        if (++l_ck == g.chunks) {
            l_ck = 0;
            ++l_b;
            l_ga += wrap_ga;
            l_xb += wrap_xb;
        }
        l_ga += RPC * WC * 2;
        l_xb += RPC * WC;
    };
    auto write_lds = [&](int buf) {
        uint8_t *A = smem + buf * BUF_BYTES, *B = A + A_BYTES;
        if (WIDE) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = tid + kThreads * i, row = e >> 5, pi = e & 31;
                const uint32_t h0 = __builtin_amdgcn_perm(regA[i].y, regA[i].x, 0x07050301);
                const uint32_t h1 = __builtin_amdgcn_perm(regA[i].w, regA[i].z, 0x07050301);
                const uint32_t l0 = __builtin_amdgcn_perm(regA[i].y, regA[i].x, 0x06040200) ^ 0x80808080u;
                const uint32_t l1 = __builtin_amdgcn_perm(regA[i].w, regA[i].z, 0x06040200) ^ 0x80808080u;
                *reinterpret_cast<uint2 *>(&A[row * APITCH + 8 * pi]) = make_uint2(h0, h1);
                *reinterpret_cast<uint2 *>(&A[(64 + row) * APITCH + 8 * pi]) = make_uint2(l0, l1);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int e = tid + kThreads * i, c = e / (BROW / 8), pi = e - c * (BROW / 8);
                if (e < 16 * (BROW / 8)) *reinterpret_cast<uint2 *>(&B[c * BPITCH + 8 * pi]) = regB[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int hsel = 0; hsel < 2; ++hsel) {
                    const int row = wave + 16 * i + 8 * hsel;
                    const uint32_t lo32 = hsel ? regA[i].z : regA[i].x, hi32 = hsel ? regA[i].w : regA[i].y;
                    const uint32_t hi = __builtin_amdgcn_perm(hi32, lo32, 0x07050301);
                    const uint32_t lo = __builtin_amdgcn_perm(hi32, lo32, 0x06040200) ^ 0x80808080u;
                    *reinterpret_cast<uint32_t *>(&A[row * APITCH + 4 * lane]) = hi;
                    *reinterpret_cast<uint32_t *>(&A[(64 + row) * APITCH + 4 * lane]) = lo;
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = tid + kThreads * i, c = e / (BROW / 4), gi = e - c * (BROW / 4);
                if (e < 16 * (BROW / 4)) *reinterpret_cast<uint32_t *>(&B[c * BPITCH + 4 * gi]) = regB[i].x;
            }
        }
    };
    int c_ck = 0;   // chunk (within its image) of the next unit to be multiplied
    auto compute = [&](int buf) {
        const uint8_t *A = smem + buf * BUF_BYTES, *B = A + A_BYTES;
        const int kstart = c_ck * KC + kl * 64;
        if (++c_ck == g.chunks) c_ck = 0;
        if (kstart >= g.Lp) return;   // wavefront-uniform: ragged last chunk of an image
        v4i a[4];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
            a[mt] = *reinterpret_cast<const v4i *>(&A[(plane * 64 + mt * 16 + l16) * APITCH + kl * 64 + kb * 16]);
            rs[mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[mt], ones, rs[mt], 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const int base = HALO + kl * 64 + kb * 16 + (r - 1) * pitch - 4;
            uint32_t d[6];
#pragma unroll
            for (int i = 0; i < 6; ++i) d[i] = *reinterpret_cast<const uint32_t *>(&B[l16 * BPITCH + base + 4 * i]);
            v4i f[3];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                f[0][i] = (int)__builtin_amdgcn_alignbyte(d[i + 1], d[i], 3);
                f[1][i] = (int)d[i + 1];
                f[2][i] = (int)__builtin_amdgcn_alignbyte(d[i + 2], d[i + 1], 1);
            }
#pragma unroll
            for (int s = 0; s < 3; ++s) {
                const int tap = r * 3 + s;
                if ((tap < 5) == (plane == 0)) {   // wavefront-uniform: the two planes share the column sums
                    asm volatile("" ::: "memory");  // keep this a scalar branch (no compute-both-and-select)
                    cs[tap] = dot4_ones(f[s][0], dot4_ones(f[s][1], dot4_ones(f[s][2], dot4_ones(f[s][3], cs[tap]))));
                }
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
                    acc[mt][tap] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[mt], f[s], acc[mt][tap], 0, 0, 0);
            }
        }
    };

    // Double-buffered LDS, one barrier per chunk.  The two wavefronts that share a SIMD run the
    // phases of an iteration in opposite order (MFMA first / staging first), so that one issues
    // matrix instructions while the other occupies the vector-memory and LDS pipes.
    const bool late = wave >= 4;
    if (units > 0) {
        load_regs();
        write_lds(0);
        if (units > 1) load_regs();
    }
    __syncthreads();
    for (int u = 0; u < units; ++u) {
        const int cur = u & 1;
        if (!late) compute(cur);
        if (u + 1 < units) {
            write_lds(cur ^ 1);
            if (u + 2 < units) load_regs();
        }
        if (late) compute(cur);
        q8t_lds_barrier();
    }

    // fold the 4 k-blocks of the column sums
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        cs[t] += __shfl_xor(cs[t], 16, 64);
        cs[t] += __shfl_xor(cs[t], 32, 64);
    }

    // ---- sum the 4 K-lanes of each plane through LDS: (1 -> 0), (3 -> 2), then (2 -> 0) ----
    int *slots = reinterpret_cast<int *>(smem);
    for (int round = 0; round < 3; ++round) {
        const int src = round == 0 ? 1 : (round == 1 ? 3 : 2);
        const int dst = round == 0 ? 0 : (round == 1 ? 2 : 0);
        int *slot = slots + plane * SLOT_INTS;
        q8t_lds_barrier();
        if (kl == src) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int t = 0; t < 9; ++t)
#pragma unroll
                    for (int j = 0; j < 4; ++j) slot[((mt * 9 + t) * 4 + j) * 64 + lane] = acc[mt][t][j];
#pragma unroll
            for (int t = 0; t < 9; ++t) slot[36 * 4 * 64 + t * 64 + lane] = cs[t];
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int j = 0; j < 4; ++j) slot[36 * 4 * 64 + (9 + mt * 4 + j) * 64 + lane] = rs[mt][j];
        }
        q8t_lds_barrier();
        if (kl == dst) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int t = 0; t < 9; ++t)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[mt][t][j] += slot[((mt * 9 + t) * 4 + j) * 64 + lane];
#pragma unroll
            for (int t = 0; t < 9; ++t) cs[t] += slot[36 * 4 * 64 + t * 64 + lane];
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int j = 0; j < 4; ++j) rs[mt][j] += slot[36 * 4 * 64 + (9 + mt * 4 + j) * 64 + lane];
        }
    }

    // ---- K-lane 0 of each plane writes the workgroup's partial, in register-tile order ----
    if (kl == 0) {
        int *out = partial + ((int64_t)(kr * g.nrg + rg) * g.ncg + cg) * PART_INTS;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int t = 0; t < 9; ++t)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    out[(((plane * 4 + mt) * 9 + t) * 4 + j) * 64 + lane] = acc[mt][t][j];
        if (kb == 0) {
#pragma unroll
            for (int t = 0; t < 9; ++t)
                if ((t < 5) == (plane == 0)) out[TILE_INTS + t * 16 + l16] = cs[t];
        }
        if (l16 == 0) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int j = 0; j < 4; ++j) out[TILE_INTS + 144 + plane * 64 + mt * 16 + kb * 4 + j] = rs[mt][j];
        }
    }
}

// int64 reduction over the k-ranges + zero-point correction + dequantization.
// Workgroup = 64 accumulator slots x 4 quarters of the k-ranges, folded through LDS.
__global__ __launch_bounds__(256) void wgrad_reduce(const int *__restrict__ partial, WGeom g,
                                                    const q8t_qparams *__restrict__ qpg,
                                                    const q8t_qparams *__restrict__ qpx, float *__restrict__ dw,
                                                    int64_t *__restrict__ acc_out)
{
    __shared__ int64_t fold[4][64];
    const int sub = blockIdx.y;               // (rg, cg)
    const int cg = sub % g.ncg, rg = sub / g.ncg;
    const int lane = threadIdx.x & 63, quarter = threadIdx.x >> 6;
    const int idx = blockIdx.x * 64 + lane;   // ((mt*9 + tap)*4 + j)*64 + lane, < 9216
    const int j = (idx >> 6) & 3, mt_tap = idx >> 8;
    const int tap = mt_tap % 9, mt = mt_tap / 9;
    const int row_l = mt * 16 + (lane >> 4) * 4 + j, ch_l = lane & 15;

    const int zsg = qpg->zero_point - (1 << (qpg->bits - 1)), zsx = qpx->zero_point - (1 << (qpx->bits - 1));
    const int64_t ca = 128 - zsg;
    const int ksteps_img = (g.Lp + 63) / 64;
    int64_t v = 0;
    for (int kr = quarter; kr < g.S; kr += 4) {
        const int *p = partial + ((int64_t)(kr * g.nrg + rg) * g.ncg + cg) * PART_INTS;
        const int nimg = min(g.N, (kr + 1) * g.ipr) - kr * g.ipr;
        const int64_t Kp = (int64_t)nimg * ksteps_img * 64;
        const int64_t hi = p[idx], lo = p[TILE_INTS / 2 + idx];
        const int64_t csv = p[TILE_INTS + tap * 16 + ch_l];
        const int64_t rsh = p[TILE_INTS + 144 + row_l], rsl = p[TILE_INTS + 144 + 64 + row_l];
        v += 256 * hi + lo + ca * csv - (int64_t)zsx * (256 * rsh + rsl + ca * Kp);
    }
    fold[quarter][lane] = v;
    __syncthreads();
    if (quarter == 0) {
        v = fold[0][lane] + fold[1][lane] + fold[2][lane] + fold[3][lane];
        const double sc = (double)(qpg->scale * qpx->scale);
        const int64_t o = ((int64_t)(rg * 64 + row_l) * g.C + cg * 16 + ch_l) * 9 + tap;
        if (acc_out) acc_out[o] = v;
        if (dw) dw[o] = (float)((double)v * sc);
    }
}

// ---------------------------------------------------------------------------------------------
// Second form of the same product for the widths whose padded pitch divides the chunk (56 -> 64,
// 28 -> 32).  The horizontal tap moves to the gradient operand: with p' = p + (s-1),
//   dW[k,c,r,s] = sum_p' g[k, p' - (s-1)] * x[c, p' + (r-1)*pitch],
// so the input fragments are plain 16-byte aligned LDS reads and only the gradient fragment of a
// wavefront is shifted (8 v_alignbyte per K-step).  A wavefront owns 16 gradient rows x 32 input
// channels x 9 taps of one byte plane and walks all four K-steps of a chunk itself: there is no
// split of the reduction inside the workgroup, so the per-chunk cost of staging, barrier and loop
// is paid once per 72 MFMAs instead of once per 36, and nothing is folded through LDS at the end.
// Row sums (one per shift) and column sums (one per vertical tap) come from MFMAs against an
// all-ones operand; the six column sums (2 channel tiles x 3 vertical taps) are dealt out to six
// wavefronts, one extra fragment read and MFMA per K-step each.
// Terms whose shifted position falls outside the processed range pair a padding column of x
// (zero-point code) with a gradient: they are zero in real arithmetic and are left out of the
// products and of all three sums alike, so the integer identity of wgrad_reduce_v2 stays exact.
constexpr int A_LEFT = 16;                       // bytes before the chunk in a gradient row: padding columns, set once
// Row pitches of 8, 24, 40 or 56 dwords (mod 64) make the 16-byte fragment reads of a wavefront
// (16 rows x 4 neighbouring 16-byte columns) conflict-free under the 4-phase service order of
// ds_read_b128.
constexpr int APITCH2 = A_LEFT + KC + 16;        // 288 B = 72 dwords; holds the 8 positions after the chunk as well
constexpr int HALO2 = 64;
constexpr int BROW2 = KC + 2 * HALO2;
constexpr int BPITCH2 = BROW2 + 32;              // 416 B = 104 dwords
constexpr int CH2 = 32;                          // input channels per workgroup
constexpr int A2_BYTES = 2 * 64 * APITCH2;
constexpr int BUF2_BYTES = A2_BYTES + CH2 * BPITCH2;
constexpr int SMEM2_BYTES = 2 * BUF2_BYTES;
constexpr int TILE2_INTS = 2 * 4 * 2 * 9 * 4 * 64;              // [plane][mt][ct][tap][j][lane]
constexpr int PART2_INTS = TILE2_INTS + 3 * CH2 + 2 * 3 * 64;   // + column sums [r][ch] + row sums [plane][s][row]

template <int WC>
__global__ __launch_bounds__(kThreads) void wgrad_s1_3x3_v2(const int16_t *__restrict__ g16,
                                                             const int8_t *__restrict__ x,
                                                             const q8t_qparams *__restrict__ qpg,
                                                             const q8t_qparams *__restrict__ qpx, WGeom g,
                                                             int *__restrict__ partial)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    constexpr bool WIDE = WC % 8 == 0;
    constexpr int PITCHC = WIDE ? WC + 8 : WC + 4;
    static_assert(KC % PITCHC == 0 && HALO2 % PITCHC == 0, "the pitch must divide the chunk and the halo");
    constexpr int RPC = KC / PITCHC, RB = HALO2 / PITCHC;   // image rows per chunk / per halo
    constexpr int PIECE = WIDE ? 8 : 4;                     // positions per staged piece
    constexpr int APR = KC / PIECE;                         // gradient pieces per row
    constexpr int NA = 64 * APR / kThreads;                 // gradient pieces per thread (4 or 8)
    constexpr int ROWSTEP = kThreads / APR;                 // rows between a thread's pieces
    constexpr int BPC = BROW2 / PIECE;                      // input pieces per channel
    constexpr int NB = CH2 * BPC / kThreads;                // input pieces per thread (3 or 6)
    constexpr int kNever = 1 << 24;

    const int bid = blockIdx.x;
    const int xcd = bid & 7, jj = bid >> 3;
    const int per = g.ncg * g.nrg;
    const int sub = jj % per, kr = (jj / per) * 8 + xcd;
    if (kr >= g.S) return;
    const int cg = sub % g.ncg, rg = sub / g.ncg;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int plane = wave & 1, mt = wave >> 1;
    const int l16 = lane & 15, kb = lane >> 4;
    const int csq = wave < 6 ? wave : wave - 6;   // (channel tile, vertical tap) whose column sums this wavefront gathers
    const int cs_ct = csq / 3, cs_r = csq - 3 * cs_ct;

    const int zsg = qpg->zero_point - (1 << (qpg->bits - 1)), zsx = qpx->zero_point - (1 << (qpx->bits - 1));
    const uint32_t a_pad = (uint32_t)(zsg & 0xFFFF) * 0x00010001u;
    const uint32_t b_pad = (uint32_t)(zsx & 255) * 0x01010101u;

    const int img0 = kr * g.ipr, img1 = min(g.N, img0 + g.ipr);
    const int units = (img1 - img0) * g.chunks;

    v4i acc[2][9], rs[3], csacc = {0, 0, 0, 0};
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int t = 0; t < 9; ++t) acc[c][t] = (v4i){0, 0, 0, 0};
#pragma unroll
    for (int t = 0; t < 3; ++t) rs[t] = (v4i){0, 0, 0, 0};
    const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};

    // the bytes before the chunk in every gradient row are padding columns: zero code, set once
    {
        const uint32_t hi4 = (uint32_t)((zsg >> 8) & 255) * 0x01010101u;
        const uint32_t lo4 = (uint32_t)((zsg & 255) ^ 0x80) * 0x01010101u;
        const int buf = tid >> 8, prow = (tid >> 1) & 127, half = tid & 1;
        const uint32_t v = prow < 64 ? hi4 : lo4;
        *reinterpret_cast<uint2 *>(&smem[buf * BUF2_BYTES + prow * APITCH2 + 8 * half]) = make_uint2(v, v);
    }

    // per-thread constants of the staging: row inside the chunk, column, global byte offset
    using AReg = typename std::conditional<WIDE, uint4, uint2>::type;
    AReg regA[NA], regH;
    uint2 regB[NB];
    const int pa = tid % APR, ta = PIECE * pa, ra = ta / PITCHC, qa = ta - ra * PITCHC;
    const int a_dp = qa < WC ? ra : kNever;
    const uint32_t a_off = (uint32_t)((tid / APR) * g.PQ + ra * WC + qa) * 2u;
    const uint32_t h_off = (uint32_t)(tid * g.PQ + RPC * WC) * 2u;          // threads 0..63: the piece after the chunk
    int b_dp[NB];
    uint32_t b_off[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int e = tid + kThreads * i, c = e / BPC, pi = e - c * BPC;
        const int t = PIECE * pi, rb = t / PITCHC, qb = t - rb * PITCHC;
        b_dp[i] = qb < WC ? rb - RB : kNever;
        b_off[i] = (uint32_t)(c * g.PQ + rb * WC + qb);
    }
    auto pad_a = [&]() {
        AReg v;
        if constexpr (WIDE) v = make_uint4(a_pad, a_pad, a_pad, a_pad);
        else v = make_uint2(a_pad, a_pad);
        return v;
    };
#pragma unroll
    for (int i = 0; i < NA; ++i) regA[i] = pad_a();
    regH = pad_a();

    int l_ck = 0;
    const char *l_ga = reinterpret_cast<const char *>(g16 + ((int64_t)img0 * g.K + rg * 64) * g.PQ);
    const char *l_xb = reinterpret_cast<const char *>(x) + ((int64_t)img0 * g.C + cg * CH2) * g.PQ - RB * WC;
    const int64_t wrap_ga = ((int64_t)g.K * g.PQ - (int64_t)g.chunks * RPC * WC) * 2;
    const int64_t wrap_xb = (int64_t)g.C * g.PQ - (int64_t)g.chunks * RPC * WC;
    auto load_regs = [&]() {
        const int P0 = l_ck * RPC;
        const char *ga = l_ga, *xb = l_xb;
        if ((uint32_t)(P0 + a_dp) < (uint32_t)g.H) {
#pragma unroll
            for (int i = 0; i < NA; ++i)
                regA[i] = *reinterpret_cast<const AReg *>(ga + (int64_t)i * ROWSTEP * 2 * g.PQ + a_off);
        } else if (a_dp != kNever) {   // rows past the image in a ragged last chunk
#pragma unroll
            for (int i = 0; i < NA; ++i) regA[i] = pad_a();
        }
        if (wave == 0) {               // first positions of the image row after the chunk
            if (P0 + RPC < g.H) regH = *reinterpret_cast<const AReg *>(ga + h_off);
            else regH = pad_a();
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const bool ld = (uint32_t)(P0 + b_dp[i]) < (uint32_t)g.H;
            regB[i] = make_uint2(b_pad, b_pad);
            if (WIDE) {
                if (ld) regB[i] = *reinterpret_cast<const uint2 *>(xb + b_off[i]);
            } else {
                if (ld) regB[i].x = *reinterpret_cast<const uint32_t *>(xb + b_off[i]);
            }
        }
        if (++l_ck == g.chunks) {
            l_ck = 0;
            l_ga += wrap_ga;
            l_xb += wrap_xb;
        }
        l_ga += RPC * WC * 2;
        l_xb += RPC * WC;
    };
    auto split_store = [&](uint8_t *A, int row, int col, const AReg &v) {
        if constexpr (WIDE) {
            const uint32_t h0 = __builtin_amdgcn_perm(v.y, v.x, 0x07050301), h1 = __builtin_amdgcn_perm(v.w, v.z, 0x07050301);
            const uint32_t l0 = __builtin_amdgcn_perm(v.y, v.x, 0x06040200) ^ 0x80808080u;
            const uint32_t l1 = __builtin_amdgcn_perm(v.w, v.z, 0x06040200) ^ 0x80808080u;
            *reinterpret_cast<uint2 *>(&A[row * APITCH2 + A_LEFT + col]) = make_uint2(h0, h1);
            *reinterpret_cast<uint2 *>(&A[(64 + row) * APITCH2 + A_LEFT + col]) = make_uint2(l0, l1);
        } else {
            const uint32_t h = __builtin_amdgcn_perm(v.y, v.x, 0x07050301);
            const uint32_t l = __builtin_amdgcn_perm(v.y, v.x, 0x06040200) ^ 0x80808080u;
            *reinterpret_cast<uint32_t *>(&A[row * APITCH2 + A_LEFT + col]) = h;
            *reinterpret_cast<uint32_t *>(&A[(64 + row) * APITCH2 + A_LEFT + col]) = l;
        }
    };
    auto write_lds = [&](int buf) {
        uint8_t *A = smem + buf * BUF2_BYTES, *B = A + A2_BYTES;
#pragma unroll
        for (int i = 0; i < NA; ++i) split_store(A, tid / APR + ROWSTEP * i, PIECE * pa, regA[i]);
        if (wave == 0) split_store(A, tid, KC, regH);
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int e = tid + kThreads * i, c = e / BPC, pi = e - c * BPC;
            if (WIDE) *reinterpret_cast<uint2 *>(&B[c * BPITCH2 + 8 * pi]) = regB[i];
            else *reinterpret_cast<uint32_t *>(&B[c * BPITCH2 + 4 * pi]) = regB[i].x;
        }
    };
    int c_ck = 0;
    auto compute = [&](int buf) {
        const uint8_t *A = smem + buf * BUF2_BYTES, *B = A + A2_BYTES;
        const int k0 = c_ck * KC;
        if (++c_ck == g.chunks) c_ck = 0;
        const uint8_t *Ar = A + (plane * 64 + mt * 16 + l16) * APITCH2 + A_LEFT + kb * 16;
        const uint8_t *Br = B + l16 * BPITCH2 + HALO2 + kb * 16;
        const uint8_t *Bcs = Br + cs_ct * 16 * BPITCH2 + (cs_r - 1) * PITCHC;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (k0 + ks * 64 >= g.Lp) break;   // uniform: ragged last chunk of an image
            const v4i c = *reinterpret_cast<const v4i *>(Ar + ks * 64);
            const uint32_t dm1 = *reinterpret_cast<const uint32_t *>(Ar + ks * 64 - 4);
            const uint32_t dp1 = *reinterpret_cast<const uint32_t *>(Ar + ks * 64 + 16);
            auto ab = [](int hi, int lo, int n) { return (int)__builtin_amdgcn_alignbyte((uint32_t)hi, (uint32_t)lo, n); };
            v4i fa[3];
            fa[0] = (v4i){ab(c[1], c[0], 1), ab(c[2], c[1], 1), ab(c[3], c[2], 1), ab((int)dp1, c[3], 1)};   // g[p' + 1]
            fa[1] = c;
            fa[2] = (v4i){ab(c[0], (int)dm1, 3), ab(c[1], c[0], 3), ab(c[2], c[1], 3), ab(c[3], c[2], 3)};   // g[p' - 1]
#pragma unroll
            for (int s = 0; s < 3; ++s) rs[s] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[s], ones, rs[s], 0, 0, 0);
            csacc = __builtin_amdgcn_mfma_i32_16x16x64_i8(ones, *reinterpret_cast<const v4i *>(Bcs + ks * 64), csacc, 0, 0, 0);
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                for (int r = 0; r < 3; ++r) {
                    const v4i fb = *reinterpret_cast<const v4i *>(Br + ct * 16 * BPITCH2 + ks * 64 + (r - 1) * PITCHC);
#pragma unroll
                    for (int s = 0; s < 3; ++s)
                        acc[ct][r * 3 + s] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[s], fb, acc[ct][r * 3 + s], 0, 0, 0);
                }
        }
    };

    const bool late = wave >= 4;
    if (units > 0) {
        load_regs();
        write_lds(0);
        if (units > 1) load_regs();
    }
    __syncthreads();
    for (int u = 0; u < units; ++u) {
        const int cur = u & 1;
        if (!late) compute(cur);
        if (u + 1 < units) {
            write_lds(cur ^ 1);
            if (u + 2 < units) load_regs();
        }
        if (late) compute(cur);
        q8t_lds_barrier();
    }

    int *out = partial + ((int64_t)(kr * g.nrg + rg) * g.ncg + cg) * PART2_INTS;
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                out[((((plane * 4 + mt) * 2 + ct) * 9 + t) * 4 + j) * 64 + lane] = acc[ct][t][j];
    if (wave < 6 && kb == 0) out[TILE2_INTS + cs_r * CH2 + cs_ct * 16 + l16] = csacc[0];
    if (l16 == 0) {
#pragma unroll
        for (int s = 0; s < 3; ++s)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                out[TILE2_INTS + 3 * CH2 + (plane * 3 + s) * 64 + mt * 16 + kb * 4 + j] = rs[s][j];
    }
}

// int64 reduction over the k-ranges for wgrad_s1_3x3_v2: the column sum depends on the vertical tap,
// the row sums on the horizontal one.
// A thread owns four neighbouring accumulator entries (four input channels of one output channel and tap) and walks
// its share of the ranges with 16-byte loads; the wavefronts of a workgroup take interleaved subsets of the ranges
// and fold through LDS.
constexpr int RQ2 = 16;   // most interleaved subsets of the k-ranges per workgroup (one wavefront each)
__global__ __launch_bounds__(64 * RQ2) void wgrad_reduce_v2(const int *__restrict__ partial, WGeom g,
                                                       const q8t_qparams *__restrict__ qpg,
                                                       const q8t_qparams *__restrict__ qpx, float *__restrict__ dw,
                                                       int64_t *__restrict__ acc_out)
{
    __shared__ int64_t fold[RQ2][4][64];
    const int sub = blockIdx.y;
    const int cg = sub % g.ncg, rg = sub / g.ncg;
    const int ln = threadIdx.x & 63, quarter = threadIdx.x >> 6, nq = blockDim.x >> 6;
    const int idx = (blockIdx.x * 64 + ln) * 4;   // (((mt*2 + ct)*9 + tap)*4 + j)*64 + lane, < 9216 (a multiple of 256)
    const int lane = idx & 63, j = (idx >> 6) & 3, t2 = idx >> 8;
    const int tap = t2 % 9, ct = (t2 / 9) & 1, mt = t2 / 18;
    const int r = tap / 3, s = tap - 3 * r;
    const int row_l = mt * 16 + (lane >> 4) * 4 + j, ch_l = ct * 16 + (lane & 15);

    const int zsg = qpg->zero_point - (1 << (qpg->bits - 1)), zsx = qpx->zero_point - (1 << (qpx->bits - 1));
    const int64_t ca = 128 - zsg;
    const int ksteps_img = (g.Lp + 63) / 64;
    int64_t v[4] = {0, 0, 0, 0};
#pragma unroll 4
    for (int kr = quarter; kr < g.S; kr += nq) {
        const int *p = partial + ((int64_t)(kr * g.nrg + rg) * g.ncg + cg) * PART2_INTS;
        const int nimg = min(g.N, (kr + 1) * g.ipr) - kr * g.ipr;
        const int64_t Kp = (int64_t)nimg * ksteps_img * 64;
        const v4i hi = *reinterpret_cast<const v4i *>(p + idx), lo = *reinterpret_cast<const v4i *>(p + TILE2_INTS / 2 + idx);
        const v4i csv = *reinterpret_cast<const v4i *>(p + TILE2_INTS + r * CH2 + ch_l);
        const int64_t rsh = p[TILE2_INTS + 3 * CH2 + s * 64 + row_l], rsl = p[TILE2_INTS + 3 * CH2 + (3 + s) * 64 + row_l];
        const int64_t common = (int64_t)zsx * (256 * rsh + rsl + ca * Kp);
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] += 256 * (int64_t)hi[e] + (int64_t)lo[e] + ca * (int64_t)csv[e] - common;
    }
    if (nq > 1) {
#pragma unroll
        for (int e = 0; e < 4; ++e) fold[quarter][e][ln] = v[e];
        __syncthreads();
        if (quarter != 0) return;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[e] = 0;
            for (int q = 0; q < nq; ++q) v[e] += fold[q][e][ln];
        }
    }
    const double sc = (double)(qpg->scale * qpx->scale);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int64_t o = ((int64_t)(rg * 64 + row_l) * g.C + cg * CH2 + ch_l + e) * 9 + tap;
        if (acc_out) acc_out[o] = v[e];
        if (dw) dw[o] = (float)((double)v[e] * sc);
    }
}

bool wgrad_shape_ok(const q8t_conv_desc *d)
{
    if (d->stride != 1 || d->R != 3 || d->S != 3 || d->pad != 1) return false;
    if (d->K % 64 || d->C % 16 || d->W % 4) return false;
    if (d->W + 8 + 1 > HALO || d->H < 1) return false;
    // every k-range stays far below the 32-bit partial bound: 2^14 * positions < 2^31
    return true;
}

// widths served by wgrad_s1_3x3_v2
bool wgrad_v2_ok(const q8t_conv_desc *d) { return (d->W == 56 || d->W == 28) && d->C % CH2 == 0; }

WGeom wgrad_geom(const q8t_conv_desc *d)
{
    WGeom g;
    g.N = d->N; g.C = d->C; g.K = d->K; g.H = d->H; g.W = d->W; g.PQ = d->H * d->W;
    g.pitch = (d->W == 56) ? d->W + 8 : d->W + 4;   // must match the kernel variant chosen for this width
    g.Lp = d->H * g.pitch;
    g.rpitch = 1.0f / (float)g.pitch;
    g.chunks = (g.Lp + KC - 1) / KC;
    g.ncg = wgrad_v2_ok(d) ? d->C / CH2 : d->C / 16;
    g.nrg = d->K / 64;
    int want = 256 / (g.ncg * g.nrg);        // one workgroup per compute unit
    if (want < 1) want = 1;
    if (want > d->N) want = d->N;
    g.ipr = (d->N + want - 1) / want;
    // bound the positions per k-range so that 2^14 * padded positions stays below 2^31
    const int max_ipr = (int)(((int64_t)1 << 16) / (g.Lp + 64));
    if (g.ipr > max_ipr) g.ipr = max_ipr > 0 ? max_ipr : 1;
    g.S = (d->N + g.ipr - 1) / g.ipr;
    return g;
}

template <int WC>
int launch_wgrad(int blocks, hipStream_t st, const int16_t *g16, const int8_t *x, const q8t_qparams *qg,
                 const q8t_qparams *qx, const WGeom &g, int *ws)
{
    static Q8tLdsOptIn optin;
    if (q8t_allow_lds(optin, (const void *)wgrad_s1_3x3<WC>, SMEM_BYTES) != Q8T_OK) return Q8T_ERR_HIP;
    hipLaunchKernelGGL(wgrad_s1_3x3<WC>, dim3(blocks), dim3(kThreads), SMEM_BYTES, st, g16, x, qg, qx, g, ws);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

template <int WC>
int launch_wgrad_v2(int blocks, hipStream_t st, const int16_t *g16, const int8_t *x, const q8t_qparams *qg,
                    const q8t_qparams *qx, const WGeom &g, int *ws)
{
    static Q8tLdsOptIn optin;
    if (q8t_allow_lds(optin, (const void *)wgrad_s1_3x3_v2<WC>, SMEM2_BYTES) != Q8T_OK) return Q8T_ERR_HIP;
    hipLaunchKernelGGL(wgrad_s1_3x3_v2<WC>, dim3(blocks), dim3(kThreads), SMEM2_BYTES, st, g16, x, qg, qx, g, ws);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

}  // namespace

bool q8t_fast_wgrad_supported(const q8t_conv_desc *d, const void *g16, const void *x, const void *dw,
                              const void *acc)
{
    if (!wgrad_shape_ok(d)) return false;
    if ((int64_t)d->H * (d->W + 4) + 64 > ((int64_t)1 << 16)) return false;
    return q8t_aligned(g16, 16) && q8t_aligned(x, 8) && q8t_aligned(dw, 4) && q8t_aligned(acc, 8);
}

size_t q8t_fast_wgrad_ws(const q8t_conv_desc *d)
{
    if (!wgrad_shape_ok(d)) return 0;
    const WGeom g = wgrad_geom(d);
    return (size_t)g.S * g.nrg * g.ncg * (wgrad_v2_ok(d) ? PART2_INTS : PART_INTS) * sizeof(int);
}

int q8t_fast_wgrad(const q8t_conv_desc *d, const int16_t *g16, const q8t_qparams *qg, const int8_t *x,
                   const q8t_qparams *qx, float *dw, int64_t *acc_out, void *ws, hipStream_t st)
{
    if (!ws || !q8t_aligned(ws, 16)) return Q8T_ERR_WORKSPACE;
    const WGeom g = wgrad_geom(d);
    const int per = g.ncg * g.nrg;
    const int blocks = ((g.S + 7) / 8) * 8 * per;
    if (wgrad_v2_ok(d)) {
        const int rc2 = d->W == 56 ? launch_wgrad_v2<56>(blocks, st, g16, x, qg, qx, g, (int *)ws)
                                   : launch_wgrad_v2<28>(blocks, st, g16, x, qg, qx, g, (int *)ws);
        if (rc2) return rc2;
        int nq = 1;   // wavefronts per workgroup: each walks two ranges or more (measured best: 16 wavefronts of one range each spend their time starting up)
        while (nq < RQ2 && g.S >= 4 * nq) nq *= 2;
        hipLaunchKernelGGL(wgrad_reduce_v2, dim3(TILE2_INTS / 2 / 256, per), dim3(64 * nq), 0, st, (const int *)ws, g, qg, qx, dw,
                           acc_out);
        Q8T_LAUNCH_CHECK();
        return Q8T_OK;
    }
    const int rc = d->W == 56   ? launch_wgrad<56>(blocks, st, g16, x, qg, qx, g, (int *)ws)
                   : d->W == 28 ? launch_wgrad<28>(blocks, st, g16, x, qg, qx, g, (int *)ws)
                                : launch_wgrad<0>(blocks, st, g16, x, qg, qx, g, (int *)ws);
    if (rc) return rc;
    hipLaunchKernelGGL(wgrad_reduce, dim3(9216 / 64, per), dim3(256), 0, st, (const int *)ws, g, qg, qx, dw,
                       acc_out);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}
