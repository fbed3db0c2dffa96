// Shared main loop of the int8 MFMA GEMM kernels (conv_nhwc.hip, wgrad_gemm.hip).
//
// Three tile configurations (rows x columns of the workgroup tile, K-step 64):
//   Big    256 x 256, 8 wavefronts of 128 x 64   (one workgroup per compute unit)
//   Mid    128 x 128, 4 wavefronts of  64 x 64   (three workgroups per compute unit)
//   Small  128 x  64, 4 wavefronts of  32 x 64
// Per K-step a wavefront of the Big tile reads 12 operand fragments from LDS for 32 MFMAs, of the
// Mid tile 8 for 16: the Big tile halves the LDS and global traffic per MFMA and is what the
// MFMA-bound shapes use.
//
// LDS holds rows of 64 bytes without padding; the 16-byte chunk q of row r sits at chunk
// q ^ swz(r), which keeps the column-wise fragment reads free of bank conflicts (the row-wise
// staging stores are insensitive to the permutation).  LDS is double-buffered with one barrier per step.  The barrier orders
// LDS traffic only (q8t_lds_barrier), so the global loads of the next steps stay in flight across
// it: two named register sets hold the tiles of steps s+1 and s+2 while step s is multiplied.
// The loop body is straight-line code (no branch around a load or a store), which lets the
// compiler's wait-count bookkeeping keep the younger loads in flight; the step count is rounded
// up to an even number and the surplus step multiplies staged zeros.
//
// The kernel supplies an `Ops` object:
//   void load(Regs &r, bool valid)     issue the global loads of the next K-step: a0 / a1 = chunk q of
//                                      tile rows ar and ar + RP, b0 / b1 likewise for the columns
//                                      (valid == false: any readable address, no advance)
//   void prepare(Regs &r, bool valid)  called right before the registers go to LDS: transform them
//                                      in place (byte-plane split, byte sums); with !valid the B
//                                      registers must become zero (and A too if sums are kept)
// with ar = tid >> 2, q = tid & 3, RP = threads / 4.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "q8t_common.h"

namespace q8t_gemm {

typedef int v4i __attribute__((ext_vector_type(4)));

// Workgroups are handed to the 8 XCDs (each with its own L2) round-robin by linear index.  The
// kernels are launched on a 1-D grid of 8*ceil(total/8) workgroups and run logical tile
// xcd_logical(blockIdx.x, total): consecutive logical tiles, which share an operand tile, then
// execute back to back on one XCD and find it in that XCD's L2.  A result >= total means "exit".
__device__ __forceinline__ int xcd_logical(int linear, int total)
{
    const int per = (total + 7) >> 3;
    return (linear & 7) * per + (linear >> 3);
}
inline unsigned xcd_grid(int64_t total) { return (unsigned)(((total + 7) >> 3) << 3); }

struct Regs {
    uint4 a0, a1, b0, b1;
};

__device__ __forceinline__ uint4 sel16(bool c, const uint4 &v)
{
    return make_uint4(c ? v.x : 0u, c ? v.y : 0u, c ? v.z : 0u, c ? v.w : 0u);
}

// Chunk permutation of an LDS row; depends on bits 1..2 of the row only, so rows 64 or 128 apart
// share it.  A 16-byte-per-lane LDS read is served in four phases of 16 lanes that are not
// consecutive lanes (measured on gfx950: lanes {0-3, 12-15, 20-23, 24-27} go together, and so on),
// so a fragment read (lane -> row lane % 16, chunk lane / 16) meets rows {0-3, 12-15} of one chunk
// with rows 4-11 of the next in one phase.  With this permutation those 16 accesses fall into 16
// different 16-byte bank groups: 207 bytes / clock / CU measured against 122 for the unpermuted
// layout, for an 80-byte row pitch or for permutations built for consecutive lanes.
__device__ __forceinline__ int swz(int r) { return (r >> 1) & 3; }

template <int BM_, int BN_>
struct Cfg {
    static constexpr int BM = BM_, BN = BN_;
    static constexpr int THREADS = BM == 256 ? 512 : 256;
    static constexpr int RP = THREADS / 4;                      // rows staged per pass
    static constexpr int MT = BM == 256 ? 8 : (BN == 128 ? 4 : 2);
    static constexpr int NT = 4;
    static constexpr int NB = BN / RP;                          // column passes (1 or 2)
    static constexpr int LDS_BYTES = 2 * (BM + BN) * 64;
    static constexpr int MINB = BM == 256 ? 1 : 3;              // workgroups per compute unit aimed at
    __device__ static __forceinline__ int rowbase(int wave)
    {
        return BM == 256 ? (wave & 1) * 128 : (BN == 128 ? (wave & 1) * 64 : wave * 32);
    }
    __device__ static __forceinline__ int colbase(int wave) { return BN == 64 ? 0 : (wave >> 1) * 64; }
};
typedef Cfg<256, 256> Big;
typedef Cfg<128, 128> Mid;
typedef Cfg<128, 64> Small;

template <class C>
__device__ __forceinline__ void compute_step(const int8_t *__restrict__ sa, const int8_t *__restrict__ sb, int rowbase,
                                             int colbase, int l16, int kb, v4i (&acc)[C::MT][C::NT])
{
    v4i bf[C::NT];
#pragma unroll
    for (int nt = 0; nt < C::NT; ++nt) {
        const int row = colbase + nt * 16 + l16;
        bf[nt] = *reinterpret_cast<const v4i *>(sb + row * 64 + ((kb ^ swz(row)) * 16));
    }
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt) {
        const int row = rowbase + mt * 16 + l16;
        const v4i af = *reinterpret_cast<const v4i *>(sa + row * 64 + ((kb ^ swz(row)) * 16));
#pragma unroll
        for (int nt = 0; nt < C::NT; ++nt)
            acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(af, bf[nt], acc[mt][nt], 0, 0, 0);
    }
}

// sA: 2 * BM * 64 bytes, sB: 2 * BN * 64 bytes
template <class C, class Ops>
__device__ __forceinline__ void pipeline(Ops &ops, int steps, int8_t *__restrict__ sA, int8_t *__restrict__ sB,
                                         v4i (&acc)[C::MT][C::NT])
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, kb = lane >> 4;
    const int rowbase = C::rowbase(wave), colbase = C::colbase(wave);
    const int ar = tid >> 2;
    const int so = ar * 64 + (((tid & 3) ^ swz(ar)) * 16);   // LDS offset of the thread's chunk in row ar
    if (steps <= 0) return;
    Regs q0, q1;
    q0.a0 = q0.a1 = q0.b0 = q0.b1 = make_uint4(0, 0, 0, 0);
    q1 = q0;
#define Q8T_GEMM_STORE(R, BUF, VALID)                                                   \
    {                                                                                   \
        Regs t_ = R;                                                                    \
        ops.prepare(t_, VALID);                                                         \
        int8_t *a_ = sA + (BUF)*C::BM * 64 + so, *b_ = sB + (BUF)*C::BN * 64 + so;      \
        *reinterpret_cast<uint4 *>(a_) = t_.a0;                                         \
        *reinterpret_cast<uint4 *>(a_ + C::RP * 64) = t_.a1;                            \
        *reinterpret_cast<uint4 *>(b_) = t_.b0;                                         \
        if (C::NB == 2) *reinterpret_cast<uint4 *>(b_ + C::RP * 64) = t_.b1;            \
    }
    // one step: MFMAs on buffer S&1 while tile S+1 goes from registers to the other buffer and the
    // loads of tile S+3 are issued; everything between two barriers is one scheduling region
#define Q8T_GEMM_STEP(R, S)                                                             \
    {                                                                                   \
        const int buf = (S)&1;                                                          \
        compute_step<C>(sA + buf * C::BM * 64, sB + buf * C::BN * 64, rowbase, colbase, l16, kb, acc); \
        Q8T_GEMM_STORE(R, buf ^ 1, (S) + 1 < steps)                                     \
        ops.load(R, (S) + 3 < steps);                                                   \
        q8t_lds_barrier();                                                              \
    }
    ops.load(q0, true);
    ops.load(q1, 1 < steps);
    Q8T_GEMM_STORE(q0, 0, true)
    ops.load(q0, 2 < steps);
    q8t_lds_barrier();
    for (int s = 0; s < steps; s += 2) {
        Q8T_GEMM_STEP(q1, s)
        Q8T_GEMM_STEP(q0, s + 1)
    }
#undef Q8T_GEMM_STEP
#undef Q8T_GEMM_STORE
}

}  // namespace q8t_gemm
