// Shared main loop of the int8 MFMA GEMM kernels (conv_nhwc.hip, wgrad_gemm.hip).
//
// Workgroup tile 128 x BN (BN = 128 or 64), K-step 64, 4 wavefronts.  Operand rows of 64 bytes
// sit 80 bytes apart in LDS (conflict-free 16-byte reads).  LDS is double-buffered with one
// barrier per step; global loads run three steps ahead through three named register sets, so
// that a wavefront waits only for the oldest of the loads it has in flight.
//
// The kernel supplies an `Ops` object:
//   void load(Regs &r)                  issue the global loads of the next K-step into r
//   void store(const Regs &r, int buf)  write r into LDS buffer buf (and keep byte sums if wanted)
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace q8t_gemm {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int BM = 128;
constexpr int PITCH = 80;

struct Regs {
    uint4 a0, a1, b0, b1;
};

template <int BN>
struct Tile {
    static constexpr int WM = BN == 128 ? 2 : 4;   // wavefronts along the rows
    static constexpr int MT = BM / WM / 16;        // 16-row MFMA tiles per wavefront
    static constexpr int NT = 4;                   // 16-column MFMA tiles per wavefront
};

template <int BN>
__device__ __forceinline__ void compute_step(const int8_t *__restrict__ sa, const int8_t *__restrict__ sb, int rowbase,
                                             int colbase, int l16, int kb, v4i (&acc)[Tile<BN>::MT][Tile<BN>::NT])
{
    constexpr int MT = Tile<BN>::MT, NT = Tile<BN>::NT;
    v4i bf[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
        bf[nt] = *reinterpret_cast<const v4i *>(sb + (colbase + nt * 16 + l16) * PITCH + kb * 16);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const v4i a = *reinterpret_cast<const v4i *>(sa + (rowbase + mt * 16 + l16) * PITCH + kb * 16);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, bf[nt], acc[mt][nt], 0, 0, 0);
    }
}

// sA: 2 * BM * PITCH bytes, sB: 2 * BN * PITCH bytes
template <int BN, class Ops>
__device__ __forceinline__ void pipeline(Ops &ops, int steps, int8_t *__restrict__ sA, int8_t *__restrict__ sB,
                                         v4i (&acc)[Tile<BN>::MT][Tile<BN>::NT])
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, kb = lane >> 4;
    const int rowbase = BN == 128 ? (wave & 1) * 64 : wave * 32;
    const int colbase = BN == 128 ? (wave >> 1) * 64 : 0;
    Regs r0, r1, r2;
    r0.a0 = r0.a1 = r0.b0 = r0.b1 = make_uint4(0, 0, 0, 0);
    r1 = r0;
    r2 = r0;
    if (steps > 0) ops.load(r0);
    if (steps > 1) ops.load(r1);
    if (steps > 2) ops.load(r2);
#define Q8T_GEMM_STEP(R, S)                                                          \
    {                                                                                \
        const int buf = (S)&1;                                                       \
        ops.store(R, buf);                                                           \
        if ((S) + 3 < steps) ops.load(R);                                            \
        __syncthreads();                                                             \
        compute_step<BN>(sA + buf * BM * PITCH, sB + buf * BN * PITCH, rowbase, colbase, l16, kb, acc); \
    }
    for (int s = 0; s < steps; s += 3) {
        Q8T_GEMM_STEP(r0, s)
        if (s + 1 < steps) Q8T_GEMM_STEP(r1, s + 1)
        if (s + 2 < steps) Q8T_GEMM_STEP(r2, s + 2)
    }
#undef Q8T_GEMM_STEP
}

}  // namespace q8t_gemm
