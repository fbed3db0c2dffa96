// Shared device/host helpers of libq8t (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "q8t.h"

#define Q8T_WAVE 64

#define Q8T_LAUNCH_CHECK()                                   \
    do {                                                     \
        if (hipGetLastError() != hipSuccess) return Q8T_ERR_HIP; \
    } while (0)

static inline bool q8t_aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also drains every global load
// in flight (s_waitcnt vmcnt(0)), which serialises a software pipeline that prefetches the next
// tiles into registers; here the wavefront waits for its LDS operations, and the registers that
// global loads are still filling are guarded by the compiler's own wait counts at their first use.
__device__ __forceinline__ void q8t_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---- wavefront (64 lanes) and workgroup reductions ------------------------------------------
template <typename T, typename Op>
__device__ __forceinline__ T wave_reduce(T v, Op op)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = op(v, __shfl_xor(v, off, Q8T_WAVE));
    return v;
}

struct OpMin {
    __device__ __forceinline__ float operator()(float a, float b) const { return fminf(a, b); }
};
struct OpMax {
    __device__ __forceinline__ float operator()(float a, float b) const { return fmaxf(a, b); }
};
struct OpAddD {
    __device__ __forceinline__ double operator()(double a, double b) const { return a + b; }
};

// ---- Appendix B: scale / zero point from a range, one fp32 rounding per operation ------------
__device__ __forceinline__ q8t_qparams make_qparams(float vmin, float vmax, int bits)
{
    if (vmin > 0.0f) vmin = 0.0f;  // widen the range so that 0 is a level
    if (vmax < 0.0f) vmax = 0.0f;
    const int qmax = (1 << bits) - 1;
    const float span = vmax - vmin;
    float scale = span / (float)qmax;
    if (scale == 0.0f) scale = 1.0f;
    const float inv_scale = 1.0f / scale;
    const float zf = (-vmin) * inv_scale;
    float zr = __builtin_rintf(zf);
    zr = fminf(fmaxf(zr, 0.0f), (float)qmax);
    q8t_qparams qp;
    qp.vmin = vmin;
    qp.vmax = vmax;
    qp.scale = scale;
    qp.inv_scale = inv_scale;
    qp.zero_point = (int)zr;
    qp.bits = bits;
    return qp;
}

// ---- Appendix B: level of one element --------------------------------------------------------
struct Affine {
    float inv_scale, zpf, qmaxf;
    int half;
};

// level of one element; separate multiply and add (the file is built without fp contraction)
template <bool STOCH>
__device__ __forceinline__ int level_of(float x, const Affine &a, uint32_t r16)
{
    const float u = x * a.inv_scale;
    const float t = u + a.zpf;
    float q;
    if (!STOCH) {
        q = __builtin_rintf(t);
    } else {
        const float f = __builtin_floorf(t);
        const float frac = t - f;
        const float lhs = frac * 65536.0f;
        const float rhs = (float)r16 + 0.5f;
        q = (lhs > rhs) ? f + 1.0f : f;
    }
    q = fminf(fmaxf(q, 0.0f), a.qmaxf);
    return (int)q;
}

__device__ __forceinline__ Affine affine_of(const q8t_qparams &qp)
{
    Affine a;
    a.inv_scale = qp.inv_scale;
    a.zpf = (float)qp.zero_point;
    a.qmaxf = (float)((1 << qp.bits) - 1);
    a.half = 1 << (qp.bits - 1);
    return a;
}

