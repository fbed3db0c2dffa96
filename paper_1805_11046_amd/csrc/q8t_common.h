// Shared device/host helpers of libq8t (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "q8t.h"

#define Q8T_WAVE 64

#define Q8T_LAUNCH_CHECK()                                   \
    do {                                                     \
        if (hipGetLastError() != hipSuccess) return Q8T_ERR_HIP; \
    } while (0)

static inline __host__ __device__ bool q8t_aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

// A kernel that wants more than 64 KB of dynamic LDS has to be given a higher limit first.  One
// flag per kernel (a function-local static at the launch site) remembers, per device, that this
// was done: atomic, so host threads may race here, and raising the limit twice is harmless.
struct Q8tLdsOptIn {
    std::atomic<uint64_t> done{0};
};
static inline int q8t_allow_lds(Q8tLdsOptIn &flag, const void *kernel, size_t bytes)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return Q8T_ERR_HIP;
    const uint64_t bit = (uint64_t)1 << (dev & 63);
    if (flag.done.load(std::memory_order_acquire) & bit) return Q8T_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
        return Q8T_ERR_HIP;
    flag.done.fetch_or(bit, std::memory_order_release);
    return Q8T_OK;
}

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

// 16-byte loads of streamed tensors: non-temporal, measured 8-12% faster than plain loads on cold
// tensors (6.4 against 5.7 TB/s for a read-only stream).  q8t_ld_last: the last pass of a call over
// its input; q8t_ld_first: the first of two passes over the same tensor.  Kept apart because the
// second pass can find part of the tensor in the Infinity Cache: measured inside the step, both
// non-temporal is the best setting for quantize and Range BN forward and neutral for the two-pass
// Range BN backward, while a plain first pass with a non-temporal second one is 15% slower there.
typedef float q8t_f4 __attribute__((ext_vector_type(4)));
#ifndef Q8T_NT_LAST
#define Q8T_NT_LAST 1
#endif
#ifndef Q8T_NT_FIRST
#define Q8T_NT_FIRST 1
#endif
__device__ __forceinline__ float4 q8t_ld_last(const float4 *p)
{
#if Q8T_NT_LAST
    const q8t_f4 v = __builtin_nontemporal_load(reinterpret_cast<const q8t_f4 *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
#else
    return *p;
#endif
}
__device__ __forceinline__ float4 q8t_ld_first(const float4 *p)
{
#if Q8T_NT_FIRST
    const q8t_f4 v = __builtin_nontemporal_load(reinterpret_cast<const q8t_f4 *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
#else
    return *p;
#endif
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

// ---- counter-based generator: 3 hashes serve the 4 elements of one group ----------------------
__device__ __forceinline__ uint32_t mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x6A09E667u;
    x ^= x >> 15;
    x *= 0xBB67AE85u;
    x ^= x >> 16;
    return x;
}
__device__ __forceinline__ void rng_group(uint32_t group, uint32_t seed_lo, uint32_t seed_hi,
                                          uint32_t &w0, uint32_t &w1)
{
    const uint32_t phi = 0x9E3779B9u;
    const uint32_t h = mix32(group * phi + seed_lo) ^ seed_hi;
    w0 = mix32(h + phi);
    w1 = mix32(h + 2u * phi);
}
__device__ __forceinline__ uint32_t rng_r16(int64_t i, uint32_t seed_lo, uint32_t seed_hi)
{
    uint32_t w0, w1;
    rng_group((uint32_t)(i >> 2), seed_lo, seed_hi, w0, w1);
    const uint32_t w = (i & 2) ? w1 : w0;
    return (w >> (16 * (uint32_t)(i & 1))) & 0xFFFFu;
}

template <typename OUT>
struct Pack4;
template <>
struct Pack4<int8_t> {
    typedef uint32_t type;
    static __device__ __forceinline__ uint32_t pack(int a, int b, int c, int d)
    {
        return (uint32_t)(a & 255) | ((uint32_t)(b & 255) << 8) | ((uint32_t)(c & 255) << 16) |
               ((uint32_t)(d & 255) << 24);
    }
};
template <>
struct Pack4<int16_t> {
    typedef uint2 type;
    static __device__ __forceinline__ uint2 pack(int a, int b, int c, int d)
    {
        return make_uint2((uint32_t)(a & 65535) | ((uint32_t)(b & 65535) << 16),
                          (uint32_t)(c & 65535) | ((uint32_t)(d & 65535) << 16));
    }
};

template <typename OUT, bool STOCH>
__device__ __forceinline__ typename Pack4<OUT>::type quant4(const float4 v, const Affine &a,
                                                           uint32_t group, uint32_t seed_lo,
                                                           uint32_t seed_hi)
{
    uint32_t w0 = 0, w1 = 0;
    if (STOCH) rng_group(group, seed_lo, seed_hi, w0, w1);
    const int q0 = level_of<STOCH>(v.x, a, w0 & 0xFFFFu) - a.half;
    const int q1 = level_of<STOCH>(v.y, a, w0 >> 16) - a.half;
    const int q2 = level_of<STOCH>(v.z, a, w1 & 0xFFFFu) - a.half;
    const int q3 = level_of<STOCH>(v.w, a, w1 >> 16) - a.half;
    return Pack4<OUT>::pack(q0, q1, q2, q3);
}


