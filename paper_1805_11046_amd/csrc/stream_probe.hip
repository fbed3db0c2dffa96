// Plain streaming kernels of known traffic: the measured ceiling that the HBM-bound calls of the
// library (quantize, Range BN) are compared with.  The access shape is the best of a sweep on this
// chip (slices against grid strides, 1024 to 32768 workgroups, 1 to 8 accesses in flight, plain
// against non-temporal loads): every workgroup streams one contiguous slice, non-temporal loads,
// two to four 16-byte accesses in flight per lane, 4096 workgroups.
#include "q8t_common.h"
#include "q8t_internal.h"

namespace {

constexpr int kThreads = 256;

typedef unsigned int u4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ldnt(const uint4 *p)
{
    const u4v v = __builtin_nontemporal_load(reinterpret_cast<const u4v *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// mode 0: dst = src (bytes read + bytes written); mode 1: read only (one word per workgroup
// written, so that the loads cannot be dropped); mode 2: fill dst with zeros
template <int MODE>
__global__ __launch_bounds__(kThreads) void probe_stream(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int64_t n16)
{
    const int64_t per = (n16 + gridDim.x - 1) / gridDim.x;
    const int64_t lo = (int64_t)blockIdx.x * per, hi = min(n16, lo + per);
    uint4 acc = make_uint4(0u, 0u, 0u, 0u);
    int64_t i = lo + threadIdx.x;
    for (; i + 3 * kThreads < hi; i += 4 * kThreads) {
        if (MODE == 2) {
            dst[i] = acc;
            dst[i + kThreads] = acc;
            dst[i + 2 * kThreads] = acc;
            dst[i + 3 * kThreads] = acc;
        } else {
            const uint4 a = ldnt(src + i), b = ldnt(src + i + kThreads), c = ldnt(src + i + 2 * kThreads), d = ldnt(src + i + 3 * kThreads);
            if (MODE == 0) {
                dst[i] = a;
                dst[i + kThreads] = b;
                dst[i + 2 * kThreads] = c;
                dst[i + 3 * kThreads] = d;
            } else {
                acc.x ^= a.x ^ b.x ^ c.x ^ d.x;
                acc.y ^= a.y ^ b.y ^ c.y ^ d.y;
                acc.z ^= a.z ^ b.z ^ c.z ^ d.z;
                acc.w ^= a.w ^ b.w ^ c.w ^ d.w;
            }
        }
    }
    for (; i < hi; i += kThreads) {
        if (MODE == 2) {
            dst[i] = acc;
        } else {
            const uint4 a = ldnt(src + i);
            if (MODE == 0) {
                dst[i] = a;
            } else {
                acc.x ^= a.x;
                acc.y ^= a.y;
                acc.z ^= a.z;
                acc.w ^= a.w;
            }
        }
    }
    if (MODE == 1) {
        uint32_t v = acc.x ^ acc.y ^ acc.z ^ acc.w;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v ^= __shfl_xor(v, off, Q8T_WAVE);
        if ((threadIdx.x & 63) == 0) ((uint32_t *)dst)[blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6)] = v;
    }
}

}  // namespace

extern "C" {

int q8t_probe_stream(int mode, const void *src, void *dst, int64_t bytes, void *stream)
{
    if (mode < 0 || mode > 2) return Q8T_ERR_SHAPE;
    if (bytes < 65536 || bytes % 16 != 0) return Q8T_ERR_SHAPE;
    if (!dst || (mode != 2 && !src)) return Q8T_ERR_NULL;
    if (!q8t_aligned(dst, 16) || (src && !q8t_aligned(src, 16))) return Q8T_ERR_SHAPE;
    const int64_t n16 = bytes / 16;
    int64_t g = (n16 + (int64_t)kThreads * 4 - 1) / ((int64_t)kThreads * 4);
    const int grid = (int)(g < 1 ? 1 : (g > 4096 ? 4096 : g));
    hipStream_t st = (hipStream_t)stream;
    const uint4 *s = (const uint4 *)src;
    uint4 *d = (uint4 *)dst;
    if (mode == 0)
        hipLaunchKernelGGL(probe_stream<0>, dim3(grid), dim3(kThreads), 0, st, s, d, n16);
    else if (mode == 1)
        hipLaunchKernelGGL(probe_stream<1>, dim3(grid), dim3(kThreads), 0, st, s, d, n16);
    else
        hipLaunchKernelGGL(probe_stream<2>, dim3(grid), dim3(kThreads), 0, st, s, d, n16);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

}  // extern "C"
