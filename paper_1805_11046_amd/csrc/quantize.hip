// Per-tensor min/max affine quantization (Appendix B), nearest or stochastic rounding
// (Section 4), and the fused 8+16-bit "gradient bifurcation" pass (Sections 1 and 7).
//
// Two launches per call, no host synchronization in between:
//   1. minmax_partials : grid-stride pass, float4 loads, wavefront-shuffle reductions, one
//                        (min,max) pair per workgroup into the workspace.
//   2. quantize_apply  : every workgroup folds the <=1024 pairs itself (identical fp32 sequence in
//                        every workgroup, so they all agree bit for bit), derives scale and zero
//                        point, then quantizes its share: 4 elements -> one packed store.
// HBM-bound: 9 algorithmic bytes per element for 8-bit output (4 read + 4 re-read + 1 written).
#include <mutex>

#include "q8t_common.h"
#include "q8t_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kMaxPartials = 1024;
}  // namespace

// Scratch of q8t_quantize_noalloc: the (min,max) pairs of pass 1.  Every GPU the library runs on
// holds its own copy at its own address until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress; kernels and copies take the per-device address kept below.
static __device__ __align__(256) unsigned char scratch[sizeof(float2) * kMaxPartials];

namespace {
constexpr int kSmallThreads = 1024;
constexpr int64_t kSmallN = 1 << 16;   // below this, one workgroup does both passes

__device__ __forceinline__ float block_reduce_min(float v, float *smem)
{
    v = wave_reduce(v, OpMin());
    if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = smem[0];
    for (int w = 1; w < kThreads / 64; ++w) r = fminf(r, smem[w]);
    __syncthreads();
    return r;
}
__device__ __forceinline__ float block_reduce_max(float v, float *smem)
{
    v = wave_reduce(v, OpMax());
    if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = smem[0];
    for (int w = 1; w < kThreads / 64; ++w) r = fmaxf(r, smem[w]);
    __syncthreads();
    return r;
}

__device__ __forceinline__ void mm4(float &mn, float &mx, const float4 v)
{
    mn = fminf(fminf(mn, v.x), fminf(v.y, fminf(v.z, v.w)));
    mx = fmaxf(fmaxf(mx, v.x), fmaxf(v.y, fmaxf(v.z, v.w)));
}

// pass 1: one (min,max) pair per workgroup
template <bool VEC>
__global__ __launch_bounds__(kThreads) void minmax_partials(const float *__restrict__ x, int64_t n,
                                                            float2 *__restrict__ partials)
{
    __shared__ float smem[kThreads / 64];
    float mn = INFINITY, mx = -INFINITY;
    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    if (VEC) {
        // each workgroup streams one contiguous slice (better DRAM channel spread than a
        // grid-wide stride), 4 independent 16-byte loads in flight per lane
        const int64_t n4 = n >> 2;
        const float4 *x4 = reinterpret_cast<const float4 *>(x);
        const int64_t per = (n4 + gridDim.x - 1) / gridDim.x;
        const int64_t lo = (int64_t)blockIdx.x * per, hi = min(n4, lo + per);
        int64_t i = lo + threadIdx.x;
        for (; i + 3 * kThreads < hi; i += 4 * kThreads) {
            const float4 a = q8t_ld_first(x4 + i), b = q8t_ld_first(x4 + i + kThreads), c = q8t_ld_first(x4 + i + 2 * kThreads), d = q8t_ld_first(x4 + i + 3 * kThreads);
            mm4(mn, mx, a);
            mm4(mn, mx, b);
            mm4(mn, mx, c);
            mm4(mn, mx, d);
        }
        for (; i < hi; i += kThreads) mm4(mn, mx, q8t_ld_first(x4 + i));
        const int64_t tail = (n4 << 2) + gid;  // the n % 4 leftover elements
        if (tail < n) {
            mn = fminf(mn, x[tail]);
            mx = fmaxf(mx, x[tail]);
        }
    } else {
        for (int64_t i = gid; i < n; i += stride) {
            mn = fminf(mn, x[i]);
            mx = fmaxf(mx, x[i]);
        }
    }
    mn = block_reduce_min(mn, smem);
    mx = block_reduce_max(mx, smem);
    if (threadIdx.x == 0) partials[blockIdx.x] = make_float2(mn, mx);
}

// every workgroup folds the partial pairs in the same order -> identical range everywhere
__device__ __forceinline__ void fold_partials(const float2 *__restrict__ partials, int npartials,
                                              float *smem, float &vmin, float &vmax)
{
    float mn = INFINITY, mx = -INFINITY;
    for (int i = threadIdx.x; i < npartials; i += kThreads) {
        const float2 p = partials[i];
        mn = fminf(mn, p.x);
        mx = fmaxf(mx, p.y);
    }
    vmin = block_reduce_min(mn, smem);
    vmax = block_reduce_max(mx, smem);
}

// pass 2, single output
template <typename OUT, bool STOCH, bool VEC>
__global__ __launch_bounds__(kThreads) void quantize_apply(
    const float *__restrict__ x, int64_t n, int bits, uint32_t seed_lo, uint32_t seed_hi,
    const float2 *__restrict__ partials, int npartials, OUT *__restrict__ q_out,
    q8t_qparams *__restrict__ qp_out)
{
    __shared__ float smem[kThreads / 64];
    float vmin, vmax;
    fold_partials(partials, npartials, smem, vmin, vmax);
    const q8t_qparams qp = make_qparams(vmin, vmax, bits);
    if (blockIdx.x == 0 && threadIdx.x == 0) *qp_out = qp;
    const Affine a = affine_of(qp);

    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    if (VEC) {
        typedef typename Pack4<OUT>::type P;
        const int64_t n4 = n >> 2;
        const float4 *x4 = reinterpret_cast<const float4 *>(x);
        P *q4 = reinterpret_cast<P *>(q_out);
        const int64_t per = (n4 + gridDim.x - 1) / gridDim.x;
        const int64_t lo = (int64_t)blockIdx.x * per, hi = min(n4, lo + per);
        int64_t i = lo + threadIdx.x;
        for (; i + 3 * kThreads < hi; i += 4 * kThreads) {
            const float4 v0 = q8t_ld_last(x4 + i), v1 = q8t_ld_last(x4 + i + kThreads), v2 = q8t_ld_last(x4 + i + 2 * kThreads), v3 = q8t_ld_last(x4 + i + 3 * kThreads);
            q4[i] = quant4<OUT, STOCH>(v0, a, (uint32_t)i, seed_lo, seed_hi);
            q4[i + kThreads] = quant4<OUT, STOCH>(v1, a, (uint32_t)(i + kThreads), seed_lo, seed_hi);
            q4[i + 2 * kThreads] = quant4<OUT, STOCH>(v2, a, (uint32_t)(i + 2 * kThreads), seed_lo, seed_hi);
            q4[i + 3 * kThreads] = quant4<OUT, STOCH>(v3, a, (uint32_t)(i + 3 * kThreads), seed_lo, seed_hi);
        }
        for (; i < hi; i += kThreads) q4[i] = quant4<OUT, STOCH>(q8t_ld_last(x4 + i), a, (uint32_t)i, seed_lo, seed_hi);
        const int64_t tail = (n4 << 2) + gid;
        if (tail < n) {
            const uint32_t r = STOCH ? rng_r16(tail, seed_lo, seed_hi) : 0u;
            q_out[tail] = (OUT)(level_of<STOCH>(x[tail], a, r) - a.half);
        }
    } else {
        for (int64_t i = gid; i < n; i += stride) {
            const uint32_t r = STOCH ? rng_r16(i, seed_lo, seed_hi) : 0u;
            q_out[i] = (OUT)(level_of<STOCH>(x[i], a, r) - a.half);
        }
    }
}

// small tensors (weights of a layer): both passes in one workgroup, one launch.  The tensor is
// read once, with every load of a thread in flight at the same time (one memory latency instead
// of one per element), and quantized out of registers.
template <typename OUT, bool STOCH, bool VEC>
__global__ __launch_bounds__(kSmallThreads) void quantize_small(const float *__restrict__ x, int n, int bits,
                                                                uint32_t seed_lo, uint32_t seed_hi,
                                                                OUT *__restrict__ q_out,
                                                                q8t_qparams *__restrict__ qp_out)
{
    constexpr int PER = kSmallN / kSmallThreads;   // elements per thread
    __shared__ float smn[kSmallThreads / 64], smx[kSmallThreads / 64];
    float mn = INFINITY, mx = -INFINITY;
    float v[PER];
    if (VEC) {
        const float4 *x4 = reinterpret_cast<const float4 *>(x);
        const int n4 = n >> 2;
#pragma unroll
        for (int k = 0; k < PER / 4; ++k) {
            const int i = threadIdx.x + k * kSmallThreads;
            float4 t = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (i < n4) t = x4[i];
            v[4 * k] = t.x;
            v[4 * k + 1] = t.y;
            v[4 * k + 2] = t.z;
            v[4 * k + 3] = t.w;
        }
#pragma unroll
        for (int k = 0; k < PER / 4; ++k)
            if (threadIdx.x + k * kSmallThreads < n4) {
                mn = fminf(fminf(mn, v[4 * k]), fminf(v[4 * k + 1], fminf(v[4 * k + 2], v[4 * k + 3])));
                mx = fmaxf(fmaxf(mx, v[4 * k]), fmaxf(v[4 * k + 1], fmaxf(v[4 * k + 2], v[4 * k + 3])));
            }
    } else {
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int i = threadIdx.x + k * kSmallThreads;
            v[k] = i < n ? x[i] : 0.0f;
        }
#pragma unroll
        for (int k = 0; k < PER; ++k)
            if (threadIdx.x + k * kSmallThreads < n) {
                mn = fminf(mn, v[k]);
                mx = fmaxf(mx, v[k]);
            }
    }
    mn = wave_reduce(mn, OpMin());
    mx = wave_reduce(mx, OpMax());
    if ((threadIdx.x & 63) == 0) {
        smn[threadIdx.x >> 6] = mn;
        smx[threadIdx.x >> 6] = mx;
    }
    __syncthreads();
    mn = smn[0];
    mx = smx[0];
    for (int w = 1; w < kSmallThreads / 64; ++w) {
        mn = fminf(mn, smn[w]);
        mx = fmaxf(mx, smx[w]);
    }
    const q8t_qparams qp = make_qparams(mn, mx, bits);
    if (threadIdx.x == 0) *qp_out = qp;
    const Affine a = affine_of(qp);
    if (VEC) {
        typedef typename Pack4<OUT>::type P;
        P *q4 = reinterpret_cast<P *>(q_out);
        const int n4 = n >> 2;
#pragma unroll
        for (int k = 0; k < PER / 4; ++k) {
            const int i = threadIdx.x + k * kSmallThreads;
            if (i < n4)
                q4[i] = quant4<OUT, STOCH>(make_float4(v[4 * k], v[4 * k + 1], v[4 * k + 2], v[4 * k + 3]), a, (uint32_t)i,
                                           seed_lo, seed_hi);
        }
    } else {
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int i = threadIdx.x + k * kSmallThreads;
            if (i < n) {
                const uint32_t r = STOCH ? rng_r16(i, seed_lo, seed_hi) : 0u;
                q_out[i] = (OUT)(level_of<STOCH>(v[k], a, r) - a.half);
            }
        }
    }
}

// pass 2, bifurcated: 8-bit and 16-bit stochastic copies from one read of g
template <bool VEC>
__global__ __launch_bounds__(kThreads) void quantize_bifurcate_apply(
    const float *__restrict__ x, int64_t n, uint32_t s8_lo, uint32_t s8_hi, uint32_t s16_lo,
    uint32_t s16_hi, const float2 *__restrict__ partials, int npartials, int8_t *__restrict__ q8,
    q8t_qparams *__restrict__ qp8_out, int16_t *__restrict__ q16, q8t_qparams *__restrict__ qp16_out)
{
    __shared__ float smem[kThreads / 64];
    float vmin, vmax;
    fold_partials(partials, npartials, smem, vmin, vmax);
    const q8t_qparams qp8 = make_qparams(vmin, vmax, 8);
    const q8t_qparams qp16 = make_qparams(vmin, vmax, 16);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        *qp8_out = qp8;
        *qp16_out = qp16;
    }
    const Affine a8 = affine_of(qp8), a16 = affine_of(qp16);
    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    if (VEC) {
        const int64_t n4 = n >> 2;
        const float4 *x4 = reinterpret_cast<const float4 *>(x);
        uint32_t *o8 = reinterpret_cast<uint32_t *>(q8);
        uint2 *o16 = reinterpret_cast<uint2 *>(q16);
        const int64_t per = (n4 + gridDim.x - 1) / gridDim.x;
        const int64_t lo = (int64_t)blockIdx.x * per, hi = min(n4, lo + per);
        int64_t i = lo + threadIdx.x;
        for (; i + kThreads < hi; i += 2 * kThreads) {
            const float4 v0 = q8t_ld_last(x4 + i), v1 = q8t_ld_last(x4 + i + kThreads);
            o8[i] = quant4<int8_t, true>(v0, a8, (uint32_t)i, s8_lo, s8_hi);
            o16[i] = quant4<int16_t, true>(v0, a16, (uint32_t)i, s16_lo, s16_hi);
            o8[i + kThreads] = quant4<int8_t, true>(v1, a8, (uint32_t)(i + kThreads), s8_lo, s8_hi);
            o16[i + kThreads] = quant4<int16_t, true>(v1, a16, (uint32_t)(i + kThreads), s16_lo, s16_hi);
        }
        for (; i < hi; i += kThreads) {
            const float4 v0 = q8t_ld_last(x4 + i);
            o8[i] = quant4<int8_t, true>(v0, a8, (uint32_t)i, s8_lo, s8_hi);
            o16[i] = quant4<int16_t, true>(v0, a16, (uint32_t)i, s16_lo, s16_hi);
        }
        const int64_t tail = (n4 << 2) + gid;
        if (tail < n) {
            q8[tail] = (int8_t)(level_of<true>(x[tail], a8, rng_r16(tail, s8_lo, s8_hi)) - a8.half);
            q16[tail] = (int16_t)(level_of<true>(x[tail], a16, rng_r16(tail, s16_lo, s16_hi)) - a16.half);
        }
    } else {
        for (int64_t i = gid; i < n; i += stride) {
            q8[i] = (int8_t)(level_of<true>(x[i], a8, rng_r16(i, s8_lo, s8_hi)) - a8.half);
            q16[i] = (int16_t)(level_of<true>(x[i], a16, rng_r16(i, s16_lo, s16_hi)) - a16.half);
        }
    }
}

// the element width follows qp->bits, which only the device knows
__global__ __launch_bounds__(kThreads) void dequantize_kernel(const void *__restrict__ q,
                                                              const q8t_qparams *__restrict__ qp,
                                                              int64_t n, float *__restrict__ out)
{
    const float scale = qp->scale;
    const int bits = qp->bits;
    const int shift = (1 << (bits - 1)) - qp->zero_point;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    const int8_t *q8 = (const int8_t *)q;
    const int16_t *q16 = (const int16_t *)q;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
        const int s = (bits <= 8) ? (int)q8[i] : (int)q16[i];
        out[i] = scale * (float)(s + shift);
    }
}

int grid_for(int64_t work_items, int per_thread, int cap)
{
    int64_t g = (work_items + (int64_t)kThreads * per_thread - 1) / ((int64_t)kThreads * per_thread);
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

constexpr int64_t kMaxElements = (int64_t)1 << 34;

template <typename OUT>
int launch_apply(const float *x, int64_t n, int bits, int stochastic, uint64_t seed,
                 const float2 *partials, int npartials, OUT *q, q8t_qparams *qp, hipStream_t st)
{
    const bool vec = q8t_aligned(x, 16) && q8t_aligned(q, 4 * sizeof(OUT));
    const int grid = grid_for(vec ? (n >> 2) : n, 4, 2048);
    const uint32_t lo = (uint32_t)seed, hi = (uint32_t)(seed >> 32);
#define Q8T_GO(S, V) \
    hipLaunchKernelGGL((quantize_apply<OUT, S, V>), dim3(grid), dim3(kThreads), 0, st, x, n, bits, lo, hi, partials, npartials, q, qp)
    if (stochastic) {
        if (vec) Q8T_GO(true, true); else Q8T_GO(true, false);
    } else {
        if (vec) Q8T_GO(false, true); else Q8T_GO(false, false);
    }
#undef Q8T_GO
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

int launch_minmax(const float *x, int64_t n, float2 *partials, hipStream_t st)
{
    if (n == 0) return 0;
    const bool vec = q8t_aligned(x, 16);
    const int grid = grid_for(vec ? (n >> 2) : n, 8, 1024);
    if (vec)
        hipLaunchKernelGGL(minmax_partials<true>, dim3(grid), dim3(kThreads), 0, st, x, n, partials);
    else
        hipLaunchKernelGGL(minmax_partials<false>, dim3(grid), dim3(kThreads), 0, st, x, n, partials);
    return grid;
}

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_addr[kMaxDevices];   // device address of `scratch` on each device, 0 = not asked yet

// address of this device's copy of `scratch` (asked from the runtime once per device)
int scratch_of_current_device(float2 **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return Q8T_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_addr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return Q8T_ERR_HIP;
        g_scratch_addr[dev] = p;
    }
    *out = (float2 *)g_scratch_addr[dev];
    return Q8T_OK;
}

int quantize_impl(const float *x, int64_t n, int bits, int stochastic, uint64_t seed, void *q_out,
                  q8t_qparams *qp_out, float2 *partials, hipStream_t st);

// ---- several tensors in two launches (the weights of a network at the start of a step) ----------
// Every tensor keeps its own range: the result for tensor t is that of q8t_quantize(x[t], n[t], bits, 0, ...).
// A workgroup handles kMultiBlock consecutive elements of one tensor; the table that maps workgroups to
// tensors travels as a kernel argument.
constexpr int kMultiMax = 32;
constexpr int kMultiBlock = 16384;
struct MultiArgs {
    const float *x[kMultiMax];
    int8_t *q[kMultiMax];
    q8t_qparams *qp[kMultiMax];
    int64_t n[kMultiMax];
    int first[kMultiMax + 1];   // first workgroup of tensor t; first[count] = number of workgroups
    int count, bits;
};

__device__ __forceinline__ int multi_tensor_of(const MultiArgs &a, int b)
{
    int t = 0;
    while (t + 1 < a.count && a.first[t + 1] <= b) ++t;
    return t;
}

__global__ __launch_bounds__(kThreads) void multi_minmax(const MultiArgs a, float2 *__restrict__ partials)
{
    __shared__ float smem[kThreads / 64];
    const int b = blockIdx.x, t = multi_tensor_of(a, b);
    const float *x = a.x[t];
    const int64_t lo = (int64_t)(b - a.first[t]) * kMultiBlock, hi = min(a.n[t], lo + kMultiBlock);
    float mn = INFINITY, mx = -INFINITY;
    if (q8t_aligned(x, 16)) {
        const int64_t hi4 = lo + ((hi - lo) & ~(int64_t)3);   // lo is a multiple of 4
        for (int64_t i = lo + 4 * threadIdx.x; i < hi4; i += 4 * kThreads) mm4(mn, mx, *reinterpret_cast<const float4 *>(x + i));
        for (int64_t i = hi4 + threadIdx.x; i < hi; i += kThreads) {
            mn = fminf(mn, x[i]);
            mx = fmaxf(mx, x[i]);
        }
    } else {
        for (int64_t i = lo + threadIdx.x; i < hi; i += kThreads) {
            mn = fminf(mn, x[i]);
            mx = fmaxf(mx, x[i]);
        }
    }
    mn = block_reduce_min(mn, smem);
    mx = block_reduce_max(mx, smem);
    if (threadIdx.x == 0) partials[b] = make_float2(mn, mx);
}

__global__ __launch_bounds__(kThreads) void multi_apply(const MultiArgs a, const float2 *__restrict__ partials)
{
    __shared__ float smem[kThreads / 64];
    const int b = blockIdx.x, t = multi_tensor_of(a, b);
    float vmin, vmax;
    fold_partials(partials + a.first[t], a.first[t + 1] - a.first[t], smem, vmin, vmax);   // min / max: any order, same bits
    const q8t_qparams qp = make_qparams(vmin, vmax, a.bits);
    if (b == a.first[t] && threadIdx.x == 0) *a.qp[t] = qp;
    const Affine af = affine_of(qp);
    const float *x = a.x[t];
    int8_t *q = a.q[t];
    const int64_t lo = (int64_t)(b - a.first[t]) * kMultiBlock, hi = min(a.n[t], lo + kMultiBlock);
    if (q8t_aligned(x, 16) && q8t_aligned(q, 4)) {
        const int64_t hi4 = lo + ((hi - lo) & ~(int64_t)3);
        for (int64_t i = lo + 4 * threadIdx.x; i < hi4; i += 4 * kThreads)
            *reinterpret_cast<uint32_t *>(q + i) = quant4<int8_t, false>(*reinterpret_cast<const float4 *>(x + i), af, 0u, 0u, 0u);
        for (int64_t i = hi4 + threadIdx.x; i < hi; i += kThreads) q[i] = (int8_t)(level_of<false>(x[i], af, 0u) - af.half);
    } else {
        for (int64_t i = lo + threadIdx.x; i < hi; i += kThreads) q[i] = (int8_t)(level_of<false>(x[i], af, 0u) - af.half);
    }
}

}  // namespace

extern "C" {

int q8t_init(void)
{
    float2 *p;
    return scratch_of_current_device(&p);
}

int q8t_quantize_noalloc(const float *x, int64_t n, int bits, int stochastic, uint64_t seed, void *q_out,
                         q8t_qparams *qp_out, void *stream)
{
    if (n < 0 || n > Q8T_NOALLOC_MAX_ELEMENTS) return Q8T_ERR_SHAPE;
    if (bits < 2 || bits > 16) return Q8T_ERR_BITS;
    if (!qp_out || (n > 0 && (!x || !q_out))) return Q8T_ERR_NULL;
    float2 *partials;
    const int rc = scratch_of_current_device(&partials);
    if (rc) return rc;
    return quantize_impl(x, n, bits, stochastic, seed, q_out, qp_out, partials, (hipStream_t)stream);
}

size_t q8t_quantize_multi_workspace_size(int count, const int64_t *n)
{
    if (count <= 0 || !n) return 0;
    size_t blocks = 0;
    for (int t = 0; t < count; ++t) blocks += (size_t)((n[t] > 0 ? n[t] : 0) + kMultiBlock - 1) / kMultiBlock + 1;
    return blocks * sizeof(float2);
}

int q8t_quantize_multi(int count, const float *const *x, const int64_t *n, int bits, int8_t *const *q_out,
                       q8t_qparams *const *qp_out, void *ws, void *stream)
{
    if (count <= 0 || !x || !n || !q_out || !qp_out) return count <= 0 ? Q8T_ERR_SHAPE : Q8T_ERR_NULL;
    if (bits < 2 || bits > 8) return Q8T_ERR_BITS;
    for (int t = 0; t < count; ++t) {
        if (n[t] <= 0 || n[t] > ((int64_t)1 << 34)) return Q8T_ERR_SHAPE;
        if (!x[t] || !q_out[t] || !qp_out[t]) return Q8T_ERR_NULL;
    }
    if (!ws || !q8t_aligned(ws, 8)) return Q8T_ERR_WORKSPACE;
    float2 *partials = (float2 *)ws;
    for (int t0 = 0; t0 < count; t0 += kMultiMax) {
        MultiArgs a;
        a.count = count - t0 < kMultiMax ? count - t0 : kMultiMax;
        a.bits = bits;
        int blocks = 0;
        for (int t = 0; t < a.count; ++t) {
            a.x[t] = x[t0 + t];
            a.q[t] = q_out[t0 + t];
            a.qp[t] = qp_out[t0 + t];
            a.n[t] = n[t0 + t];
            a.first[t] = blocks;
            blocks += (int)((n[t0 + t] + kMultiBlock - 1) / kMultiBlock);
        }
        a.first[a.count] = blocks;
        hipLaunchKernelGGL(multi_minmax, dim3(blocks), dim3(kThreads), 0, (hipStream_t)stream, a, partials);
        Q8T_LAUNCH_CHECK();
        hipLaunchKernelGGL(multi_apply, dim3(blocks), dim3(kThreads), 0, (hipStream_t)stream, a, (const float2 *)partials);
        Q8T_LAUNCH_CHECK();
        partials += blocks;
    }
    return Q8T_OK;
}

size_t q8t_quantize_workspace_size(int64_t n)
{
    (void)n;
    return sizeof(float2) * kMaxPartials;
}

int q8t_quantize(const float *x, int64_t n, int bits, int stochastic, uint64_t seed, void *q_out,
                 q8t_qparams *qp_out, void *ws, void *stream)
{
    if (n < 0 || n > kMaxElements) return Q8T_ERR_SHAPE;
    if (bits < 2 || bits > 16) return Q8T_ERR_BITS;
    if (!qp_out || (n > 0 && (!x || !q_out))) return Q8T_ERR_NULL;
    if (!ws || !q8t_aligned(ws, 8)) return Q8T_ERR_WORKSPACE;
    return quantize_impl(x, n, bits, stochastic, seed, q_out, qp_out, (float2 *)ws, (hipStream_t)stream);
}

}  // extern "C"

namespace {

// both passes of q8t_quantize / q8t_quantize_noalloc; arguments already checked
int quantize_impl(const float *x, int64_t n, int bits, int stochastic, uint64_t seed, void *q_out,
                  q8t_qparams *qp_out, float2 *partials, hipStream_t st)
{
    if (n > 0 && n <= kSmallN) {
        const uint32_t lo = (uint32_t)seed, hi = (uint32_t)(seed >> 32);
#define Q8T_SMALL(T, S, V) hipLaunchKernelGGL((quantize_small<T, S, V>), dim3(1), dim3(kSmallThreads), 0, st, x, (int)n, bits, lo, hi, (T *)q_out, qp_out)
        const bool vec = n % 4 == 0 && q8t_aligned(x, 16) && q8t_aligned(q_out, bits <= 8 ? 4 : 8);
        if (bits <= 8) {
            if (stochastic) { if (vec) Q8T_SMALL(int8_t, true, true); else Q8T_SMALL(int8_t, true, false); }
            else            { if (vec) Q8T_SMALL(int8_t, false, true); else Q8T_SMALL(int8_t, false, false); }
        } else {
            if (stochastic) { if (vec) Q8T_SMALL(int16_t, true, true); else Q8T_SMALL(int16_t, true, false); }
            else            { if (vec) Q8T_SMALL(int16_t, false, true); else Q8T_SMALL(int16_t, false, false); }
        }
#undef Q8T_SMALL
        Q8T_LAUNCH_CHECK();
        return Q8T_OK;
    }
    const int np = launch_minmax(x, n, partials, st);
    Q8T_LAUNCH_CHECK();
    if (bits <= 8)
        return launch_apply<int8_t>(x, n, bits, stochastic, seed, partials, np, (int8_t *)q_out, qp_out, st);
    return launch_apply<int16_t>(x, n, bits, stochastic, seed, partials, np, (int16_t *)q_out, qp_out, st);
}

}  // namespace

// second pass of q8t_quantize alone, the range given as up to 1024 (min, max) pairs that a producing
// kernel left behind (glue.hip: the rectified residual sum knows its maximum when it is written)
int q8t_quantize8_from_partials(const float *x, int64_t n, const void *minmax_pairs, int npairs, int8_t *q_out,
                                q8t_qparams *qp_out, hipStream_t st)
{
    return launch_apply<int8_t>(x, n, 8, 0, 0, (const float2 *)minmax_pairs, npairs, q_out, qp_out, st);
}

extern "C" {

int q8t_quantize_with_range(const float *x, int64_t n, int bits, int stochastic, uint64_t seed,
                            const float *vmin_vmax, void *q_out, q8t_qparams *qp_out, void *stream)
{
    if (n < 0 || n > kMaxElements) return Q8T_ERR_SHAPE;
    if (bits < 2 || bits > 16) return Q8T_ERR_BITS;
    if (!qp_out || !vmin_vmax || (n > 0 && (!x || !q_out))) return Q8T_ERR_NULL;
    if (!q8t_aligned(vmin_vmax, 8)) return Q8T_ERR_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    // the supplied pair plays the role of a single partial result
    const float2 *partials = (const float2 *)vmin_vmax;
    if (bits <= 8)
        return launch_apply<int8_t>(x, n, bits, stochastic, seed, partials, 1, (int8_t *)q_out, qp_out, st);
    return launch_apply<int16_t>(x, n, bits, stochastic, seed, partials, 1, (int16_t *)q_out, qp_out, st);
}

int q8t_quantize_bifurcate(const float *g, int64_t n, uint64_t seed8, uint64_t seed16, int8_t *q8_out,
                           q8t_qparams *qp8_out, int16_t *q16_out, q8t_qparams *qp16_out, void *ws,
                           void *stream)
{
    if (n < 0 || n > kMaxElements) return Q8T_ERR_SHAPE;
    if (!qp8_out || !qp16_out || (n > 0 && (!g || !q8_out || !q16_out))) return Q8T_ERR_NULL;
    if (!ws || !q8t_aligned(ws, 8)) return Q8T_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    float2 *partials = (float2 *)ws;
    const int np = launch_minmax(g, n, partials, st);
    Q8T_LAUNCH_CHECK();
    const bool vec = q8t_aligned(g, 16) && q8t_aligned(q8_out, 4) && q8t_aligned(q16_out, 8);
    const int grid = grid_for(vec ? (n >> 2) : n, 2, 2048);
    if (vec)
        hipLaunchKernelGGL(quantize_bifurcate_apply<true>, dim3(grid), dim3(kThreads), 0, st, g, n,
                           (uint32_t)seed8, (uint32_t)(seed8 >> 32), (uint32_t)seed16,
                           (uint32_t)(seed16 >> 32), partials, np, q8_out, qp8_out, q16_out, qp16_out);
    else
        hipLaunchKernelGGL(quantize_bifurcate_apply<false>, dim3(grid), dim3(kThreads), 0, st, g, n,
                           (uint32_t)seed8, (uint32_t)(seed8 >> 32), (uint32_t)seed16,
                           (uint32_t)(seed16 >> 32), partials, np, q8_out, qp8_out, q16_out, qp16_out);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

}  // extern "C"

extern "C" {

int q8t_dequantize(const void *q, const q8t_qparams *qp, int64_t n, float *out, void *stream)
{
    if (n < 0 || n > kMaxElements) return Q8T_ERR_SHAPE;
    if (!qp || (n > 0 && (!q || !out))) return Q8T_ERR_NULL;
    if (n == 0) return Q8T_OK;
    hipLaunchKernelGGL(dequantize_kernel, dim3(grid_for(n, 4, 8192)), dim3(kThreads), 0,
                       (hipStream_t)stream, q, qp, n, out);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

}  // extern "C"
