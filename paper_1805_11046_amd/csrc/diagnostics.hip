// Two small reductions around the quantizer.
//
//  q8t_quant_angle   Sec. 5.1 (Problem Statement), eq. (1): cos(theta) = (x . Q(x)) / (||x|| ||Q(x)||) between a tensor and
//                    the dequantized value of its stored codes; the paper's measure of how well a
//                    quantizer preserves direction.  Three fp64 sums in one pass over x and q.
//  q8t_chunk_range   App. B: clamping range of an activation tensor as the average, over K
//                    contiguous chunks, of the chunk maxima and of the chunk minima.  The result
//                    feeds q8t_quantize_with_range (values outside it saturate).
#include "q8t_common.h"
#include "q8t_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kMaxAngleBlocks = 1024;
constexpr int64_t kMaxElements = (int64_t)1 << 34;

__device__ __forceinline__ double block_sum(double v, double *smem)
{
    v = wave_reduce(v, OpAddD());
    if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = smem[0];
    for (int w = 1; w < kThreads / 64; ++w) r += smem[w];
    __syncthreads();
    return r;
}

// pass 1: per-workgroup sums of x*xq, x*x, xq*xq over a contiguous slice
__global__ __launch_bounds__(kThreads) void angle_partials(const float *__restrict__ x, const void *__restrict__ q,
                                                           const q8t_qparams *__restrict__ qp, int64_t n,
                                                           double *__restrict__ part)
{
    __shared__ double smem[kThreads / 64];
    const int bits = qp->bits;
    const int shift = (1 << (bits - 1)) - qp->zero_point;   // stored code + shift = level - zero point
    const float scale = qp->scale;
    const int64_t per = (n + gridDim.x - 1) / gridDim.x;
    const int64_t lo = (int64_t)blockIdx.x * per, hi = min(n, lo + per);
    double dot = 0.0, nx = 0.0, nq = 0.0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kThreads) {
        const int s = bits <= 8 ? (int)((const int8_t *)q)[i] : (int)((const int16_t *)q)[i];
        const float xq = scale * (float)(s + shift);
        const double a = (double)x[i], b = (double)xq;
        dot += a * b;
        nx += a * a;
        nq += b * b;
    }
    dot = block_sum(dot, smem);
    nx = block_sum(nx, smem);
    nq = block_sum(nq, smem);
    if (threadIdx.x == 0) {
        part[3 * blockIdx.x] = dot;
        part[3 * blockIdx.x + 1] = nx;
        part[3 * blockIdx.x + 2] = nq;
    }
}

// pass 2 (one workgroup): fold the partial sums, out = { x.Q(x), |x|^2, |Q(x)|^2, cos(theta) }
__global__ __launch_bounds__(kThreads) void angle_finish(const double *__restrict__ part, int np, double *__restrict__ out)
{
    __shared__ double smem[kThreads / 64];
    double dot = 0.0, nx = 0.0, nq = 0.0;
    for (int i = threadIdx.x; i < np; i += kThreads) {
        dot += part[3 * i];
        nx += part[3 * i + 1];
        nq += part[3 * i + 2];
    }
    dot = block_sum(dot, smem);
    nx = block_sum(nx, smem);
    nq = block_sum(nq, smem);
    if (threadIdx.x == 0) {
        out[0] = dot;
        out[1] = nx;
        out[2] = nq;
        out[3] = (nx > 0.0 && nq > 0.0) ? dot / sqrt(nx * nq) : 0.0;
    }
}

// chunk k is [k*len, min(n, (k+1)*len)); grid (K, S): S workgroups share one chunk
__global__ __launch_bounds__(kThreads) void chunk_minmax(const float *__restrict__ x, int64_t n, int64_t len,
                                                         float2 *__restrict__ part)
{
    __shared__ float smn[kThreads / 64], smx[kThreads / 64];
    const int k = blockIdx.x, S = gridDim.y;
    const int64_t lo = (int64_t)k * len, hi = min(n, lo + len);
    const int64_t per = (len + S - 1) / S;
    const int64_t a = lo + (int64_t)blockIdx.y * per, b = min(hi, a + per);
    float mn = INFINITY, mx = -INFINITY;
    for (int64_t i = a + threadIdx.x; i < b; i += kThreads) {
        const float v = x[i];
        mn = fminf(mn, v);
        mx = fmaxf(mx, v);
    }
    mn = wave_reduce(mn, OpMin());
    mx = wave_reduce(mx, OpMax());
    if ((threadIdx.x & 63) == 0) {
        smn[threadIdx.x >> 6] = mn;
        smx[threadIdx.x >> 6] = mx;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kThreads / 64; ++w) {
            mn = fminf(mn, smn[w]);
            mx = fmaxf(mx, smx[w]);
        }
        part[(size_t)k * S + blockIdx.y] = make_float2(mn, mx);
    }
}

// The K chunk extrema are averaged in fp64 in chunk order by one lane (the order is part of the
// definition: the mean decides integer codes downstream, so it has to come out bit-identical).
__global__ __launch_bounds__(64) void chunk_average(const float2 *__restrict__ part, int K, int S, int64_t n, int64_t len,
                                                    float *__restrict__ range_out)
{
    if (threadIdx.x != 0) return;
    double smin = 0.0, smax = 0.0;
    int used = 0;
    for (int k = 0; k < K; ++k) {
        if ((int64_t)k * len >= n) break;   // chunks that would start past the end do not exist
        float mn = INFINITY, mx = -INFINITY;
        for (int s = 0; s < S; ++s) {
            const float2 p = part[(size_t)k * S + s];
            mn = fminf(mn, p.x);
            mx = fmaxf(mx, p.y);
        }
        smin += (double)mn;
        smax += (double)mx;
        ++used;
    }
    range_out[0] = (float)(smin / (double)used);
    range_out[1] = (float)(smax / (double)used);
}

int chunk_split(int64_t n, int K)
{
    const int64_t len = (n + K - 1) / K;
    int64_t S = (2048 + K - 1) / K;                       // about 2048 workgroups in total
    const int64_t most = (len + 4 * kThreads - 1) / (4 * kThreads);   // at least 1024 elements each
    if (S > most) S = most;
    if (S < 1) S = 1;
    if (S > 1024) S = 1024;
    return (int)S;
}

}  // namespace

extern "C" {

size_t q8t_quant_angle_workspace_size(int64_t n)
{
    (void)n;
    return (size_t)kMaxAngleBlocks * 3 * sizeof(double);
}

int q8t_quant_angle(const float *x, const void *q, const q8t_qparams *qp, int64_t n, double *out, void *ws, void *stream)
{
    if (n < 0 || n > kMaxElements) return Q8T_ERR_SHAPE;
    if (!qp || !out || (n > 0 && (!x || !q))) return Q8T_ERR_NULL;
    if (!ws || !q8t_aligned(ws, 8)) return Q8T_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    double *part = (double *)ws;
    int64_t blocks = (n + 4 * kThreads - 1) / (4 * kThreads);
    if (blocks > kMaxAngleBlocks) blocks = kMaxAngleBlocks;
    if (blocks > 0) {
        hipLaunchKernelGGL(angle_partials, dim3((unsigned)blocks), dim3(kThreads), 0, st, x, q, qp, n, part);
        Q8T_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(angle_finish, dim3(1), dim3(kThreads), 0, st, part, (int)blocks, out);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

size_t q8t_chunk_range_workspace_size(int64_t n, int K)
{
    if (n <= 0 || K <= 0 || K > n) return 0;
    return (size_t)K * chunk_split(n, K) * sizeof(float2);
}

int q8t_chunk_range(const float *x, int64_t n, int K, float *range_out, void *ws, void *stream)
{
    if (n <= 0 || n > kMaxElements || K <= 0 || K > n || K > 65535) return Q8T_ERR_SHAPE;
    if (!x || !range_out) return Q8T_ERR_NULL;
    if (!ws || !q8t_aligned(ws, 8)) return Q8T_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const int64_t len = (n + K - 1) / K;
    const int S = chunk_split(n, K);
    hipLaunchKernelGGL(chunk_minmax, dim3((unsigned)K, (unsigned)S), dim3(kThreads), 0, st, x, n, len, (float2 *)ws);
    Q8T_LAUNCH_CHECK();
    hipLaunchKernelGGL(chunk_average, dim3(1), dim3(64), 0, st, (const float2 *)ws, K, S, n, len, range_out);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

}  // extern "C"
