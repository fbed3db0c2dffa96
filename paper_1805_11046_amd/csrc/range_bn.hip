// Range Batch-Norm forward / backward over NCHW (Section 3, eq. (range); Section 7 for the
// derivative of max and min).  HBM-bound streaming kernels.
//
// forward : stats_partial (one coalesced pass: fp64 sum, min, max per channel slice)
//           -> finalize (per channel mean/min/max; optional per-tensor output range)
//           -> apply (normalize, optional fused 8-bit output)          12 B/element (9 with int8 out)
// backward: bwd_partial (fp64 sums of dy and dy*xhat) -> finalize (dgamma, dbeta, per-channel
//           constants) -> apply (dx)                                    20 B/element
// backward with the 8-bit / 16-bit stochastic copies of dx (gradient bifurcation, Sections 1, 4):
//           bwdq_partial (the same sums + extremes of dy per kind of coordinate, which fix the
//           range of dx) -> bwdq_finalize -> bwdq_apply (dx optional, codes written where dx is
//           computed)                                                   19 B/element (23 with dx)
// Every elementwise kernel takes an optional rectifier: Range BN followed by ReLU in one pass.
#include "q8t_common.h"
#include "q8t_internal.h"
#include "pool_gather.h"

namespace {

constexpr int kThreads = 256;
constexpr int kMaxSplit = 64;
constexpr int kApplyBlocks = 4096;   // workgroups of the second pass of the fused backward (16 per compute unit)

struct FwdPartial {
    double sum;
    float mn, mx;
};

__device__ __forceinline__ double block_sum_d(double v, double *smem)
{
    v = wave_reduce(v, OpAddD());
    if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = smem[0];
    for (int w = 1; w < kThreads / 64; ++w) r += smem[w];
    __syncthreads();
    return r;
}
__device__ __forceinline__ float block_min_f(float v, float *smem)
{
    v = wave_reduce(v, OpMin());
    if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = smem[0];
    for (int w = 1; w < kThreads / 64; ++w) r = fminf(r, smem[w]);
    __syncthreads();
    return r;
}
__device__ __forceinline__ float block_max_f(float v, float *smem)
{
    v = wave_reduce(v, OpMax());
    if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = smem[0];
    for (int w = 1; w < kThreads / 64; ++w) r = fmaxf(r, smem[w]);
    __syncthreads();
    return r;
}

// 1 / (C(n)*(max-min) + eps): one fp32 rounding per operation
__device__ __forceinline__ float bn_inv(float mn, float mx, float cn, float eps)
{
    const float range = mx - mn;
    const float scaled = cn * range;
    const float denom = scaled + eps;
    return 1.0f / denom;
}
// gamma * ((x - mu) * inv) + beta, no fused operations
__device__ __forceinline__ float bn_map(float x, float mu, float inv, float g, float b)
{
    const float cen = x - mu;
    const float xh = cen * inv;
    const float sc = xh * g;
    return sc + b;
}

// ---- forward, pass 1 --------------------------------------------------------------------------
// workgroup (c, sp) reduces images [sp*NB, (sp+1)*NB) of channel c
template <bool VEC>
__global__ __launch_bounds__(kThreads) void bn_stats_partial(const float *__restrict__ x, int N, int C,
                                                             int HW, int NB,
                                                             FwdPartial *__restrict__ parts)
{
    __shared__ double smd[kThreads / 64];
    __shared__ float smf[kThreads / 64];
    const int c = blockIdx.x, sp = blockIdx.y;
    const int b0 = sp * NB, b1 = min(N, b0 + NB);
    double sum = 0.0;
    float mn = INFINITY, mx = -INFINITY;
    if (VEC) {
        const int hw4 = HW >> 2;
        for (int b = b0; b < b1; ++b) {
            const float4 *p = reinterpret_cast<const float4 *>(x + ((int64_t)b * C + c) * HW);
#pragma unroll 4
            for (int i = threadIdx.x; i < hw4; i += kThreads) {
                const float4 v = q8t_ld_first(p + i);
                sum += (double)v.x;
                sum += (double)v.y;
                sum += (double)v.z;
                sum += (double)v.w;
                mn = fminf(fminf(mn, v.x), fminf(v.y, fminf(v.z, v.w)));
                mx = fmaxf(fmaxf(mx, v.x), fmaxf(v.y, fmaxf(v.z, v.w)));
            }
        }
    } else {
        const int cnt = (b1 - b0) * HW;
        for (int idx = threadIdx.x; idx < cnt; idx += kThreads) {
            const int b = b0 + idx / HW, i = idx % HW;
            const float v = x[((int64_t)b * C + c) * HW + i];
            sum += (double)v;
            mn = fminf(mn, v);
            mx = fmaxf(mx, v);
        }
    }
    sum = block_sum_d(sum, smd);
    mn = block_min_f(mn, smf);
    mx = block_max_f(mx, smf);
    if (threadIdx.x == 0) {
        FwdPartial r;
        r.sum = sum;
        r.mn = mn;
        r.mx = mx;
        parts[(int64_t)c * gridDim.y + sp] = r;
    }
}

// ---- forward, finalize (one workgroup) ----------------------------------------------------------
__global__ __launch_bounds__(kThreads) void bn_fwd_finalize(const FwdPartial *__restrict__ parts, int C,
                                                            int split, double n, float cn, float eps,
                                                            const float *__restrict__ gamma,
                                                            const float *__restrict__ beta,
                                                            float *__restrict__ stats,
                                                            q8t_qparams *__restrict__ qp_out)
{
    __shared__ float smf[kThreads / 64];
    float lo = INFINITY, hi = -INFINITY;
    for (int c = threadIdx.x; c < C; c += kThreads) {
        double s = 0.0;
        float mn = INFINITY, mx = -INFINITY;
        for (int k = 0; k < split; ++k) {
            const FwdPartial p = parts[(int64_t)c * split + k];
            s += p.sum;
            mn = fminf(mn, p.mn);
            mx = fmaxf(mx, p.mx);
        }
        const float mu = (float)(s / n);
        stats[c] = mu;
        stats[C + c] = mn;
        stats[2 * C + c] = mx;
        if (qp_out) {
            // images of the channel's extrema under the output map (monotone in x)
            const float g = gamma ? gamma[c] : 1.0f, b = beta ? beta[c] : 0.0f;
            const float inv = bn_inv(mn, mx, cn, eps);
            const float a = bn_map(mn, mu, inv, g, b), z = bn_map(mx, mu, inv, g, b);
            lo = fminf(lo, fminf(a, z));
            hi = fmaxf(hi, fmaxf(a, z));
        }
    }
    if (qp_out) {
        lo = block_min_f(lo, smf);
        hi = block_max_f(hi, smf);
        if (threadIdx.x == 0) *qp_out = make_qparams(lo, hi, 8);
    }
}

// per-tensor range of the 8-bit output from ready-made statistics (one workgroup)
__global__ __launch_bounds__(kThreads) void bn_qrange_from_stats(const float *__restrict__ stats, int C, float cn, float eps,
                                                                 const float *__restrict__ gamma,
                                                                 const float *__restrict__ beta, int relu,
                                                                 q8t_qparams *__restrict__ qp_out)
{
    __shared__ float smf[kThreads / 64];
    float lo = INFINITY, hi = -INFINITY;
    for (int c = threadIdx.x; c < C; c += kThreads) {
        const float mu = stats[c], mn = stats[C + c], mx = stats[2 * C + c];
        const float g = gamma ? gamma[c] : 1.0f, b = beta ? beta[c] : 0.0f;
        const float inv = bn_inv(mn, mx, cn, eps);
        const float a = bn_map(mn, mu, inv, g, b), z = bn_map(mx, mu, inv, g, b);
        lo = fminf(lo, fminf(a, z));
        hi = fmaxf(hi, fmaxf(a, z));
    }
    lo = block_min_f(lo, smf);
    hi = block_max_f(hi, smf);
    if (relu) {   // the rectified output spans the rectified images of the extrema
        lo = lo > 0.0f ? lo : 0.0f;
        hi = hi > 0.0f ? hi : 0.0f;
    }
    if (threadIdx.x == 0) *qp_out = make_qparams(lo, hi, 8);
}

// ---- forward, pass 2 ----------------------------------------------------------------------------
// one (image, channel) plane per workgroup iteration
// fold the slices of one channel inside a wavefront (lane k holds slice k; fixed butterfly order,
// so every workgroup of the channel obtains bit-identical statistics)
__device__ __forceinline__ void fold_fwd_parts(const FwdPartial *__restrict__ parts, int c, int split, double n,
                                               float &mu, float &mn, float &mx)
{
    const int lane = threadIdx.x & 63;
    double s = 0.0;
    float a = INFINITY, b = -INFINITY;
    if (lane < split) {
        const FwdPartial p = parts[(int64_t)c * split + lane];
        s = p.sum;
        a = p.mn;
        b = p.mx;
    }
    s = wave_reduce(s, OpAddD());
    mn = wave_reduce(a, OpMin());
    mx = wave_reduce(b, OpMax());
    mu = (float)(s / n);
}

// With `parts` != NULL the statistics are folded here from the slices of pass 1 (and written to
// `stats` by the workgroups of image 0), which saves the separate finalize launch.
template <bool VEC, bool QOUT>
__global__ __launch_bounds__(kThreads) void bn_fwd_apply(const float *__restrict__ x, int64_t planes,
                                                         int C, int HW, float *__restrict__ stats,
                                                         const FwdPartial *__restrict__ parts, int split,
                                                         double n,
                                                         const float *__restrict__ gamma,
                                                         const float *__restrict__ beta, float cn,
                                                         float eps, float *__restrict__ y,
                                                         int8_t *__restrict__ q,
                                                         const q8t_qparams *__restrict__ qp, int relu, int flat4)
{
    Affine a;
    if (QOUT) a = affine_of(*qp);
    if (VEC && flat4) {
        // small planes, statistics given: one float4 per thread over the flat tensor
        const int hw4 = HW >> 2;
        const int64_t total4 = planes * hw4, stride = (int64_t)gridDim.x * kThreads;
        for (int64_t i4 = (int64_t)blockIdx.x * kThreads + threadIdx.x; i4 < total4; i4 += stride) {
            const int c = (int)((i4 / hw4) % C);
            const float mu = stats[c];
            const float inv = bn_inv(stats[C + c], stats[2 * C + c], cn, eps);
            const float g = gamma ? gamma[c] : 1.0f, b = beta ? beta[c] : 0.0f;
            const float4 v = q8t_ld_last(reinterpret_cast<const float4 *>(x) + i4);
            float4 r;
            r.x = bn_map(v.x, mu, inv, g, b);
            r.y = bn_map(v.y, mu, inv, g, b);
            r.z = bn_map(v.z, mu, inv, g, b);
            r.w = bn_map(v.w, mu, inv, g, b);
            if (relu) {
                r.x = r.x > 0.0f ? r.x : 0.0f;
                r.y = r.y > 0.0f ? r.y : 0.0f;
                r.z = r.z > 0.0f ? r.z : 0.0f;
                r.w = r.w > 0.0f ? r.w : 0.0f;
            }
            if (y) reinterpret_cast<float4 *>(y)[i4] = r;
            if (QOUT) {
                const int q0 = level_of<false>(r.x, a, 0) - 128, q1 = level_of<false>(r.y, a, 0) - 128,
                          q2 = level_of<false>(r.z, a, 0) - 128, q3 = level_of<false>(r.w, a, 0) - 128;
                reinterpret_cast<uint32_t *>(q)[i4] = (uint32_t)(q0 & 255) | ((uint32_t)(q1 & 255) << 8) |
                                                      ((uint32_t)(q2 & 255) << 16) | ((uint32_t)(q3 & 255) << 24);
            }
        }
        return;
    }
    for (int64_t pl = blockIdx.x; pl < planes; pl += gridDim.x) {
        const int c = (int)(pl % C);
        float mu, cmn, cmx;
        if (parts) {
            fold_fwd_parts(parts, c, split, n, mu, cmn, cmx);   // every wavefront folds the same slices
            if (pl < C && threadIdx.x == 0) {
                stats[c] = mu;
                stats[C + c] = cmn;
                stats[2 * C + c] = cmx;
            }
        } else {
            mu = stats[c];
            cmn = stats[C + c];
            cmx = stats[2 * C + c];
        }
        const float inv = bn_inv(cmn, cmx, cn, eps);
        const float g = gamma ? gamma[c] : 1.0f, b = beta ? beta[c] : 0.0f;
        const int64_t base = pl * HW;
        if (VEC) {
            const float4 *p = reinterpret_cast<const float4 *>(x + base);
            float4 *o = reinterpret_cast<float4 *>(y + base);
            uint32_t *oq = reinterpret_cast<uint32_t *>(q + base);
            const int hw4 = HW >> 2;
#pragma unroll 4
            for (int i = threadIdx.x; i < hw4; i += kThreads) {
                const float4 v = q8t_ld_last(p + i);
                float4 r;
                r.x = bn_map(v.x, mu, inv, g, b);
                r.y = bn_map(v.y, mu, inv, g, b);
                r.z = bn_map(v.z, mu, inv, g, b);
                r.w = bn_map(v.w, mu, inv, g, b);
                if (relu) {
                    r.x = r.x > 0.0f ? r.x : 0.0f;
                    r.y = r.y > 0.0f ? r.y : 0.0f;
                    r.z = r.z > 0.0f ? r.z : 0.0f;
                    r.w = r.w > 0.0f ? r.w : 0.0f;
                }
                if (y) o[i] = r;
                if (QOUT) {
                    const int q0 = level_of<false>(r.x, a, 0) - 128, q1 = level_of<false>(r.y, a, 0) - 128,
                              q2 = level_of<false>(r.z, a, 0) - 128, q3 = level_of<false>(r.w, a, 0) - 128;
                    oq[i] = (uint32_t)(q0 & 255) | ((uint32_t)(q1 & 255) << 8) |
                            ((uint32_t)(q2 & 255) << 16) | ((uint32_t)(q3 & 255) << 24);
                }
            }
        } else {
            for (int i = threadIdx.x; i < HW; i += kThreads) {
                float r = bn_map(x[base + i], mu, inv, g, b);
                if (relu) r = r > 0.0f ? r : 0.0f;
                if (y) y[base + i] = r;
                if (QOUT) q[base + i] = (int8_t)(level_of<false>(r, a, 0) - 128);
            }
        }
    }
}

// small planes: one thread per element
template <bool QOUT>
__global__ __launch_bounds__(kThreads) void bn_fwd_apply_flat(const float *__restrict__ x, int64_t total,
                                                              int C, int HW,
                                                              const float *__restrict__ stats,
                                                              const float *__restrict__ gamma,
                                                              const float *__restrict__ beta, float cn,
                                                              float eps, float *__restrict__ y,
                                                              int8_t *__restrict__ q,
                                                              const q8t_qparams *__restrict__ qp, int relu)
{
    Affine a;
    if (QOUT) a = affine_of(*qp);
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
        const int c = (int)((i / HW) % C);
        const float inv = bn_inv(stats[C + c], stats[2 * C + c], cn, eps);
        float r = bn_map(x[i], stats[c], inv, gamma ? gamma[c] : 1.0f, beta ? beta[c] : 0.0f);
        if (relu) r = r > 0.0f ? r : 0.0f;
        if (y) y[i] = r;
        if (QOUT) q[i] = (int8_t)(level_of<false>(r, a, 0) - 128);
    }
}

// ---- backward, pass 1 ---------------------------------------------------------------------------
template <bool VEC>
__global__ __launch_bounds__(kThreads) void bn_bwd_partial(const float *__restrict__ x,
                                                           const float *__restrict__ dy,
                                                           const float *__restrict__ stats, int N, int C,
                                                           int HW, int NB, float cn, float eps,
                                                           const float *__restrict__ gamma,
                                                           const float *__restrict__ beta, int relu,
                                                           double2 *__restrict__ parts)
{
    __shared__ double smd[kThreads / 64];
    const int c = blockIdx.x, sp = blockIdx.y;
    const int b0 = sp * NB, b1 = min(N, b0 + NB);
    const float mu = stats[c];
    const float inv = bn_inv(stats[C + c], stats[2 * C + c], cn, eps);
    const float ga = gamma ? gamma[c] : 1.0f, be = beta ? beta[c] : 0.0f;
    double s0 = 0.0, s1 = 0.0;
    if (VEC) {
        const int hw4 = HW >> 2;
        for (int b = b0; b < b1; ++b) {
            const int64_t base = ((int64_t)b * C + c) * HW;
            const float4 *px = reinterpret_cast<const float4 *>(x + base);
            const float4 *pg = reinterpret_cast<const float4 *>(dy + base);
#pragma unroll 2
            for (int i = threadIdx.x; i < hw4; i += kThreads) {
                const float4 v = q8t_ld_first(px + i);
                float4 g = q8t_ld_first(pg + i);
                const float h0 = (v.x - mu) * inv, h1 = (v.y - mu) * inv, h2 = (v.z - mu) * inv,
                            h3 = (v.w - mu) * inv;
                if (relu) {   // the gradient passes where the forward output was positive
                    g.x = bn_map(v.x, mu, inv, ga, be) > 0.0f ? g.x : 0.0f;
                    g.y = bn_map(v.y, mu, inv, ga, be) > 0.0f ? g.y : 0.0f;
                    g.z = bn_map(v.z, mu, inv, ga, be) > 0.0f ? g.z : 0.0f;
                    g.w = bn_map(v.w, mu, inv, ga, be) > 0.0f ? g.w : 0.0f;
                }
                s0 += (double)g.x;
                s0 += (double)g.y;
                s0 += (double)g.z;
                s0 += (double)g.w;
                s1 += (double)g.x * (double)h0;
                s1 += (double)g.y * (double)h1;
                s1 += (double)g.z * (double)h2;
                s1 += (double)g.w * (double)h3;
            }
        }
    } else {
        const int cnt = (b1 - b0) * HW;
        for (int idx = threadIdx.x; idx < cnt; idx += kThreads) {
            const int b = b0 + idx / HW, i = idx % HW;
            const int64_t j = ((int64_t)b * C + c) * HW + i;
            const float h = (x[j] - mu) * inv;
            const float d = relu && !(bn_map(x[j], mu, inv, ga, be) > 0.0f) ? 0.0f : dy[j];
            s0 += (double)d;
            s1 += (double)d * (double)h;
        }
    }
    s0 = block_sum_d(s0, smd);
    s1 = block_sum_d(s1, smd);
    if (threadIdx.x == 0) parts[(int64_t)c * gridDim.y + sp] = make_double2(s0, s1);
}

__global__ __launch_bounds__(kThreads) void bn_bwd_finalize(const double2 *__restrict__ parts, int C,
                                                            int split, double n, float cn, float eps,
                                                            const float *__restrict__ stats,
                                                            const float *__restrict__ gamma,
                                                            float *__restrict__ dgamma,
                                                            float *__restrict__ dbeta,
                                                            float2 *__restrict__ consts)
{
    const int c = blockIdx.x * kThreads + threadIdx.x;
    if (c >= C) return;
    double s0 = 0.0, s1 = 0.0;
    for (int k = 0; k < split; ++k) {
        const double2 p = parts[(int64_t)c * split + k];
        s0 += p.x;
        s1 += p.y;
    }
    if (dbeta) dbeta[c] = (float)s0;
    if (dgamma) dgamma[c] = (float)s1;
    const float g = gamma ? gamma[c] : 1.0f;
    const float inv = bn_inv(stats[C + c], stats[2 * C + c], cn, eps);
    const double A = (double)g * s0, B = (double)g * s1;
    const float mean_g = (float)(A / n);
    const float kb = (float)((double)inv * (double)cn * B);
    consts[c] = make_float2(mean_g, kb);
}

// dx_j = inv*(gamma*dy_j - mean_g) -/+ kb at the coordinates that attain max / min
__device__ __forceinline__ float bn_dx(float xv, float dyv, float g, float mean_g, float inv, float kb,
                                       float mn, float mx)
{
    const float gh = g * dyv;
    const float t = gh - mean_g;
    float v = inv * t;
    if (xv == mx) v = v - kb;
    if (xv == mn) v = v + kb;
    return v;
}

// With `parts` != NULL the per-channel sums are folded here (fixed butterfly order inside a
// wavefront) and dgamma / dbeta are written by the workgroups of image 0: no finalize launch.
template <bool VEC>
__global__ __launch_bounds__(kThreads) void bn_bwd_apply(const float *__restrict__ x,
                                                         const float *__restrict__ dy, int64_t planes,
                                                         int C, int HW, const float *__restrict__ stats,
                                                         const float *__restrict__ gamma,
                                                         const float2 *__restrict__ consts,
                                                         const double2 *__restrict__ parts, int split, double n,
                                                         float *__restrict__ dgamma, float *__restrict__ dbeta,
                                                         float cn, float eps, float *__restrict__ dx,
                                                         const float *__restrict__ beta, int relu)
{
    for (int64_t pl = blockIdx.x; pl < planes; pl += gridDim.x) {
        const int c = (int)(pl % C);
        const float mn = stats[C + c], mx = stats[2 * C + c];
        const float inv = bn_inv(mn, mx, cn, eps);
        const float g = gamma ? gamma[c] : 1.0f;
        const float mu = stats[c], be = beta ? beta[c] : 0.0f;
        float2 k;
        if (parts) {
            const int lane = threadIdx.x & 63;
            double s0 = 0.0, s1 = 0.0;
            if (lane < split) {
                const double2 p = parts[(int64_t)c * split + lane];
                s0 = p.x;
                s1 = p.y;
            }
            s0 = wave_reduce(s0, OpAddD());
            s1 = wave_reduce(s1, OpAddD());
            if (pl < C && threadIdx.x == 0) {
                if (dbeta) dbeta[c] = (float)s0;
                if (dgamma) dgamma[c] = (float)s1;
            }
            const double A = (double)g * s0, B = (double)g * s1;
            k = make_float2((float)(A / n), (float)((double)inv * (double)cn * B));
        } else {
            k = consts[c];
        }
        const int64_t base = pl * HW;
        if (VEC) {
            const float4 *px = reinterpret_cast<const float4 *>(x + base);
            const float4 *pg = reinterpret_cast<const float4 *>(dy + base);
            float4 *o = reinterpret_cast<float4 *>(dx + base);
            const int hw4 = HW >> 2;
#pragma unroll 2
            for (int i = threadIdx.x; i < hw4; i += kThreads) {
                const float4 v = q8t_ld_last(px + i);
                float4 d = q8t_ld_last(pg + i);
                if (relu) {
                    d.x = bn_map(v.x, mu, inv, g, be) > 0.0f ? d.x : 0.0f;
                    d.y = bn_map(v.y, mu, inv, g, be) > 0.0f ? d.y : 0.0f;
                    d.z = bn_map(v.z, mu, inv, g, be) > 0.0f ? d.z : 0.0f;
                    d.w = bn_map(v.w, mu, inv, g, be) > 0.0f ? d.w : 0.0f;
                }
                float4 r;
                r.x = bn_dx(v.x, d.x, g, k.x, inv, k.y, mn, mx);
                r.y = bn_dx(v.y, d.y, g, k.x, inv, k.y, mn, mx);
                r.z = bn_dx(v.z, d.z, g, k.x, inv, k.y, mn, mx);
                r.w = bn_dx(v.w, d.w, g, k.x, inv, k.y, mn, mx);
                o[i] = r;
            }
        } else {
            for (int i = threadIdx.x; i < HW; i += kThreads) {
                const float xv = x[base + i];
                const float d = relu && !(bn_map(xv, mu, inv, g, be) > 0.0f) ? 0.0f : dy[base + i];
                const float r = bn_dx(xv, d, g, k.x, inv, k.y, mn, mx);
                dx[base + i] = r;
            }
        }
    }
}

__global__ __launch_bounds__(kThreads) void bn_bwd_apply_flat(const float *__restrict__ x,
                                                              const float *__restrict__ dy, int64_t total,
                                                              int C, int HW,
                                                              const float *__restrict__ stats,
                                                              const float *__restrict__ gamma,
                                                              const float2 *__restrict__ consts, float cn,
                                                              float eps, float *__restrict__ dx,
                                                              const float *__restrict__ beta, int relu)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
        const int c = (int)((i / HW) % C);
        const float mn = stats[C + c], mx = stats[2 * C + c];
        const float2 k = consts[c];
        const float g = gamma ? gamma[c] : 1.0f, inv = bn_inv(mn, mx, cn, eps);
        const float d = relu && !(bn_map(x[i], stats[c], inv, g, beta ? beta[c] : 0.0f) > 0.0f) ? 0.0f : dy[i];
        dx[i] = bn_dx(x[i], d, g, k.x, inv, k.y, mn, mx);
    }
}

// ---- backward with its 8-bit / 16-bit copies, two passes -------------------------------------------
// dx is an affine, monotone function of dy inside a channel (v = inv*(gamma*dy - mean_g); every fp32
// step is monotone), except at the coordinates that attain the channel's max / min, which get -/+ kb.
// So the range of dx follows from the extremes of dy per channel, kept apart for the four kinds of
// coordinate (ordinary, at the max, at the min, at both), and pass 1 can collect those beside its
// sums: no pass over dx is needed to find the quantizer's range, and dx itself need not be written
// at all.  8 + 8 + 3 bytes per element (+4 with dx) instead of 27.
struct BwdPartialQ {
    double s0, s1;
    float lo[4], hi[4];   // extremes of (masked) dy: ordinary, at max, at min, at both
};

// Pass 2 does not have to read x again: an ordinary coordinate's dx depends on x only through the rectifier's
// mask, which pass 1 leaves behind as one byte per four coordinates, and the few coordinates that attain the
// channel's max or min are listed by pass 1 and patched by a small kernel afterwards.  A workgroup of pass 1
// that meets more than kExtCap of them marks its channel as crowded, and pass 2 handles that channel the old way.
constexpr int kExtCap = 7;
struct ExtList {
    int cnt, pad;
    int b[kExtCap], pos[kExtCap];   // image, position inside the plane
};

// POOL: the upstream gradient is not a tensor in memory but the backward of the stem's 3x3 / stride 2 max pooling,
// gathered from the pooled gradient and the window indices (one pooled plane at a time staged in LDS); planes of at
// least 4 * kThreads positions with a width that is a multiple of 4.
struct PoolSrc {
    const float *g;
    const uint8_t *idx;
    int W4, P, Q;    // float4 groups per row of the unpooled plane, pooled plane
    float rw4;       // 1 / W4
};
__device__ __forceinline__ float4 pool_grad4(const PoolSrc &ps, const uint8_t *lds, int i)
{
    const int h = q8t_pool::small_div(i, ps.W4, ps.rw4), qa = 2 * (i - h * ps.W4);
    return q8t_pool::bwd_gather4(reinterpret_cast<const float *>(lds), lds + (size_t)ps.P * ps.Q * sizeof(float), h, qa, ps.P,
                                 ps.Q);
}

template <bool VEC, bool POOL = false>
__global__ __launch_bounds__(kThreads) void bn_bwdq_partial(const float *__restrict__ x, const float *__restrict__ dy,
                                                            const float *__restrict__ stats, int N, int C, int HW, int NB,
                                                            float cn, float eps, const float *__restrict__ gamma,
                                                            const float *__restrict__ beta, int relu,
                                                            BwdPartialQ *__restrict__ parts, ExtList *__restrict__ lists,
                                                            uint8_t *__restrict__ flags, const PoolSrc pool)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t pool_lds[];
    __shared__ double smd[kThreads / 64];
    __shared__ float smf[kThreads / 64];
    __shared__ int ext_cnt, ext_b[kExtCap], ext_pos[kExtCap];
    if (threadIdx.x == 0) ext_cnt = 0;
    __syncthreads();
    const int c = blockIdx.x, sp = blockIdx.y;
    const int b0 = sp * NB, b1 = min(N, b0 + NB);
    const float mu = stats[c], mn = stats[C + c], mx = stats[2 * C + c];
    const float inv = bn_inv(mn, mx, cn, eps);
    const float ga = gamma ? gamma[c] : 1.0f, be = beta ? beta[c] : 0.0f;
    double s0 = 0.0, s1 = 0.0;
    float lo[4] = {INFINITY, INFINITY, INFINITY, INFINITY}, hi[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    auto one = [&](float xv, float d, int b, int pos) -> uint32_t {   // returns 1 if the rectifier passes the gradient
        uint32_t pass = 1;
        if (relu) {
            pass = bn_map(xv, mu, inv, ga, be) > 0.0f ? 1u : 0u;
            d = pass ? d : 0.0f;
        }
        const float h = (xv - mu) * inv;
        s0 += (double)d;
        s1 += (double)d * (double)h;
        if (xv == mx || xv == mn) {   // a few coordinates per channel
            if (lists) {
                const int slot = atomicAdd(&ext_cnt, 1);
                if (slot < kExtCap) {
                    ext_b[slot] = b;
                    ext_pos[slot] = pos;
                }
            }
            const int k = (xv == mx ? 1 : 0) + (xv == mn ? 2 : 0);
#pragma unroll
            for (int q = 1; q < 4; ++q)
                if (k == q) {
                    lo[q] = fminf(lo[q], d);
                    hi[q] = fmaxf(hi[q], d);
                }
        } else {
            lo[0] = fminf(lo[0], d);
            hi[0] = fmaxf(hi[0], d);
        }
        return pass;
    };
    if (VEC) {
        const int hw4 = HW >> 2;
        if (hw4 >= kThreads) {
            for (int b = b0; b < b1; ++b) {
                const int64_t base = ((int64_t)b * C + c) * HW;
                const float4 *px = reinterpret_cast<const float4 *>(x + base);
                const float4 *pg = reinterpret_cast<const float4 *>(dy + base);
                if (POOL) {
                    __syncthreads();   // the gather of the previous plane is over
                    const int64_t pp = ((int64_t)b * C + c) * (pool.P * pool.Q);
                    q8t_pool::stage_plane<kThreads>(pool.g + pp, pool.idx + pp, pool.P * pool.Q, pool_lds);
                    __syncthreads();
                }
#pragma unroll 2
                for (int i = threadIdx.x; i < hw4; i += kThreads) {
                    const float4 v = q8t_ld_first(px + i);
                    const float4 g = POOL ? pool_grad4(pool, pool_lds, i) : q8t_ld_first(pg + i);
                    const uint32_t m = one(v.x, g.x, b, 4 * i) | (one(v.y, g.y, b, 4 * i + 1) << 1) |
                                       (one(v.z, g.z, b, 4 * i + 2) << 2) | (one(v.w, g.w, b, 4 * i + 3) << 3);
                    if (flags) flags[(base >> 2) + i] = (uint8_t)m;
                }
            }
        } else {
            // planes smaller than a sweep of the workgroup: one loop over (image, float4) keeps the lanes busy
            const int items = (b1 - b0) * hw4;
#pragma unroll 2
            for (int idx = threadIdx.x; idx < items; idx += kThreads) {
                const int bl = idx / hw4, i = idx - bl * hw4;
                const int64_t base = ((int64_t)(b0 + bl) * C + c) * HW;
                const float4 v = q8t_ld_first(reinterpret_cast<const float4 *>(x + base) + i);
                const float4 g = q8t_ld_first(reinterpret_cast<const float4 *>(dy + base) + i);
                const uint32_t m = one(v.x, g.x, b0 + bl, 4 * i) | (one(v.y, g.y, b0 + bl, 4 * i + 1) << 1) |
                                   (one(v.z, g.z, b0 + bl, 4 * i + 2) << 2) | (one(v.w, g.w, b0 + bl, 4 * i + 3) << 3);
                if (flags) flags[(base >> 2) + i] = (uint8_t)m;
            }
        }
    } else {
        const int cnt = (b1 - b0) * HW;
        for (int idx = threadIdx.x; idx < cnt; idx += kThreads) {
            const int b = b0 + idx / HW, i = idx % HW;
            const int64_t j = ((int64_t)b * C + c) * HW + i;
            one(x[j], dy[j], b, i);
        }
    }
    BwdPartialQ r;
    r.s0 = block_sum_d(s0, smd);
    r.s1 = block_sum_d(s1, smd);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        r.lo[q] = block_min_f(lo[q], smf);
        r.hi[q] = block_max_f(hi[q], smf);
    }
    if (threadIdx.x == 0) parts[(int64_t)c * gridDim.y + sp] = r;
    if (lists) {
        __syncthreads();
        ExtList *l = lists + (int64_t)c * gridDim.y + sp;
        if (threadIdx.x == 0) l->cnt = ext_cnt;
        if (threadIdx.x < kExtCap && threadIdx.x < ext_cnt) {
            l->b[threadIdx.x] = ext_b[threadIdx.x];
            l->pos[threadIdx.x] = ext_pos[threadIdx.x];
        }
    }
}

// dx of one coordinate of kind k (bit 0: at the max, bit 1: at the min), same operations as bn_dx
__device__ __forceinline__ float bn_dx_kind(float dyv, float g, float mean_g, float inv, float kb, int k)
{
    const float gh = g * dyv;
    const float t = gh - mean_g;
    float v = inv * t;
    if (k & 1) v = v - kb;
    if (k & 2) v = v + kb;
    return v;
}

// per-channel sums -> dgamma, dbeta, constants, and the range of dx over the workgroup's channels
// (one channel per wavefront; pass 2 folds the workgroups' ranges).  A wavefront folds the slices of
// a channel in the butterfly order of bn_bwd_apply (lane k holds slice k), so the constants are
// bit-identical to that path.
__global__ __launch_bounds__(kThreads) void bn_bwdq_finalize(const BwdPartialQ *__restrict__ parts, int C, int split, double n,
                                                             float cn, float eps, const float *__restrict__ stats,
                                                             const float *__restrict__ gamma, float *__restrict__ dgamma,
                                                             float *__restrict__ dbeta, float2 *__restrict__ consts,
                                                             float2 *__restrict__ mm, const ExtList *__restrict__ lists,
                                                             int *__restrict__ crowded)
{
    __shared__ float smf[kThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float dmn = INFINITY, dmx = -INFINITY;
    const int c = blockIdx.x * (kThreads / 64) + wave;
    if (c < C && lists) {
        const int over = lane < split && lists[(int64_t)c * split + lane].cnt > kExtCap;
        const unsigned long long any = __ballot(over);
        if (lane == 0) crowded[c] = any != 0ull;
    }
    if (c < C) {
        double s0 = 0.0, s1 = 0.0;
        float lo[4] = {INFINITY, INFINITY, INFINITY, INFINITY}, hi[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        if (lane < split) {
            const BwdPartialQ p = parts[(int64_t)c * split + lane];
            s0 = p.s0;
            s1 = p.s1;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                lo[q] = p.lo[q];
                hi[q] = p.hi[q];
            }
        }
        s0 = wave_reduce(s0, OpAddD());
        s1 = wave_reduce(s1, OpAddD());
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            lo[q] = wave_reduce(lo[q], OpMin());
            hi[q] = wave_reduce(hi[q], OpMax());
        }
        const float g = gamma ? gamma[c] : 1.0f;
        const float inv = bn_inv(stats[C + c], stats[2 * C + c], cn, eps);
        const double A = (double)g * s0, B = (double)g * s1;
        const float mean_g = (float)(A / n);
        const float kb = (float)((double)inv * (double)cn * B);
        if (lane == 0) {
            if (dbeta) dbeta[c] = (float)s0;
            if (dgamma) dgamma[c] = (float)s1;
            consts[c] = make_float2(mean_g, kb);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (lo[q] > hi[q]) continue;   // no coordinate of this kind
            const float a = bn_dx_kind(lo[q], g, mean_g, inv, kb, q), b = bn_dx_kind(hi[q], g, mean_g, inv, kb, q);
            dmn = fminf(dmn, fminf(a, b));
            dmx = fmaxf(dmx, fmaxf(a, b));
        }
    }
    dmn = block_min_f(dmn, smf);
    dmx = block_max_f(dmx, smf);
    if (threadIdx.x == 0) mm[blockIdx.x] = make_float2(dmn, dmx);
}

// pass 2: dx (optional) and its two stochastic copies
template <bool VEC, bool POOL = false>
__global__ __launch_bounds__(kThreads) void bn_bwdq_apply(const float *__restrict__ x, const float *__restrict__ dy,
                                                          int64_t planes, int C, int HW, const float *__restrict__ stats,
                                                          const float *__restrict__ gamma, const float *__restrict__ beta,
                                                          int relu, const float2 *__restrict__ consts, float cn, float eps,
                                                          uint32_t s8_lo, uint32_t s8_hi, uint32_t s16_lo, uint32_t s16_hi,
                                                          const float2 *__restrict__ mm, int nmm,
                                                          q8t_qparams *__restrict__ qp8_out,
                                                          q8t_qparams *__restrict__ qp16_out, float *__restrict__ dx,
                                                          int8_t *__restrict__ q8, int16_t *__restrict__ q16,
                                                          const int *__restrict__ crowded, const uint8_t *__restrict__ flags,
                                                          const PoolSrc pool)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t pool_lds[];
    // q8 == NULL: the 16-bit copy alone (a layer whose input needs no gradient)
    // crowded != NULL: x is read only for channels marked there; elsewhere every coordinate is treated as an
    // ordinary one (mask from `flags` under the rectifier) and bn_bwdq_fixup rewrites the listed ones afterwards
    // every workgroup folds the ranges of pass 1 (min / max: any order gives the same bits)
    __shared__ float smf[kThreads / 64];
    float vmin = INFINITY, vmax = -INFINITY;
    for (int i = threadIdx.x; i < nmm; i += kThreads) {
        const float2 p = mm[i];
        vmin = fminf(vmin, p.x);
        vmax = fmaxf(vmax, p.y);
    }
    vmin = block_min_f(vmin, smf);
    vmax = block_max_f(vmax, smf);
    const q8t_qparams qp8 = make_qparams(vmin, vmax, 8), qp16 = make_qparams(vmin, vmax, 16);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (qp8_out) *qp8_out = qp8;
        *qp16_out = qp16;
    }
    const Affine a8 = affine_of(qp8), a16 = affine_of(qp16);
    if (VEC && HW < 4 * kThreads) {
        // small planes: one float4 per thread over the flat tensor (a float4 never leaves its plane)
        // The channel of a float4: the 64-bit division is done once per workgroup and sweep, on the index of the
        // workgroup's first float4; a thread is at most kThreads float4s past it, which a float reciprocal
        // resolves (as a 64-bit division and a modulo per thread this lookup cost as much as half the rounding work).
        const int hw4 = HW >> 2;
        const float rhw4 = 1.0f / (float)hw4, rC = 1.0f / (float)C;
        const int64_t total4 = planes * hw4, stride = (int64_t)gridDim.x * kThreads;
        for (int64_t b4 = (int64_t)blockIdx.x * kThreads; b4 < total4; b4 += stride) {
            const int64_t pl0 = b4 / hw4;                         // uniform in the workgroup
            const int rem0 = (int)(b4 - pl0 * hw4), c0 = (int)(pl0 % C);
            const int64_t i4 = b4 + threadIdx.x;
            if (i4 >= total4) continue;
            const int cc = c0 + q8t_pool::small_div(rem0 + (int)threadIdx.x, hw4, rhw4);   // < C + kThreads + 1
            const int c = cc - q8t_pool::small_div(cc, C, rC) * C;
            const float mu = stats[c], mn = stats[C + c], mx = stats[2 * C + c];
            const float inv = bn_inv(mn, mx, cn, eps);
            const float g = gamma ? gamma[c] : 1.0f, be = beta ? beta[c] : 0.0f;
            const float2 k = consts[c];
            float4 d = q8t_ld_last(reinterpret_cast<const float4 *>(dy) + i4);
            float4 r;
            if (crowded && !crowded[c]) {
                if (relu) {
                    const uint32_t m = flags[i4];
                    d.x = (m & 1u) ? d.x : 0.0f;
                    d.y = (m & 2u) ? d.y : 0.0f;
                    d.z = (m & 4u) ? d.z : 0.0f;
                    d.w = (m & 8u) ? d.w : 0.0f;
                }
                r.x = bn_dx_kind(d.x, g, k.x, inv, k.y, 0);
                r.y = bn_dx_kind(d.y, g, k.x, inv, k.y, 0);
                r.z = bn_dx_kind(d.z, g, k.x, inv, k.y, 0);
                r.w = bn_dx_kind(d.w, g, k.x, inv, k.y, 0);
            } else {
                const float4 v = q8t_ld_last(reinterpret_cast<const float4 *>(x) + i4);
                if (relu) {
                    d.x = bn_map(v.x, mu, inv, g, be) > 0.0f ? d.x : 0.0f;
                    d.y = bn_map(v.y, mu, inv, g, be) > 0.0f ? d.y : 0.0f;
                    d.z = bn_map(v.z, mu, inv, g, be) > 0.0f ? d.z : 0.0f;
                    d.w = bn_map(v.w, mu, inv, g, be) > 0.0f ? d.w : 0.0f;
                }
                r.x = bn_dx(v.x, d.x, g, k.x, inv, k.y, mn, mx);
                r.y = bn_dx(v.y, d.y, g, k.x, inv, k.y, mn, mx);
                r.z = bn_dx(v.z, d.z, g, k.x, inv, k.y, mn, mx);
                r.w = bn_dx(v.w, d.w, g, k.x, inv, k.y, mn, mx);
            }
            if (dx) reinterpret_cast<float4 *>(dx)[i4] = r;
            if (q8) reinterpret_cast<uint32_t *>(q8)[i4] = quant4<int8_t, true>(r, a8, (uint32_t)i4, s8_lo, s8_hi);
            reinterpret_cast<uint2 *>(q16)[i4] = quant4<int16_t, true>(r, a16, (uint32_t)i4, s16_lo, s16_hi);
        }
    } else if (VEC) {
        for (int64_t pl = blockIdx.x; pl < planes; pl += gridDim.x) {
            const int c = (int)(pl % C);
            const float mu = stats[c], mn = stats[C + c], mx = stats[2 * C + c];
            const float inv = bn_inv(mn, mx, cn, eps);
            const float g = gamma ? gamma[c] : 1.0f, be = beta ? beta[c] : 0.0f;
            const float2 k = consts[c];
            const int64_t base = pl * HW;
            const float4 *px = reinterpret_cast<const float4 *>(x + base);
            const float4 *pg = reinterpret_cast<const float4 *>(dy + base);
            float4 *o = reinterpret_cast<float4 *>(dx + base);
            uint32_t *o8 = reinterpret_cast<uint32_t *>(q8 + base);
            uint2 *o16 = reinterpret_cast<uint2 *>(q16 + base);
            const int64_t g0 = base >> 2;   // generator group of the plane's first element
            const int hw4 = HW >> 2;
            if (POOL) {
                __syncthreads();   // the gather of the previous plane is over
                const int64_t pp = pl * (pool.P * pool.Q);
                q8t_pool::stage_plane<kThreads>(pool.g + pp, pool.idx + pp, pool.P * pool.Q, pool_lds);
                __syncthreads();
            }
            if (crowded && !crowded[c]) {
                const uint8_t *pf = flags + g0;
#pragma unroll 2
                for (int i = threadIdx.x; i < hw4; i += kThreads) {
                    float4 d = POOL ? pool_grad4(pool, pool_lds, i) : q8t_ld_last(pg + i);
                    if (relu) {
                        const uint32_t m = pf[i];
                        d.x = (m & 1u) ? d.x : 0.0f;
                        d.y = (m & 2u) ? d.y : 0.0f;
                        d.z = (m & 4u) ? d.z : 0.0f;
                        d.w = (m & 8u) ? d.w : 0.0f;
                    }
                    float4 r;
                    r.x = bn_dx_kind(d.x, g, k.x, inv, k.y, 0);
                    r.y = bn_dx_kind(d.y, g, k.x, inv, k.y, 0);
                    r.z = bn_dx_kind(d.z, g, k.x, inv, k.y, 0);
                    r.w = bn_dx_kind(d.w, g, k.x, inv, k.y, 0);
                    if (dx) o[i] = r;
                    const uint32_t grp = (uint32_t)(g0 + i);
                    if (q8) o8[i] = quant4<int8_t, true>(r, a8, grp, s8_lo, s8_hi);
                    o16[i] = quant4<int16_t, true>(r, a16, grp, s16_lo, s16_hi);
                }
                continue;
            }
#pragma unroll 2
            for (int i = threadIdx.x; i < hw4; i += kThreads) {
                const float4 v = q8t_ld_last(px + i);
                float4 d = POOL ? pool_grad4(pool, pool_lds, i) : q8t_ld_last(pg + i);
                if (relu) {
                    d.x = bn_map(v.x, mu, inv, g, be) > 0.0f ? d.x : 0.0f;
                    d.y = bn_map(v.y, mu, inv, g, be) > 0.0f ? d.y : 0.0f;
                    d.z = bn_map(v.z, mu, inv, g, be) > 0.0f ? d.z : 0.0f;
                    d.w = bn_map(v.w, mu, inv, g, be) > 0.0f ? d.w : 0.0f;
                }
                float4 r;
                r.x = bn_dx(v.x, d.x, g, k.x, inv, k.y, mn, mx);
                r.y = bn_dx(v.y, d.y, g, k.x, inv, k.y, mn, mx);
                r.z = bn_dx(v.z, d.z, g, k.x, inv, k.y, mn, mx);
                r.w = bn_dx(v.w, d.w, g, k.x, inv, k.y, mn, mx);
                if (dx) o[i] = r;
                const uint32_t grp = (uint32_t)(g0 + i);
                if (q8) o8[i] = quant4<int8_t, true>(r, a8, grp, s8_lo, s8_hi);
                o16[i] = quant4<int16_t, true>(r, a16, grp, s16_lo, s16_hi);
            }
        }
    } else {
        const int64_t total = planes * HW, stride = (int64_t)gridDim.x * kThreads;
        for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
            const int c = (int)((i / HW) % C);
            const float mn = stats[C + c], mx = stats[2 * C + c];
            const float inv = bn_inv(mn, mx, cn, eps);
            const float g = gamma ? gamma[c] : 1.0f;
            const float2 k = consts[c];
            const float xv = x[i];
            const float d = relu && !(bn_map(xv, stats[c], inv, g, beta ? beta[c] : 0.0f) > 0.0f) ? 0.0f : dy[i];
            const float r = bn_dx(xv, d, g, k.x, inv, k.y, mn, mx);
            if (dx) dx[i] = r;
            if (q8) q8[i] = (int8_t)(level_of<true>(r, a8, rng_r16(i, s8_lo, s8_hi)) - a8.half);
            q16[i] = (int16_t)(level_of<true>(r, a16, rng_r16(i, s16_lo, s16_hi)) - a16.half);
        }
    }
}

// pass 2 for planes whose size is not a multiple of 4 (7x7): groups of four consecutive elements of the flat tensor
// (one generator call per group and copy, packed stores), the channel looked up per element since a group can
// straddle planes.  total is a multiple of 4.
__global__ __launch_bounds__(kThreads) void bn_bwdq_apply_flat4(const float *__restrict__ x, const float *__restrict__ dy,
                                                                int64_t total4, int C, int HW, const float *__restrict__ stats,
                                                                const float *__restrict__ gamma, const float *__restrict__ beta,
                                                                int relu, const float2 *__restrict__ consts, float cn, float eps,
                                                                uint32_t s8_lo, uint32_t s8_hi, uint32_t s16_lo, uint32_t s16_hi,
                                                                const float2 *__restrict__ mm, int nmm,
                                                                q8t_qparams *__restrict__ qp8_out,
                                                                q8t_qparams *__restrict__ qp16_out, float *__restrict__ dx,
                                                                int8_t *__restrict__ q8, int16_t *__restrict__ q16,
                                                                const int *__restrict__ crowded)
{
    __shared__ float smf[kThreads / 64];
    float vmin = INFINITY, vmax = -INFINITY;
    for (int i = threadIdx.x; i < nmm; i += kThreads) {
        const float2 p = mm[i];
        vmin = fminf(vmin, p.x);
        vmax = fmaxf(vmax, p.y);
    }
    vmin = block_min_f(vmin, smf);
    vmax = block_max_f(vmax, smf);
    const q8t_qparams qp8 = make_qparams(vmin, vmax, 8), qp16 = make_qparams(vmin, vmax, 16);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (qp8_out) *qp8_out = qp8;
        *qp16_out = qp16;
    }
    const Affine a8 = affine_of(qp8), a16 = affine_of(qp16);
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    const float rHW = 1.0f / (float)HW, rC = 1.0f / (float)C;
    const bool small = HW < (1 << 20) && C < (1 << 21);   // the float-reciprocal quotients below are exact in this range
    for (int64_t b4 = (int64_t)blockIdx.x * kThreads; b4 < total4; b4 += stride) {
        const int64_t i4 = b4 + threadIdx.x;
        if (i4 >= total4) continue;
        // plane and offset of the group's first element, channel of that plane and of the next one (HW >= 4: a group
        // meets at most two planes).  One 64-bit division per workgroup and sweep; a thread is at most
        // 4 * kThreads elements past the workgroup's first one.
        int off0, ca, cb;
        if (small) {
            const int64_t plb = (4 * b4) / HW;                   // uniform in the workgroup
            const int remb = (int)(4 * b4 - plb * HW), cbase = (int)(plb % C);
            const int el = remb + 4 * (int)threadIdx.x;
            const int dpl = q8t_pool::small_div(el, HW, rHW);
            off0 = el - dpl * HW;
            const int cc = cbase + dpl;
            ca = cc - q8t_pool::small_div(cc, C, rC) * C;
        } else {
            const int64_t pl0 = (4 * i4) / HW;
            off0 = (int)(4 * i4 - pl0 * HW);
            ca = (int)(pl0 % C);
        }
        cb = ca + 1 == C ? 0 : ca + 1;
        const bool two = off0 + 3 >= HW;                        // the group straddles two planes
        const float4 d4 = q8t_ld_last(reinterpret_cast<const float4 *>(dy) + i4);
        const float dv[4] = {d4.x, d4.y, d4.z, d4.w};
        float rv[4];
        const bool need_x = relu != 0 || !crowded || crowded[ca] || (two && crowded[cb]);
        float xv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (need_x) {
            const float4 x4 = q8t_ld_last(reinterpret_cast<const float4 *>(x) + i4);
            xv[0] = x4.x; xv[1] = x4.y; xv[2] = x4.z; xv[3] = x4.w;
        }
        // per-channel constants of the first plane, and of the second one where the group straddles
        struct Ch {
            float mu, mn, mx, inv, g, be;
            float2 k;
            bool plain;   // not crowded: extremal coordinates come from the patch kernel, ordinary rule here
        };
        auto load = [&](int c) {
            Ch h;
            h.mu = stats[c];
            h.mn = stats[C + c];
            h.mx = stats[2 * C + c];
            h.inv = bn_inv(h.mn, h.mx, cn, eps);
            h.g = gamma ? gamma[c] : 1.0f;
            h.be = beta ? beta[c] : 0.0f;
            h.k = consts[c];
            h.plain = crowded && !crowded[c];
            return h;
        };
        const Ch ha = load(ca);
        const Ch hb = two ? load(cb) : ha;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const Ch &h = off0 + j >= HW ? hb : ha;
            if (need_x) {
                float d = dv[j];
                if (relu) {
                    const float out = bn_map(xv[j], h.mu, h.inv, h.g, h.be);
                    d = out > 0.0f ? d : 0.0f;
                }
                rv[j] = h.plain ? bn_dx_kind(d, h.g, h.k.x, h.inv, h.k.y, 0) : bn_dx(xv[j], d, h.g, h.k.x, h.inv, h.k.y, h.mn, h.mx);
            } else {
                rv[j] = bn_dx_kind(dv[j], h.g, h.k.x, h.inv, h.k.y, 0);
            }
        }
        const float4 r = make_float4(rv[0], rv[1], rv[2], rv[3]);
        if (dx) reinterpret_cast<float4 *>(dx)[i4] = r;
        if (q8) reinterpret_cast<uint32_t *>(q8)[i4] = quant4<int8_t, true>(r, a8, (uint32_t)i4, s8_lo, s8_hi);
        reinterpret_cast<uint2 *>(q16)[i4] = quant4<int16_t, true>(r, a16, (uint32_t)i4, s16_lo, s16_hi);
    }
}

// after pass 2: the listed coordinates (at the channel's max or min) get their real dx and codes
template <bool POOL = false>
__global__ __launch_bounds__(64) void bn_bwdq_fixup(const float *__restrict__ x, const float *__restrict__ dy, int C, int HW,
                                                    int split, const float *__restrict__ stats,
                                                    const float *__restrict__ gamma, const float *__restrict__ beta, int relu,
                                                    const float2 *__restrict__ consts, float cn, float eps, uint32_t s8_lo,
                                                    uint32_t s8_hi, uint32_t s16_lo, uint32_t s16_hi,
                                                    const q8t_qparams *__restrict__ qp8, const q8t_qparams *__restrict__ qp16,
                                                    const ExtList *__restrict__ lists, const int *__restrict__ crowded,
                                                    float *__restrict__ dx, int8_t *__restrict__ q8, int16_t *__restrict__ q16,
                                                    const PoolSrc pool)
{
    const int c = blockIdx.x;
    if (crowded[c]) return;
    const float mu = stats[c], mn = stats[C + c], mx = stats[2 * C + c];
    const float inv = bn_inv(mn, mx, cn, eps);
    const float g = gamma ? gamma[c] : 1.0f, be = beta ? beta[c] : 0.0f;
    const float2 k = consts[c];
    const Affine a16 = affine_of(*qp16), a8 = q8 ? affine_of(*qp8) : a16;
    for (int e = threadIdx.x; e < split * kExtCap; e += 64) {
        const int sp = e / kExtCap, slot = e - sp * kExtCap;
        const ExtList *l = lists + (int64_t)c * split + sp;
        if (slot >= l->cnt) continue;
        const int64_t j = ((int64_t)l->b[slot] * C + c) * HW + l->pos[slot];
        const float xv = x[j];
        float up;
        if (POOL) {
            const int W = 4 * pool.W4, h = l->pos[slot] / W, w = l->pos[slot] - h * W;
            const int64_t pp = ((int64_t)l->b[slot] * C + c) * (pool.P * pool.Q);
            up = q8t_pool::bwd_at(pool.g + pp, pool.idx + pp, h, w, pool.P, pool.Q);
        } else {
            up = dy[j];
        }
        const float d = relu && !(bn_map(xv, mu, inv, g, be) > 0.0f) ? 0.0f : up;
        const float r = bn_dx(xv, d, g, k.x, inv, k.y, mn, mx);
        if (dx) dx[j] = r;
        if (q8) q8[j] = (int8_t)(level_of<true>(r, a8, rng_r16(j, s8_lo, s8_hi)) - a8.half);
        q16[j] = (int16_t)(level_of<true>(r, a16, rng_r16(j, s16_lo, s16_hi)) - a16.half);
    }
}

// ---- host side ------------------------------------------------------------------------------------
int split_for(int N, int C)
{
    int s = (2048 + C - 1) / C;
    if (s > kMaxSplit) s = kMaxSplit;
    if (s > N) s = N;
    if (s < 1) s = 1;
    return s;
}

size_t ws_parts_bytes(int C) { return (size_t)C * kMaxSplit * sizeof(FwdPartial); }

int check_shape(int N, int C, int H, int W)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return Q8T_ERR_SHAPE;
    const int64_t hw = (int64_t)H * W;
    if (hw > (1 << 30) || (int64_t)N * hw < 2 || (int64_t)N * hw > ((int64_t)1 << 40)) return Q8T_ERR_SHAPE;
    if (C > 65535 * 16) return Q8T_ERR_SHAPE;
    return Q8T_OK;
}

int planes_grid(int64_t planes) { return (int)(planes < 65536 * 16 ? planes : 65536 * 16); }

size_t align16(size_t v) { return (v + 15) & ~(size_t)15; }
size_t bwdq_head_bytes(int C)
{
    return align16((size_t)C * kMaxSplit * sizeof(BwdPartialQ) + (size_t)C * sizeof(float2) + (size_t)((C + 3) / 4) * sizeof(float2));
}
size_t bwdq_fixed_bytes(int C)
{
    return bwdq_head_bytes(C) + align16((size_t)C * kMaxSplit * sizeof(ExtList)) + align16((size_t)C * sizeof(int));
}

}  // namespace

extern "C" {

double q8t_range_bn_scale(int64_t n) { return 1.0 / sqrt(2.0 * log((double)n)); }

size_t q8t_range_bn_workspace_size(int N, int C, int H, int W)
{
    (void)N; (void)H; (void)W;
    if (C <= 0) return 0;
    return ws_parts_bytes(C) + (size_t)C * sizeof(float2);
}

int q8t_range_bn_fwd(const float *x, int N, int C, int H, int W, const float *gamma,
                     const float *beta, float eps, float *y, float *stats_out, int8_t *q_out,
                     q8t_qparams *qp_out, void *ws, void *stream)
{
    const int rc = check_shape(N, C, H, W);
    if (rc) return rc;
    if (!x || !stats_out || (q_out && !qp_out)) return Q8T_ERR_NULL;
    if (!ws || !q8t_aligned(ws, 16)) return Q8T_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const int HW = H * W;
    const double n = (double)N * HW;
    const float cn = (float)q8t_range_bn_scale((int64_t)N * HW);
    FwdPartial *parts = (FwdPartial *)ws;
    const int split = split_for(N, C), NB = (N + split - 1) / split;
    const int nsplit = (N + NB - 1) / NB;
    const bool vec = (HW % 4 == 0) && q8t_aligned(x, 16) && (!y || q8t_aligned(y, 16)) &&
                     (!q_out || q8t_aligned(q_out, 4));
    if (vec)
        hipLaunchKernelGGL(bn_stats_partial<true>, dim3(C, nsplit), dim3(kThreads), 0, st, x, N, C, HW, NB, parts);
    else
        hipLaunchKernelGGL(bn_stats_partial<false>, dim3(C, nsplit), dim3(kThreads), 0, st, x, N, C, HW, NB, parts);
    Q8T_LAUNCH_CHECK();
    // the per-tensor range of the fused 8-bit output needs all channels: separate finalize then.
    // Otherwise the plane kernel folds the slices itself (one launch less).
    const bool fused = !q_out && y && HW >= 256;
    if (!fused) {
        hipLaunchKernelGGL(bn_fwd_finalize, dim3(1), dim3(kThreads), 0, st, parts, C, nsplit, n, cn, eps, gamma,
                           beta, stats_out, q_out ? qp_out : (q8t_qparams *)nullptr);
        Q8T_LAUNCH_CHECK();
    }
    if (!y && !q_out) return Q8T_OK;
    const int64_t planes = (int64_t)N * C;
    const FwdPartial *fparts = fused ? parts : (const FwdPartial *)nullptr;
    if (HW >= 256) {
        const dim3 grid(planes_grid(planes));
#define Q8T_GO(V, Q) \
    hipLaunchKernelGGL((bn_fwd_apply<V, Q>), grid, dim3(kThreads), 0, st, x, planes, C, HW, stats_out, fparts, nsplit, n, gamma, beta, cn, eps, y, q_out, qp_out, 0, 0)
        if (vec) { if (q_out) Q8T_GO(true, true); else Q8T_GO(true, false); }
        else     { if (q_out) Q8T_GO(false, true); else Q8T_GO(false, false); }
#undef Q8T_GO
    } else {
        const int64_t total = planes * HW;
        const dim3 grid((unsigned)((total + kThreads - 1) / kThreads < 65536 * 16 ? (total + kThreads - 1) / kThreads : 65536 * 16));
        if (q_out)
            hipLaunchKernelGGL(bn_fwd_apply_flat<true>, grid, dim3(kThreads), 0, st, x, total, C, HW, stats_out, gamma, beta, cn, eps, y, q_out, qp_out, 0);
        else
            hipLaunchKernelGGL(bn_fwd_apply_flat<false>, grid, dim3(kThreads), 0, st, x, total, C, HW, stats_out, gamma, beta, cn, eps, y, q_out, qp_out, 0);
    }
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

// Forward with statistics that something else already produced (the convolution epilogue):
// normalization (and 8-bit output) only, one pass over x.
static int range_bn_fwd_apply_impl(const float *x, int N, int C, int H, int W, const float *gamma, const float *beta,
                                   float eps, const float *stats, float *y, int8_t *q_out, q8t_qparams *qp_out,
                                   void *stream, int relu)
{
    const int rc = check_shape(N, C, H, W);
    if (rc) return rc;
    if (!x || !stats || (!y && !q_out) || (q_out && !qp_out)) return Q8T_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    const int HW = H * W;
    const double n = (double)N * HW;
    const float cn = (float)q8t_range_bn_scale((int64_t)N * HW);
    const bool vec = (HW % 4 == 0) && q8t_aligned(x, 16) && (!y || q8t_aligned(y, 16)) &&
                     (!q_out || q8t_aligned(q_out, 4));
    if (q_out) {
        hipLaunchKernelGGL(bn_qrange_from_stats, dim3(1), dim3(kThreads), 0, st, stats, C, cn, eps, gamma, beta, relu, qp_out);
        Q8T_LAUNCH_CHECK();
    }
    float *stats_rw = const_cast<float *>(stats);   // only read when no partial sums are passed
    const FwdPartial *fparts = nullptr;
    const int64_t planes = (int64_t)N * C;
    const int flat4 = vec && HW < 4 * kThreads;   // planes below 1024 positions: a float4 per thread
    if (HW >= 256 || flat4) {
        const int64_t blocks4 = (planes * (HW >> 2) + kThreads - 1) / kThreads;
        const dim3 grid((unsigned)(flat4 ? (blocks4 < 65536 * 16 ? blocks4 : 65536 * 16) : planes_grid(planes)));
#define Q8T_GO(V, Q) \
    hipLaunchKernelGGL((bn_fwd_apply<V, Q>), grid, dim3(kThreads), 0, st, x, planes, C, HW, stats_rw, fparts, 1, n, gamma, beta, cn, eps, y, q_out, qp_out, relu, flat4)
        if (vec) { if (q_out) Q8T_GO(true, true); else Q8T_GO(true, false); }
        else     { if (q_out) Q8T_GO(false, true); else Q8T_GO(false, false); }
#undef Q8T_GO
    } else {
        const int64_t total = planes * HW;
        const dim3 grid((unsigned)((total + kThreads - 1) / kThreads < 65536 * 16 ? (total + kThreads - 1) / kThreads : 65536 * 16));
        if (q_out)
            hipLaunchKernelGGL(bn_fwd_apply_flat<true>, grid, dim3(kThreads), 0, st, x, total, C, HW, stats_rw, gamma, beta, cn, eps, y, q_out, qp_out, relu);
        else
            hipLaunchKernelGGL(bn_fwd_apply_flat<false>, grid, dim3(kThreads), 0, st, x, total, C, HW, stats_rw, gamma, beta, cn, eps, y, q_out, qp_out, relu);
    }
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

int q8t_range_bn_fwd_apply(const float *x, int N, int C, int H, int W, const float *gamma, const float *beta, float eps,
                           const float *stats, float *y, int8_t *q_out, q8t_qparams *qp_out, void *stream)
{
    return range_bn_fwd_apply_impl(x, N, C, H, W, gamma, beta, eps, stats, y, q_out, qp_out, stream, 0);
}

int q8t_range_bn_relu_fwd_apply(const float *x, int N, int C, int H, int W, const float *gamma, const float *beta,
                                float eps, const float *stats, float *y, int8_t *q_out, q8t_qparams *qp_out,
                                void *stream)
{
    return range_bn_fwd_apply_impl(x, N, C, H, W, gamma, beta, eps, stats, y, q_out, qp_out, stream, 1);
}

static int range_bn_bwd_impl(const float *x, const float *dy, const float *stats, int N, int C, int H, int W,
                             const float *gamma, float eps, float *dx, float *dgamma, float *dbeta, void *ws,
                             void *stream)
{
    const float *beta = nullptr;
    const int relu = 0;
    const int rc = check_shape(N, C, H, W);
    if (rc) return rc;
    if (!x || !dy || !stats) return Q8T_ERR_NULL;
    if (!ws || !q8t_aligned(ws, 16)) return Q8T_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const int HW = H * W;
    const double n = (double)N * HW;
    const float cn = (float)q8t_range_bn_scale((int64_t)N * HW);
    double2 *parts = (double2 *)ws;
    float2 *consts = (float2 *)((char *)ws + ws_parts_bytes(C));
    const int split = split_for(N, C), NB = (N + split - 1) / split;
    const int nsplit = (N + NB - 1) / NB;
    const bool vec = (HW % 4 == 0) && q8t_aligned(x, 16) && q8t_aligned(dy, 16) && (!dx || q8t_aligned(dx, 16));
    if (vec)
        hipLaunchKernelGGL(bn_bwd_partial<true>, dim3(C, nsplit), dim3(kThreads), 0, st, x, dy, stats, N, C, HW, NB, cn, eps, gamma, beta, relu, parts);
    else
        hipLaunchKernelGGL(bn_bwd_partial<false>, dim3(C, nsplit), dim3(kThreads), 0, st, x, dy, stats, N, C, HW, NB, cn, eps, gamma, beta, relu, parts);
    Q8T_LAUNCH_CHECK();
    const bool fused = dx && HW >= 256;
    if (!fused) {
        hipLaunchKernelGGL(bn_bwd_finalize, dim3((C + kThreads - 1) / kThreads), dim3(kThreads), 0, st, parts, C,
                           nsplit, n, cn, eps, stats, gamma, dgamma, dbeta, consts);
        Q8T_LAUNCH_CHECK();
    }
    if (!dx) return Q8T_OK;
    const int64_t planes = (int64_t)N * C;
    if (HW >= 256) {
        const dim3 grid((unsigned)planes_grid(planes));
        if (vec)
            hipLaunchKernelGGL(bn_bwd_apply<true>, grid, dim3(kThreads), 0, st, x, dy, planes, C, HW, stats, gamma, consts, parts, nsplit, n, dgamma, dbeta, cn, eps, dx, beta, relu);
        else
            hipLaunchKernelGGL(bn_bwd_apply<false>, grid, dim3(kThreads), 0, st, x, dy, planes, C, HW, stats, gamma, consts, parts, nsplit, n, dgamma, dbeta, cn, eps, dx, beta, relu);
    } else {
        const int64_t total = planes * HW;
        const dim3 grid((unsigned)((total + kThreads - 1) / kThreads < 65536 * 16 ? (total + kThreads - 1) / kThreads : 65536 * 16));
        hipLaunchKernelGGL(bn_bwd_apply_flat, grid, dim3(kThreads), 0, st, x, dy, total, C, HW, stats, gamma, consts, cn, eps, dx, beta, relu);
    }
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

int q8t_range_bn_bwd(const float *x, const float *dy, const float *stats, int N, int C, int H, int W,
                     const float *gamma, float eps, float *dx, float *dgamma, float *dbeta, void *ws,
                     void *stream)
{
    return range_bn_bwd_impl(x, dy, stats, N, C, H, W, gamma, eps, dx, dgamma, dbeta, ws, stream);
}

size_t q8t_range_bn_bwd_bifurcate_workspace_size(int N, int C, int H, int W)
{
    if (C <= 0 || N <= 0 || H <= 0 || W <= 0) return 0;
    // partial sums, per-channel constants, range pairs | lists of extremal coordinates, crowded flags
    return bwdq_fixed_bytes(C);
}

// the pooled-gradient variant serves planes of at least 4 * kThreads positions whose width is a multiple of 4 and
// whose pooled plane (a multiple of 16 elements) fits in LDS; other shapes go through an unpooled gradient
static bool pooled_direct(int H, int W)
{
    const int P = (H - 1) / 2 + 1, Q = (W - 1) / 2 + 1;
    return W % 4 == 0 && (int64_t)H * W >= 4 * kThreads && (int64_t)H * W < (1 << 22) && (P * Q) % 16 == 0 &&
           q8t_pool::lds_bytes(P * Q) <= 60 * 1024;
}

// gpool / idx != NULL: dy is not read; the upstream gradient is gathered from the pooled one (pooled_direct shapes)
static int range_bn_bwd_bifurcate_impl(const float *x, const float *dy, const float *stats, int N, int C, int H, int W,
                                       const float *gamma, const float *beta, int relu, float eps, float *dx,
                                       float *dgamma, float *dbeta, uint64_t seed8, uint64_t seed16, int8_t *q8_out,
                                       q8t_qparams *qp8_out, int16_t *q16_out, q8t_qparams *qp16_out, void *ws,
                                       void *stream, const float *gpool = nullptr, const uint8_t *idx = nullptr)
{
    const int rc = check_shape(N, C, H, W);
    if (rc) return rc;
    const bool pooled = gpool != nullptr;
    if (!x || (!dy && !pooled) || !stats || (q8_out && !qp8_out) || !q16_out || !qp16_out) return Q8T_ERR_NULL;
    if (!ws || !q8t_aligned(ws, 16)) return Q8T_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const int HW = H * W;
    const double n = (double)N * HW;
    const float cn = (float)q8t_range_bn_scale((int64_t)N * HW);
    BwdPartialQ *parts = (BwdPartialQ *)ws;
    float2 *consts = (float2 *)((char *)ws + (size_t)C * kMaxSplit * sizeof(BwdPartialQ));
    const int split = split_for(N, C), NB = (N + split - 1) / split;
    const int nsplit = (N + NB - 1) / NB;
    const bool vec = (HW % 4 == 0) && q8t_aligned(x, 16) && q8t_aligned(dy, 16) && (!dx || q8t_aligned(dx, 16)) &&
                     q8t_aligned(q8_out, 4) && q8t_aligned(q16_out, 8);
    if (pooled && !(vec && !relu && pooled_direct(H, W) && q8t_aligned(gpool, 16) && q8t_aligned(idx, 16))) return Q8T_ERR_SHAPE;
    PoolSrc pool = {gpool, idx, W >> 2, (H - 1) / 2 + 1, (W - 1) / 2 + 1, 1.0f / (float)(W >> 2 ? W >> 2 : 1)};
    const size_t pool_lds = pooled ? q8t_pool::lds_bytes(pool.P * pool.Q) : 0;
    // Without the rectifier (and with float4 access) pass 2 leaves x alone: 15 instead of 19 bytes per element.
    // Measured: -6% only, the pass is as much bound by the ~45 vector operations per element of the two hashed
    // roundings as by memory; with the rectifier the mask bytes cost more than the x they replace (+4%), so that
    // variant keeps reading x (flags == NULL; the kernels still take them).
    const int64_t total = (int64_t)N * C * HW;
    const bool flat4 = !vec && HW >= 4 && total % 4 == 0 && q8t_aligned(x, 16) && q8t_aligned(dy, 16) &&
                       (!dx || q8t_aligned(dx, 16)) && q8t_aligned(q8_out, 4) && q8t_aligned(q16_out, 8);
    const bool nox = (vec || flat4) && !relu;
    ExtList *lists = nox ? (ExtList *)((char *)ws + bwdq_head_bytes(C)) : (ExtList *)nullptr;
    int *crowded = nox ? (int *)((char *)lists + align16((size_t)C * kMaxSplit * sizeof(ExtList))) : (int *)nullptr;
    uint8_t *flags = nullptr;
    if (pooled)
        hipLaunchKernelGGL((bn_bwdq_partial<true, true>), dim3(C, nsplit), dim3(kThreads), pool_lds, st, x, dy, stats, N, C, HW, NB,
                           cn, eps, gamma, beta, relu, parts, lists, flags, pool);
    else if (vec)
        hipLaunchKernelGGL((bn_bwdq_partial<true, false>), dim3(C, nsplit), dim3(kThreads), 0, st, x, dy, stats, N, C, HW, NB, cn,
                           eps, gamma, beta, relu, parts, lists, flags, pool);
    else
        hipLaunchKernelGGL((bn_bwdq_partial<false, false>), dim3(C, nsplit), dim3(kThreads), 0, st, x, dy, stats, N, C, HW, NB, cn,
                           eps, gamma, beta, relu, parts, lists, flags, pool);
    Q8T_LAUNCH_CHECK();
    float2 *mm = consts + C;
    const int nmm = (C + kThreads / 64 - 1) / (kThreads / 64);
    hipLaunchKernelGGL(bn_bwdq_finalize, dim3(nmm), dim3(kThreads), 0, st, parts, C, nsplit, n, cn, eps, stats, gamma, dgamma,
                       dbeta, consts, mm, lists, crowded);
    Q8T_LAUNCH_CHECK();
    const int64_t planes = (int64_t)N * C;
    const uint32_t s8l = (uint32_t)seed8, s8h = (uint32_t)(seed8 >> 32), s16l = (uint32_t)seed16, s16h = (uint32_t)(seed16 >> 32);
    if (vec) {
        // planes of at least 1024 positions: a workgroup per plane; smaller ones: a float4 per thread
        const int64_t blocks4 = (planes * (HW >> 2) + kThreads - 1) / kThreads;
        // at most kApplyBlocks workgroups, which sweep: every workgroup first folds the ranges of pass 1 and derives the
        // two quantizers, and with one short-lived workgroup per 256 float4s that prologue cost a quarter of the pass
        const int64_t gridx = HW >= 4 * kThreads ? (planes < kApplyBlocks ? planes : kApplyBlocks)
                                                 : (blocks4 < kApplyBlocks ? blocks4 : kApplyBlocks);
        if (pooled)
            hipLaunchKernelGGL((bn_bwdq_apply<true, true>), dim3((unsigned)gridx), dim3(kThreads), pool_lds, st, x, dy, planes, C,
                               HW, stats, gamma, beta, relu, consts, cn, eps, s8l, s8h, s16l, s16h, mm, nmm, qp8_out, qp16_out, dx,
                               q8_out, q16_out, crowded, flags, pool);
        else
            hipLaunchKernelGGL((bn_bwdq_apply<true, false>), dim3((unsigned)gridx), dim3(kThreads), 0, st, x, dy, planes, C, HW,
                               stats, gamma, beta, relu, consts, cn, eps, s8l, s8h, s16l, s16h, mm, nmm, qp8_out, qp16_out, dx,
                               q8_out, q16_out, crowded, flags, pool);
        if (nox) {
            Q8T_LAUNCH_CHECK();
            if (pooled)
                hipLaunchKernelGGL(bn_bwdq_fixup<true>, dim3(C), dim3(64), 0, st, x, dy, C, HW, nsplit, stats, gamma, beta, relu,
                                   consts, cn, eps, s8l, s8h, s16l, s16h, qp8_out, qp16_out, lists, crowded, dx, q8_out, q16_out,
                                   pool);
            else
                hipLaunchKernelGGL(bn_bwdq_fixup<false>, dim3(C), dim3(64), 0, st, x, dy, C, HW, nsplit, stats, gamma, beta, relu,
                                   consts, cn, eps, s8l, s8h, s16l, s16h, qp8_out, qp16_out, lists, crowded, dx, q8_out, q16_out,
                                   pool);
        }
    } else if (flat4) {
        const int64_t blocks4 = (total / 4 + kThreads - 1) / kThreads;
        hipLaunchKernelGGL(bn_bwdq_apply_flat4, dim3((unsigned)(blocks4 < kApplyBlocks ? blocks4 : kApplyBlocks)), dim3(kThreads), 0, st,
                           x, dy, total / 4, C, HW, stats, gamma, beta, relu, consts, cn, eps, s8l, s8h, s16l, s16h, mm, nmm,
                           qp8_out, qp16_out, dx, q8_out, q16_out, crowded);
        if (nox) {
            Q8T_LAUNCH_CHECK();
            hipLaunchKernelGGL(bn_bwdq_fixup<false>, dim3(C), dim3(64), 0, st, x, dy, C, HW, nsplit, stats, gamma, beta, relu,
                               consts, cn, eps, s8l, s8h, s16l, s16h, qp8_out, qp16_out, lists, crowded, dx, q8_out, q16_out, pool);
        }
    } else {
        const int64_t blocks = (total + kThreads - 1) / kThreads;
        hipLaunchKernelGGL((bn_bwdq_apply<false, false>), dim3((unsigned)(blocks < 65536 * 16 ? blocks : 65536 * 16)),
                           dim3(kThreads), 0, st, x, dy, planes, C, HW, stats, gamma, beta, relu, consts, cn, eps, s8l, s8h, s16l,
                           s16h, mm, nmm, qp8_out, qp16_out, dx, q8_out, q16_out, (const int *)nullptr, (const uint8_t *)nullptr,
                           pool);
    }
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

int q8t_range_bn_bwd_bifurcate(const float *x, const float *dy, const float *stats, int N, int C, int H, int W,
                               const float *gamma, float eps, float *dx, float *dgamma, float *dbeta,
                               uint64_t seed8, uint64_t seed16, int8_t *q8_out, q8t_qparams *qp8_out,
                               int16_t *q16_out, q8t_qparams *qp16_out, void *ws, void *stream)
{
    return range_bn_bwd_bifurcate_impl(x, dy, stats, N, C, H, W, gamma, nullptr, 0, eps, dx, dgamma, dbeta, seed8, seed16,
                                       q8_out, qp8_out, q16_out, qp16_out, ws, stream);
}

int q8t_range_bn_relu_bwd_bifurcate(const float *x, const float *dy, const float *stats, int N, int C, int H, int W,
                                    const float *gamma, const float *beta, float eps, float *dx, float *dgamma,
                                    float *dbeta, uint64_t seed8, uint64_t seed16, int8_t *q8_out,
                                    q8t_qparams *qp8_out, int16_t *q16_out, q8t_qparams *qp16_out, void *ws,
                                    void *stream)
{
    return range_bn_bwd_bifurcate_impl(x, dy, stats, N, C, H, W, gamma, beta, 1, eps, dx, dgamma, dbeta, seed8, seed16,
                                       q8_out, qp8_out, q16_out, qp16_out, ws, stream);
}

size_t q8t_maxpool_range_bn_bwd_bifurcate_workspace_size(int N, int C, int H, int W)
{
    if (C <= 0 || N <= 0 || H <= 0 || W <= 0) return 0;
    const size_t fixed = align16(bwdq_fixed_bytes(C));
    return pooled_direct(H, W) ? fixed : fixed + sizeof(float) * (size_t)N * C * H * W;
}

int q8t_maxpool_range_bn_bwd_bifurcate(const float *x, const float *gpool, const uint8_t *idx, const float *stats, int N, int C,
                                       int H, int W, const float *gamma, float eps, float *dgamma, float *dbeta, uint64_t seed8,
                                       uint64_t seed16, int8_t *q8_out, q8t_qparams *qp8_out, int16_t *q16_out,
                                       q8t_qparams *qp16_out, void *ws, void *stream)
{
    const int rc = check_shape(N, C, H, W);
    if (rc) return rc;
    if (!gpool || !idx) return Q8T_ERR_NULL;
    if (!ws || !q8t_aligned(ws, 16)) return Q8T_ERR_WORKSPACE;
    if (pooled_direct(H, W)) {
        if (!q8t_aligned(x, 16) || !q8t_aligned(gpool, 16) || !q8t_aligned(idx, 16) || !q8t_aligned(q8_out, 4) ||
            !q8t_aligned(q16_out, 8))
            return Q8T_ERR_SHAPE;
        return range_bn_bwd_bifurcate_impl(x, nullptr, stats, N, C, H, W, gamma, nullptr, 0, eps, nullptr, dgamma, dbeta, seed8,
                                           seed16, q8_out, qp8_out, q16_out, qp16_out, ws, stream, gpool, idx);
    }
    // other shapes: the unpooled gradient goes through the workspace
    float *dy = (float *)((char *)ws + align16(bwdq_fixed_bytes(C)));
    const int rp = q8t_maxpool_relu_bwd(gpool, idx, N, C, H, W, dy, stream);
    if (rp) return rp;
    return range_bn_bwd_bifurcate_impl(x, dy, stats, N, C, H, W, gamma, nullptr, 0, eps, nullptr, dgamma, dbeta, seed8, seed16,
                                       q8_out, qp8_out, q16_out, qp16_out, ws, stream);
}

}  // extern "C"

int q8t_range_bn_stats(const float *x, int N, int C, int H, int W, float *stats_out, void *ws, hipStream_t st)
{
    return q8t_range_bn_fwd(x, N, C, H, W, nullptr, nullptr, 0.0f, nullptr, stats_out, nullptr, nullptr, ws, (void *)st);
}
