// Network plumbing around the method (not from the paper): the pieces of a ResNet training step
// that sit between the library's products and normalizations, fused with their neighbours so that
// the large activation tensors make one trip through HBM instead of three:
//   * stem: Range BN (Section 3, eq. (range)) + ReLU + 3x3 / stride 2 / pad 1 max pooling in one
//     pass, and the matching backward that hands the Range BN backward its upstream gradient;
//   * block end: residual sum + ReLU, which also leaves the maximum of its result behind, so the
//     8-bit quantization of the next layer's operand (Appendix B) needs no min/max pass (the
//     minimum of a rectified tensor, widened to contain 0, is 0);
//   * ReLU backward, optionally added to the gradient of the other branch.
#include "q8t_common.h"
#include "q8t_internal.h"
#include "pool_gather.h"

namespace {

using q8t_pool::small_div;

constexpr int kThreads = 256;
constexpr int kMaxPartials = 1024;

// 1 / (C(n) * (max - min) + eps) and gamma * ((x - mu) * inv) + beta: one fp32 rounding per
// operation, the same sequence as the Range BN kernels (the results must agree bit for bit)
__device__ __forceinline__ float g_bn_inv(float mn, float mx, float cn, float eps)
{
    const float range = mx - mn;
    const float scaled = cn * range;
    const float denom = scaled + eps;
    return 1.0f / denom;
}
__device__ __forceinline__ float g_bn_relu(float x, float mu, float inv, float g, float b)
{
    const float cen = x - mu;
    const float xh = cen * inv;
    const float sc = xh * g;
    const float y = sc + b;
    return y > 0.0f ? y : 0.0f;
}

// a workgroup per (image, channel) plane (32-bit index arithmetic inside it).  VEC (W a multiple of 4):
// a thread owns two neighbouring pooled columns 2t, 2t+1 of a pooled row; their windows span the input
// columns 4t-1 .. 4t+3 = one scalar and one aligned 16-byte load per input row, normalized once each.
template <bool VEC>
__global__ __launch_bounds__(kThreads) void bn_relu_maxpool_fwd(const float *__restrict__ x, int C, int H, int W, int P, int Q,
                                                                const float *__restrict__ stats, const float *__restrict__ gamma,
                                                                const float *__restrict__ beta, float cn, float eps,
                                                                float *__restrict__ out, uint8_t *__restrict__ idx)
{
    const int64_t pl = blockIdx.x;
    const int c = (int)(pl % C);
    const float mu = stats[c];
    const float inv = g_bn_inv(stats[C + c], stats[2 * C + c], cn, eps);
    const float g = gamma ? gamma[c] : 1.0f, b = beta ? beta[c] : 0.0f;
    const float *xp = x + pl * (int64_t)H * W;
    float *op = out + pl * (int64_t)P * Q;
    uint8_t *ip = idx + pl * (int64_t)P * Q;
    if (VEC) {
        const int Q2 = Q >> 1;                 // W % 4 == 0: Q = W / 2 is even
        const float rq = 1.0f / (float)Q2;
        for (int o = threadIdx.x; o < P * Q2; o += kThreads) {
            const int p = small_div(o, Q2, rq), t = o - p * Q2;
            float b0 = -INFINITY, b1 = -INFINITY;
            int w0 = 255, w1 = 255;
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                const int h = 2 * p - 1 + i;
                if (h < 0 || h >= H) continue;
                const float *row = xp + h * W + 4 * t;
                const float4 v = *reinterpret_cast<const float4 *>(row);
                float e[5];
                e[0] = t > 0 ? g_bn_relu(row[-1], mu, inv, g, b) : -INFINITY;     // column 4t-1 (outside for t = 0)
                e[1] = g_bn_relu(v.x, mu, inv, g, b);
                e[2] = g_bn_relu(v.y, mu, inv, g, b);
                e[3] = g_bn_relu(v.z, mu, inv, g, b);
                e[4] = g_bn_relu(v.w, mu, inv, g, b);
#pragma unroll
                for (int j = 0; j < 3; ++j) {      // the first maximum in row-major order
                    if (e[j] > b0) { b0 = e[j]; w0 = 3 * i + j; }
                    if (e[j + 2] > b1) { b1 = e[j + 2]; w1 = 3 * i + j; }
                }
            }
            *reinterpret_cast<float2 *>(op + p * Q + 2 * t) = make_float2(b0, b1);
            *reinterpret_cast<uchar2 *>(ip + p * Q + 2 * t) =
                make_uchar2((unsigned char)(b0 > 0.0f ? w0 : 255), (unsigned char)(b1 > 0.0f ? w1 : 255));
        }
        return;
    }
    const float rq = 1.0f / (float)Q;
    for (int o = threadIdx.x; o < P * Q; o += kThreads) {
        const int p = small_div(o, Q, rq), q = o - p * Q;
        float best = -INFINITY;
        int where = 255;
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const int h = 2 * p - 1 + i;
            if (h < 0 || h >= H) continue;
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const int w = 2 * q - 1 + j;
                if (w < 0 || w >= W) continue;
                const float v = g_bn_relu(xp[h * W + w], mu, inv, g, b);
                if (v > best) {       // the first maximum in row-major order
                    best = v;
                    where = 3 * i + j;
                }
            }
        }
        op[o] = best;
        ip[o] = (uint8_t)(best > 0.0f ? where : 255);
    }
}

// a workgroup per plane; with W a multiple of 4 a thread writes 4 neighbouring positions at once.  LDS: the pooled
// plane and its indices are first copied into LDS with wide coalesced loads and gathered from there (a position
// looks at up to six pooled elements: as global loads those dozen narrow accesses per 16 bytes written bound
// the kernel at a third of the streaming rate)
template <bool VEC, bool LDS>
__global__ __launch_bounds__(kThreads) void maxpool_relu_bwd(const float *__restrict__ gpool, const uint8_t *__restrict__ idx, int H,
                                                             int W, int P, int Q, float *__restrict__ dy)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t pool_lds[];
    const int64_t pl = blockIdx.x;
    const float *gp = gpool + pl * (int64_t)P * Q;
    const uint8_t *ip = idx + pl * (int64_t)P * Q;
    float *dp = dy + pl * (int64_t)H * W;
    if (LDS) {
        // P * Q is a multiple of 16 here and both planes start 16-byte aligned
        q8t_pool::stage_plane<kThreads>(gp, ip, P * Q, pool_lds);
        __syncthreads();
        gp = reinterpret_cast<const float *>(pool_lds);
        ip = pool_lds + (size_t)P * Q * sizeof(float);
    }
    if (VEC) {
        const int W4 = W >> 2;
        const float rw = 1.0f / (float)W4;
        for (int e = threadIdx.x; e < H * W4; e += kThreads) {
            const int h = small_div(e, W4, rw), qa = 2 * (e - h * W4);
            reinterpret_cast<float4 *>(dp)[e] = q8t_pool::bwd_gather4(gp, ip, h, qa, P, Q);
        }
    } else {
        const float rw = 1.0f / (float)W;
        for (int e = threadIdx.x; e < H * W; e += kThreads) {
            const int h = small_div(e, W, rw), w = e - h * W;
            dp[e] = q8t_pool::bwd_at(gp, ip, h, w, P, Q);
        }
    }
}

__device__ __forceinline__ float block_max(float v, float *smem)
{
    v = wave_reduce(v, OpMax());
    if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = smem[0];
    for (int w = 1; w < kThreads / 64; ++w) r = fmaxf(r, smem[w]);
    return r;
}

// out = relu(a + b); one (0, max) pair per workgroup for the quantization that follows
template <bool VEC>
__global__ __launch_bounds__(kThreads) void add_relu_fwd(const float *__restrict__ a, const float *__restrict__ b, int64_t n,
                                                         float *__restrict__ out, float2 *__restrict__ partials)
{
    __shared__ float smem[kThreads / 64];
    float mx = 0.0f;
    if (VEC) {
        const int64_t n4 = n >> 2;
        const float4 *a4 = reinterpret_cast<const float4 *>(a), *b4 = reinterpret_cast<const float4 *>(b);
        float4 *o4 = reinterpret_cast<float4 *>(out);
        const int64_t per = (n4 + gridDim.x - 1) / gridDim.x;
        const int64_t lo = (int64_t)blockIdx.x * per, hi = min(n4, lo + per);
#pragma unroll 2
        for (int64_t i = lo + threadIdx.x; i < hi; i += kThreads) {
            const float4 u = q8t_ld_last(a4 + i), v = q8t_ld_last(b4 + i);
            float4 r;
            r.x = u.x + v.x; r.y = u.y + v.y; r.z = u.z + v.z; r.w = u.w + v.w;
            r.x = r.x > 0.0f ? r.x : 0.0f; r.y = r.y > 0.0f ? r.y : 0.0f;
            r.z = r.z > 0.0f ? r.z : 0.0f; r.w = r.w > 0.0f ? r.w : 0.0f;
            o4[i] = r;
            mx = fmaxf(fmaxf(mx, r.x), fmaxf(r.y, fmaxf(r.z, r.w)));
        }
        const int64_t tail = (n4 << 2) + (int64_t)blockIdx.x * kThreads + threadIdx.x;
        if (tail < n) {
            const float s = a[tail] + b[tail];
            const float r = s > 0.0f ? s : 0.0f;
            out[tail] = r;
            mx = fmaxf(mx, r);
        }
    } else {
        const int64_t stride = (int64_t)gridDim.x * kThreads;
        for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
            const float s = a[i] + b[i];
            const float r = s > 0.0f ? s : 0.0f;
            out[i] = r;
            mx = fmaxf(mx, r);
        }
    }
    mx = block_max(mx, smem);
    if (threadIdx.x == 0) partials[blockIdx.x] = make_float2(0.0f, mx);
}

// tail of a residual block: out = relu(bn(x) + o), o = other or bn'(other) (a shortcut that is convolution + Range BN);
// one (0, max) pair per workgroup for the quantization that follows.  hw4 > 0: planes are whole float4 groups.
__device__ __forceinline__ float g_bn(float x, float mu, float inv, float g, float b)
{
    const float cen = x - mu;
    const float xh = cen * inv;
    const float sc = xh * g;
    return sc + b;
}
struct TailBN {
    const float *stats, *gamma, *beta;   // stats == NULL: the operand is taken as it is
};
__device__ __forceinline__ void tail_consts(const TailBN &t, int c, int C, float cn, float eps, float &mu, float &inv, float &g, float &b)
{
    mu = t.stats[c];
    inv = g_bn_inv(t.stats[C + c], t.stats[2 * C + c], cn, eps);
    g = t.gamma ? t.gamma[c] : 1.0f;
    b = t.beta ? t.beta[c] : 0.0f;
}
template <bool VEC>
__global__ __launch_bounds__(kThreads) void bn_add_relu_fwd(const float *__restrict__ x, TailBN bx, const float *__restrict__ other,
                                                            TailBN bo, int64_t n, int C, int HW, float cn, float eps,
                                                            float *__restrict__ out, float2 *__restrict__ partials)
{
    __shared__ float smem[kThreads / 64];
    float mx = 0.0f;
    if (VEC) {
        const uint32_t hw4 = (uint32_t)(HW >> 2);
        const int64_t n4 = n >> 2;
        const float4 *x4 = reinterpret_cast<const float4 *>(x), *o4 = reinterpret_cast<const float4 *>(other);
        float4 *r4 = reinterpret_cast<float4 *>(out);
        const int64_t per = (n4 + gridDim.x - 1) / gridDim.x;
        const int64_t lo = (int64_t)blockIdx.x * per, hi = min(n4, lo + per);
#pragma unroll 2
        for (int64_t i = lo + threadIdx.x; i < hi; i += kThreads) {
            const int c = (int)(((uint32_t)i / hw4) % (uint32_t)C);   // n4 < 2^32 (checked on the host)
            float mu, inv, g, b;
            tail_consts(bx, c, C, cn, eps, mu, inv, g, b);
            const float4 u = q8t_ld_last(x4 + i);
            float4 v = q8t_ld_last(o4 + i);
            if (bo.stats) {
                float omu, oinv, og, ob;
                tail_consts(bo, c, C, cn, eps, omu, oinv, og, ob);
                v.x = g_bn(v.x, omu, oinv, og, ob); v.y = g_bn(v.y, omu, oinv, og, ob);
                v.z = g_bn(v.z, omu, oinv, og, ob); v.w = g_bn(v.w, omu, oinv, og, ob);
            }
            float4 r;
            r.x = g_bn(u.x, mu, inv, g, b) + v.x; r.y = g_bn(u.y, mu, inv, g, b) + v.y;
            r.z = g_bn(u.z, mu, inv, g, b) + v.z; r.w = g_bn(u.w, mu, inv, g, b) + v.w;
            r.x = r.x > 0.0f ? r.x : 0.0f; r.y = r.y > 0.0f ? r.y : 0.0f;
            r.z = r.z > 0.0f ? r.z : 0.0f; r.w = r.w > 0.0f ? r.w : 0.0f;
            r4[i] = r;
            mx = fmaxf(fmaxf(mx, r.x), fmaxf(r.y, fmaxf(r.z, r.w)));
        }
    } else {
        const int64_t stride = (int64_t)gridDim.x * kThreads;
        for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
            const int c = (int)((i / HW) % C);
            float mu, inv, g, b;
            tail_consts(bx, c, C, cn, eps, mu, inv, g, b);
            float v = other[i];
            if (bo.stats) {
                float omu, oinv, og, ob;
                tail_consts(bo, c, C, cn, eps, omu, oinv, og, ob);
                v = g_bn(v, omu, oinv, og, ob);
            }
            const float s = g_bn(x[i], mu, inv, g, b) + v;
            const float r = s > 0.0f ? s : 0.0f;
            out[i] = r;
            mx = fmaxf(mx, r);
        }
    }
    mx = block_max(mx, smem);
    if (threadIdx.x == 0) partials[blockIdx.x] = make_float2(0.0f, mx);
}

// out[pl][p][q] = x[pl][p * s][q * s] for 8-bit codes: the operand of a 1x1 convolution with stride s and no padding,
// which is the stride-1 layer on these positions.  PAIRS (s = 2, Q a multiple of 4, rows 8-byte aligned): a thread turns
// 8 input bytes into 4 output bytes with one byte permute.
template <bool PAIRS>
__global__ __launch_bounds__(kThreads) void subsample_codes(const int8_t *__restrict__ x, int64_t planes, int H, int W, int P,
                                                            int Q, int s, int8_t *__restrict__ out)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    if (PAIRS) {
        const int Q4 = Q >> 2;
        const int64_t total = planes * P * Q4;
        for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
            const int64_t row = i / Q4;                       // (plane, p)
            const int q4 = (int)(i - row * Q4);
            const int64_t pl = row / P;
            const int p = (int)(row - pl * P);
            const uint2 v = *reinterpret_cast<const uint2 *>(x + (pl * H + 2 * p) * W + 8 * q4);
            reinterpret_cast<uint32_t *>(out)[i] = __builtin_amdgcn_perm(v.y, v.x, 0x06040200);   // bytes 0, 2, 4, 6
        }
    } else {
        const int64_t total = planes * P * Q;
        for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += stride) {
            const int64_t row = i / Q, pl = row / P;
            const int q = (int)(i - row * Q), p = (int)(row - pl * P);
            out[i] = x[(pl * H + (int64_t)p * s) * W + (int64_t)q * s];
        }
    }
}

// res = out > 0 ? g1 + t : 0 with t = g2s at the positions whose row and column are even (stride 2: the lattice a
// 1x1 / stride-2 convolution reads), 0 elsewhere; the addition is performed everywhere (x + 0 is not x for x = -0), so
// the result is bit-identical to the plain sum with the zero-filled gradient.  A wavefront per plane and sweep.
// ROWS4: W is a multiple of 4, so a float4 stays inside an image row; otherwise only the plane is a multiple of 4.
template <bool ROWS4>
__global__ __launch_bounds__(kThreads) void relu_bwd_sum_lattice2(const float *__restrict__ g1, const float *__restrict__ g2s,
                                                                  const float *__restrict__ outv, int64_t planes, int H, int W,
                                                                  int Hs, int Ws, float *__restrict__ res)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 6, nw = (int64_t)gridDim.x * (kThreads / 64);
    const int hw4 = (H * W) >> 2, W4 = W >> 2;
    const float rW4 = 1.0f / (float)(W4 > 0 ? W4 : 1), rW = 1.0f / (float)W;
    for (int64_t pl = wave; pl < planes; pl += nw) {
        const float4 *a4 = reinterpret_cast<const float4 *>(g1) + pl * hw4;
        const float4 *o4 = reinterpret_cast<const float4 *>(outv) + pl * hw4;
        float4 *r4 = reinterpret_cast<float4 *>(res) + pl * hw4;
        const float *sp = g2s + pl * (int64_t)Hs * Ws;
        for (int i = lane; i < hw4; i += 64) {
            float4 r = q8t_ld_last(a4 + i);
            float4 t = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (ROWS4) {
                const int h = small_div(i, W4, rW4), w0 = 4 * (i - h * W4);
                if (!(h & 1)) {
                    const float2 p = *reinterpret_cast<const float2 *>(sp + (h >> 1) * Ws + (w0 >> 1));
                    t.x = p.x;
                    t.z = p.y;
                }
            } else {
                float tv[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int e = 4 * i + j, h = small_div(e, W, rW), w = e - h * W;
                    tv[j] = (!(h & 1) && !(w & 1)) ? sp[(h >> 1) * Ws + (w >> 1)] : 0.0f;
                }
                t = make_float4(tv[0], tv[1], tv[2], tv[3]);
            }
            r.x = r.x + t.x; r.y = r.y + t.y; r.z = r.z + t.z; r.w = r.w + t.w;
            if (outv) {
                const float4 v = q8t_ld_last(o4 + i);
                r.x = v.x > 0.0f ? r.x : 0.0f; r.y = v.y > 0.0f ? r.y : 0.0f;
                r.z = v.z > 0.0f ? r.z : 0.0f; r.w = v.w > 0.0f ? r.w : 0.0f;
            }
            r4[i] = r;
        }
    }
}

// any stride and shape, one element per thread and sweep
__global__ __launch_bounds__(kThreads) void relu_bwd_sum_lattice_any(const float *__restrict__ g1, const float *__restrict__ g2s,
                                                                     const float *__restrict__ outv, int64_t n, int H, int W,
                                                                     int Hs, int Ws, int s, float *__restrict__ res)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
        const int64_t row = i / W, pl = row / H;
        const int w = (int)(i - row * W), h = (int)(row - pl * H);
        const float t = (h % s == 0 && w % s == 0) ? g2s[(pl * Hs + h / s) * Ws + w / s] : 0.0f;
        const float sum = g1[i] + t;
        res[i] = (!outv || outv[i] > 0.0f) ? sum : 0.0f;
    }
}

// res = out > 0 ? g1 + g2 : 0 (out nullable: no mask; g2 nullable: nothing added)
template <bool VEC>
__global__ __launch_bounds__(kThreads) void relu_bwd_sum(const float *__restrict__ g1, const float *__restrict__ g2,
                                                         const float *__restrict__ outv, int64_t n, float *__restrict__ res)
{
    if (VEC) {
        const int64_t n4 = n >> 2;
        const float4 *a4 = reinterpret_cast<const float4 *>(g1), *b4 = reinterpret_cast<const float4 *>(g2);
        const float4 *o4 = reinterpret_cast<const float4 *>(outv);
        float4 *r4 = reinterpret_cast<float4 *>(res);
        const int64_t per = (n4 + gridDim.x - 1) / gridDim.x;
        const int64_t lo = (int64_t)blockIdx.x * per, hi = min(n4, lo + per);
#pragma unroll 2
        for (int64_t i = lo + threadIdx.x; i < hi; i += kThreads) {
            float4 r = q8t_ld_last(a4 + i);
            if (g2) {
                const float4 t = q8t_ld_last(b4 + i);
                r.x = r.x + t.x; r.y = r.y + t.y; r.z = r.z + t.z; r.w = r.w + t.w;
            }
            if (outv) {
                const float4 v = q8t_ld_last(o4 + i);
                r.x = v.x > 0.0f ? r.x : 0.0f; r.y = v.y > 0.0f ? r.y : 0.0f;
                r.z = v.z > 0.0f ? r.z : 0.0f; r.w = v.w > 0.0f ? r.w : 0.0f;
            }
            r4[i] = r;
        }
        const int64_t tail = (n4 << 2) + (int64_t)blockIdx.x * kThreads + threadIdx.x;
        if (tail < n) {
            const float s = g2 ? g1[tail] + g2[tail] : g1[tail];
            res[tail] = (!outv || outv[tail] > 0.0f) ? s : 0.0f;
        }
    } else {
        const int64_t stride = (int64_t)gridDim.x * kThreads;
        for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
            const float s = g2 ? g1[i] + g2[i] : g1[i];
            res[i] = (!outv || outv[i] > 0.0f) ? s : 0.0f;
        }
    }
}

// res = (out > 0 ? g : 0) [+ other]
template <bool VEC>
__global__ __launch_bounds__(kThreads) void relu_bwd_add(const float *__restrict__ g, const float *__restrict__ outv,
                                                         const float *__restrict__ other, int64_t n, float *__restrict__ res)
{
    if (VEC) {
        const int64_t n4 = n >> 2;
        const float4 *g4 = reinterpret_cast<const float4 *>(g), *o4 = reinterpret_cast<const float4 *>(outv);
        const float4 *t4 = reinterpret_cast<const float4 *>(other);
        float4 *r4 = reinterpret_cast<float4 *>(res);
        const int64_t per = (n4 + gridDim.x - 1) / gridDim.x;
        const int64_t lo = (int64_t)blockIdx.x * per, hi = min(n4, lo + per);
#pragma unroll 2
        for (int64_t i = lo + threadIdx.x; i < hi; i += kThreads) {
            const float4 u = q8t_ld_last(g4 + i), v = q8t_ld_last(o4 + i);
            float4 r;
            r.x = v.x > 0.0f ? u.x : 0.0f; r.y = v.y > 0.0f ? u.y : 0.0f;
            r.z = v.z > 0.0f ? u.z : 0.0f; r.w = v.w > 0.0f ? u.w : 0.0f;
            if (other) {
                const float4 t = q8t_ld_last(t4 + i);
                r.x = r.x + t.x; r.y = r.y + t.y; r.z = r.z + t.z; r.w = r.w + t.w;
            }
            r4[i] = r;
        }
        const int64_t tail = (n4 << 2) + (int64_t)blockIdx.x * kThreads + threadIdx.x;
        if (tail < n) {
            const float m = outv[tail] > 0.0f ? g[tail] : 0.0f;
            res[tail] = other ? m + other[tail] : m;
        }
    } else {
        const int64_t stride = (int64_t)gridDim.x * kThreads;
        for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
            const float m = outv[i] > 0.0f ? g[i] : 0.0f;
            res[i] = other ? m + other[i] : m;
        }
    }
}

int grid_for(int64_t items, int per_thread, int cap)
{
    int64_t g = (items + (int64_t)kThreads * per_thread - 1) / ((int64_t)kThreads * per_thread);
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

constexpr int64_t kMaxElements = (int64_t)1 << 34;

}  // namespace

extern "C" {

int q8t_range_bn_relu_maxpool_fwd(const float *x, int N, int C, int H, int W, const float *gamma, const float *beta, float eps,
                                  const float *stats, float *out, uint8_t *idx, void *stream)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || (int64_t)N * H * W < 2) return Q8T_ERR_SHAPE;
    if ((int64_t)N * C * H * W > kMaxElements) return Q8T_ERR_SHAPE;
    if (!x || !stats || !out || !idx) return Q8T_ERR_NULL;
    const int P = (H - 1) / 2 + 1, Q = (W - 1) / 2 + 1;
    const int64_t planes = (int64_t)N * C;
    if (planes > 0x7FFFFFFF || (int64_t)H * W >= (1 << 22)) return Q8T_ERR_SHAPE;
    const float cn = (float)q8t_range_bn_scale((int64_t)N * H * W);
    if (W % 4 == 0 && q8t_aligned(x, 16) && q8t_aligned(out, 8) && q8t_aligned(idx, 2))
        hipLaunchKernelGGL(bn_relu_maxpool_fwd<true>, dim3((unsigned)planes), dim3(kThreads), 0, (hipStream_t)stream, x, C, H, W, P,
                           Q, stats, gamma, beta, cn, eps, out, idx);
    else
        hipLaunchKernelGGL(bn_relu_maxpool_fwd<false>, dim3((unsigned)planes), dim3(kThreads), 0, (hipStream_t)stream, x, C, H, W,
                           P, Q, stats, gamma, beta, cn, eps, out, idx);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

int q8t_maxpool_relu_bwd(const float *gpool, const uint8_t *idx, int N, int C, int H, int W, float *dy, void *stream)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return Q8T_ERR_SHAPE;
    if ((int64_t)N * C * H * W > kMaxElements) return Q8T_ERR_SHAPE;
    if (!gpool || !idx || !dy) return Q8T_ERR_NULL;
    const int P = (H - 1) / 2 + 1, Q = (W - 1) / 2 + 1;
    const int64_t planes = (int64_t)N * C;
    if (planes > 0x7FFFFFFF || (int64_t)H * W >= (1 << 22)) return Q8T_ERR_SHAPE;
    const int PQ = P * Q;
    const size_t lds = q8t_pool::lds_bytes(PQ);
    if (W % 4 == 0 && q8t_aligned(dy, 16)) {
        if (PQ % 16 == 0 && lds <= 48 * 1024 && q8t_aligned(gpool, 16) && q8t_aligned(idx, 16))
            hipLaunchKernelGGL((maxpool_relu_bwd<true, true>), dim3((unsigned)planes), dim3(kThreads), lds, (hipStream_t)stream,
                               gpool, idx, H, W, P, Q, dy);
        else
            hipLaunchKernelGGL((maxpool_relu_bwd<true, false>), dim3((unsigned)planes), dim3(kThreads), 0, (hipStream_t)stream,
                               gpool, idx, H, W, P, Q, dy);
    } else
        hipLaunchKernelGGL((maxpool_relu_bwd<false, false>), dim3((unsigned)planes), dim3(kThreads), 0, (hipStream_t)stream, gpool,
                           idx, H, W, P, Q, dy);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

size_t q8t_add_relu_quantize_workspace_size(int64_t n)
{
    (void)n;
    return sizeof(float2) * kMaxPartials;
}

int q8t_add_relu_quantize(const float *a, const float *b, int64_t n, float *out, int8_t *q_out, q8t_qparams *qp_out, void *ws,
                          void *stream)
{
    if (n <= 0 || n > kMaxElements) return Q8T_ERR_SHAPE;
    if (!a || !b || !out || (q_out && !qp_out)) return Q8T_ERR_NULL;
    if (!ws || !q8t_aligned(ws, 8)) return Q8T_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const bool vec = q8t_aligned(a, 16) && q8t_aligned(b, 16) && q8t_aligned(out, 16);
    const int grid = grid_for(vec ? (n >> 2) : n, 4, kMaxPartials);
    if (vec)
        hipLaunchKernelGGL(add_relu_fwd<true>, dim3(grid), dim3(kThreads), 0, st, a, b, n, out, (float2 *)ws);
    else
        hipLaunchKernelGGL(add_relu_fwd<false>, dim3(grid), dim3(kThreads), 0, st, a, b, n, out, (float2 *)ws);
    Q8T_LAUNCH_CHECK();
    if (!q_out) return Q8T_OK;
    return q8t_quantize8_from_partials(out, n, ws, grid, q_out, qp_out, st);
}

int q8t_range_bn_add_relu_quantize(const float *x, const float *stats, const float *gamma, const float *beta,
                                   const float *other, const float *other_stats, const float *other_gamma,
                                   const float *other_beta, int N, int C, int H, int W, float eps, float *out, int8_t *q_out,
                                   q8t_qparams *qp_out, void *ws, void *stream)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || (int64_t)N * H * W < 2) return Q8T_ERR_SHAPE;
    const int64_t n = (int64_t)N * C * H * W;
    if (n > kMaxElements || (int64_t)H * W > (1 << 30)) return Q8T_ERR_SHAPE;
    if (!x || !stats || !other || !out || (q_out && !qp_out)) return Q8T_ERR_NULL;
    if (!ws || !q8t_aligned(ws, 8)) return Q8T_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const int HW = H * W;
    const float cn = (float)q8t_range_bn_scale((int64_t)N * HW);
    const bool vec = HW % 4 == 0 && (n >> 2) < ((int64_t)1 << 32) && q8t_aligned(x, 16) && q8t_aligned(other, 16) &&
                     q8t_aligned(out, 16);
    const int grid = grid_for(vec ? (n >> 2) : n, 4, kMaxPartials);
    const TailBN bx = {stats, gamma, beta}, bo = {other_stats, other_gamma, other_beta};
    if (vec)
        hipLaunchKernelGGL(bn_add_relu_fwd<true>, dim3(grid), dim3(kThreads), 0, st, x, bx, other, bo, n, C, HW, cn, eps, out,
                           (float2 *)ws);
    else
        hipLaunchKernelGGL(bn_add_relu_fwd<false>, dim3(grid), dim3(kThreads), 0, st, x, bx, other, bo, n, C, HW, cn, eps, out,
                           (float2 *)ws);
    Q8T_LAUNCH_CHECK();
    if (!q_out) return Q8T_OK;
    return q8t_quantize8_from_partials(out, n, ws, grid, q_out, qp_out, st);
}

int q8t_relu_bwd_sum(const float *g1, const float *g2, const float *out, int64_t n, float *res, void *stream)
{
    if (n <= 0 || n > kMaxElements) return Q8T_ERR_SHAPE;
    if (!g1 || !res) return Q8T_ERR_NULL;
    const bool vec = q8t_aligned(g1, 16) && q8t_aligned(g2, 16) && q8t_aligned(out, 16) && q8t_aligned(res, 16);
    const int grid = grid_for(vec ? (n >> 2) : n, 4, 4096);
    if (vec)
        hipLaunchKernelGGL(relu_bwd_sum<true>, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream, g1, g2, out, n, res);
    else
        hipLaunchKernelGGL(relu_bwd_sum<false>, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream, g1, g2, out, n, res);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

int q8t_relu_bwd_sum_lattice(const float *g1, const float *g2s, const float *out, int N, int C, int H, int W, int stride,
                             float *res, void *stream)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || stride < 1) return Q8T_ERR_SHAPE;
    const int64_t planes = (int64_t)N * C, n = planes * H * W;
    if (n > kMaxElements || (int64_t)H * W >= (1 << 22)) return Q8T_ERR_SHAPE;
    if (!g1 || !g2s || !res) return Q8T_ERR_NULL;
    const int Hs = (H + stride - 1) / stride, Ws = (W + stride - 1) / stride;
    hipStream_t st = (hipStream_t)stream;
    const bool vec = stride == 2 && (H * W) % 4 == 0 && W % 2 == 0 && H % 2 == 0 && q8t_aligned(g1, 16) && q8t_aligned(g2s, 16) &&
                     q8t_aligned(out, 16) && q8t_aligned(res, 16);
    if (vec) {
        // a wavefront per plane and sweep
        const int64_t wgs = (planes + kThreads / 64 - 1) / (kThreads / 64);
        const dim3 grid((unsigned)(wgs < 4096 ? wgs : 4096));
        if (W % 4 == 0)
            hipLaunchKernelGGL(relu_bwd_sum_lattice2<true>, grid, dim3(kThreads), 0, st, g1, g2s, out, planes, H, W, Hs, Ws, res);
        else
            hipLaunchKernelGGL(relu_bwd_sum_lattice2<false>, grid, dim3(kThreads), 0, st, g1, g2s, out, planes, H, W, Hs, Ws, res);
    } else {
        const int grid = grid_for(n, 4, 4096);
        hipLaunchKernelGGL(relu_bwd_sum_lattice_any, dim3(grid), dim3(kThreads), 0, st, g1, g2s, out, n, H, W, Hs, Ws, stride, res);
    }
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

int q8t_relu_bwd_add(const float *g, const float *out, const float *other, int64_t n, float *res, void *stream)
{
    if (n <= 0 || n > kMaxElements) return Q8T_ERR_SHAPE;
    if (!g || !out || !res) return Q8T_ERR_NULL;
    const bool vec = q8t_aligned(g, 16) && q8t_aligned(out, 16) && q8t_aligned(res, 16) && q8t_aligned(other, 16);
    const int grid = grid_for(vec ? (n >> 2) : n, 4, 4096);
    if (vec)
        hipLaunchKernelGGL(relu_bwd_add<true>, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream, g, out, other, n, res);
    else
        hipLaunchKernelGGL(relu_bwd_add<false>, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream, g, out, other, n, res);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

}  // extern "C"

int q8t_subsample_codes(const int8_t *x, int N, int C, int H, int W, int s, int8_t *out, hipStream_t st)
{
    const int P = (H - 1) / s + 1, Q = (W - 1) / s + 1;
    const int64_t planes = (int64_t)N * C;
    const bool pairs = s == 2 && W % 8 == 0 && q8t_aligned(x, 8) && q8t_aligned(out, 4);   // then Q = W / 2 is a multiple of 4
    if (pairs)
        hipLaunchKernelGGL(subsample_codes<true>, dim3(grid_for(planes * P * (Q >> 2), 4, 4096)), dim3(kThreads), 0, st, x, planes,
                           H, W, P, Q, s, out);
    else
        hipLaunchKernelGGL(subsample_codes<false>, dim3(grid_for(planes * P * Q, 4, 4096)), dim3(kThreads), 0, st, x, planes, H, W,
                           P, Q, s, out);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}
