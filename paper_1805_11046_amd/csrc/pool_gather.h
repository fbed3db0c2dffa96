// Backward of the 3x3 / stride 2 / pad 1 max pooling of the stem as a gather: the gradient that reaches a position of
// the unpooled plane, from the pooled gradient and the byte that names each window's maximum (network plumbing, not
// from the paper).  Shared by the stand-alone pooling backward and by the Range BN backward that takes the pooled
// gradient directly; both sum the windows of a position in the same order, so their results agree bit for bit.
#pragma once
#include "q8t_common.h"

namespace q8t_pool {

// quotient n / d for n < 2^22 (positions inside one plane): float estimate + fix-up
__device__ __forceinline__ int small_div(int n, int d, float rd)
{
    int q = (int)((float)n * rd);
    const int r = n - q * d;
    q += r >= d ? 1 : 0;
    q -= r < 0 ? 1 : 0;
    return q;
}

// gradient that reaches position (h, w): an even row / column belongs to one window, an odd one to
// two; windows in the order a scatter over the pooled plane visits them (rows ascending, then columns)
__device__ __forceinline__ float bwd_at(const float *__restrict__ gp, const uint8_t *__restrict__ ip, int h, int w, int P, int Q)
{
    const int p1 = (h + 1) >> 1, p0 = p1 - (h & 1);
    const int q1 = (w + 1) >> 1, q0 = q1 - (w & 1);
    float acc = 0.0f;
    for (int p = p0; p <= p1; ++p) {
        if (p >= P) continue;
        for (int q = q0; q <= q1; ++q) {
            if (q >= Q) continue;
            const int local = 3 * (h - (2 * p - 1)) + (w - (2 * q - 1));
            if (ip[p * Q + q] == local) acc += gp[p * Q + q];
        }
    }
    return acc;
}

// the same for positions w..w+3 of row h, w = 2 * qa a multiple of 4 (the plane's width is one, so Q is even and
// qa + 1 < Q).  They meet the pooled columns qa, qa+1, qa+2 at fixed places inside their windows: w -> (qa, col 1);
// w+1 -> (qa, 2), (qa+1, 0); w+2 -> (qa+1, 1); w+3 -> (qa+1, 2), (qa+2, 0); an even row h meets pooled row h/2 at
// window row 1, an odd one rows (h-1)/2 and (h+1)/2 at window rows 2 and 0.
__device__ __forceinline__ float4 bwd_gather4(const float *gp, const uint8_t *ip, int h, int qa, int P, int Q)
{
    float4 r = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    const int np = (h & 1) ? 2 : 1;
    for (int k = 0; k < np; ++k) {
        const int p = (h >> 1) + k, i = (h & 1) ? 2 - 2 * k : 1;
        if (p >= P) break;
        const uint8_t *ir = ip + p * Q + qa;
        const float *gr = gp + p * Q + qa;
        const int ia = ir[0], ib = ir[1], ic = qa + 2 < Q ? ir[2] : 255;
        const float ga = gr[0], gb = gr[1], gc = qa + 2 < Q ? gr[2] : 0.0f;
        r.x += ia == 3 * i + 1 ? ga : 0.0f;
        r.y += ia == 3 * i + 2 ? ga : 0.0f;
        r.y += ib == 3 * i ? gb : 0.0f;
        r.z += ib == 3 * i + 1 ? gb : 0.0f;
        r.w += ib == 3 * i + 2 ? gb : 0.0f;
        r.w += ic == 3 * i ? gc : 0.0f;
    }
    return r;
}

// LDS bytes of one staged pooled plane: PQ floats, then PQ index bytes
__host__ __device__ inline size_t lds_bytes(int PQ) { return (size_t)PQ * 5; }

// copy one pooled plane and its indices into LDS (PQ a multiple of 16, both planes 16-byte aligned: wide coalesced
// loads); the caller synchronizes before the gather and before the next plane is staged
template <int THREADS>
__device__ __forceinline__ void stage_plane(const float *__restrict__ gp, const uint8_t *__restrict__ ip, int PQ, uint8_t *lds)
{
    float *sg = reinterpret_cast<float *>(lds);
    uint8_t *si = lds + (size_t)PQ * sizeof(float);
    for (int i = threadIdx.x; i < PQ / 4; i += THREADS)
        reinterpret_cast<float4 *>(sg)[i] = q8t_ld_last(reinterpret_cast<const float4 *>(gp) + i);
    for (int i = threadIdx.x; i < PQ / 16; i += THREADS)
        reinterpret_cast<uint4 *>(si)[i] = reinterpret_cast<const uint4 *>(ip)[i];
}

}  // namespace q8t_pool
