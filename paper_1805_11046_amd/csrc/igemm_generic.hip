// General int8 MFMA product kernel behind every FC call and behind the convolution shapes that
// have no specialised kernel (any stride / filter size / channel count).
//
// Section 4 of the paper: forward Y = X W, layer gradient g_{l-1} = g_l W^T (8-bit operands),
// weight gradient g_W = g_l I^T with the 16-bit copy of g_l (Sections 1, 7).
//
// One kernel, parameterised by a "problem" policy that says how a logical operand element
// A(row, kk) / B(kk, col) is fetched (row-major FC operands, im2col gathers for the convolution
// forms) and where an output element goes.  64x64 output tile per workgroup, 4 wavefronts of
// 2x2 v_mfma_i32_16x16x64_i8 tiles, operands staged through LDS with the reduction index
// contiguous.  Stored codes are signed (level - 2^(M-1)); the exact accumulator
//   sum_k (a_k - za)(b_k - zb) = sum a b - zb sum a - za sum b + Kp za zb
// is recovered in the epilogue from row / column sums kept beside the MFMA accumulators.
// A 16-bit operand is split into two signed bytes, s = 256*hi + lo + 128, and run as two int8
// products whose results are recombined in 64-bit.  Long reductions are split over blockIdx.z
// (each slice stays below the 32-bit accumulator bound) and summed in int64 by a second kernel.
#include "q8t_common.h"
#include "q8t_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int BM = 64, BN = 64, BK = 64;
constexpr int LDS_STRIDE = BK + 16;  // bytes per staged row: 16-byte aligned, conflict-free b128 reads
constexpr int kMaxSliceK = 65536;    // products per 32-bit partial accumulator (|a*b| <= 2^14)

struct QZ {
    int za, zb;  // stored zero points (zero_point - 2^(bits-1)) of the A and B operands
};

// ------------------------------------------------------------------------------------------------
// Problem policies.  kdec(kk) decodes a reduction index once per K-step into an int4 that the
// element fetchers use; rowctx / colctx decode the output row / column once per thread.
// fetchA / fetchB return the stored code, or the operand's stored zero point where the logical
// element is padding or outside the matrix (so that it contributes exactly nothing).
// ------------------------------------------------------------------------------------------------

// FC forward: rows m, cols n, kk = k.  A = X[M,K], B = W[K,N].
struct FcFwd {
    const int8_t *X, *W;
    int M, N, K;
    float *y;
    int32_t *acc;
    static constexpr bool A16 = false, A_KFAST = true, B_KFAST = false;
    __device__ int rows() const { return M; }
    __device__ int cols() const { return N; }
    __device__ int red() const { return K; }
    __device__ int4 kdec(int kk) const { return make_int4(kk, kk < K, 0, 0); }
    __device__ int4 rowctx(int r) const { return make_int4(r, r < M, 0, 0); }
    __device__ int4 colctx(int c) const { return make_int4(c, c < N, 0, 0); }
    __device__ int fetchA(const int4 &r, const int4 &k, int z) const
    {
        return (r.y && k.y) ? (int)X[(int64_t)r.x * K + k.x] : z;
    }
    __device__ int fetchB(const int4 &c, const int4 &k, int z) const
    {
        return (c.y && k.y) ? (int)W[(int64_t)k.x * N + c.x] : z;
    }
    __device__ int64_t out_index(int r, int c) const { return (int64_t)r * N + c; }
};

// FC layer gradient: rows m, cols k, kk = n.  A = dY[M,N], B(kk,col) = W[col,kk].
struct FcDgrad {
    const int8_t *G, *W;
    int M, N, K;
    static constexpr bool A16 = false, A_KFAST = true, B_KFAST = true;
    __device__ int rows() const { return M; }
    __device__ int cols() const { return K; }
    __device__ int red() const { return N; }
    __device__ int4 kdec(int kk) const { return make_int4(kk, kk < N, 0, 0); }
    __device__ int4 rowctx(int r) const { return make_int4(r, r < M, 0, 0); }
    __device__ int4 colctx(int c) const { return make_int4(c, c < K, 0, 0); }
    __device__ int fetchA(const int4 &r, const int4 &k, int z) const
    {
        return (r.y && k.y) ? (int)G[(int64_t)r.x * N + k.x] : z;
    }
    __device__ int fetchB(const int4 &c, const int4 &k, int z) const
    {
        return (c.y && k.y) ? (int)W[(int64_t)c.x * N + k.x] : z;
    }
    __device__ int64_t out_index(int r, int c) const { return (int64_t)r * K + c; }
};

// FC weight gradient, computed transposed so that the 16-bit operand is A:
// rows n, cols k, kk = m.  A(row,kk) = dY16[kk,row], B(kk,col) = X[kk,col]; output dW[col,row].
struct FcWgrad {
    const int16_t *G16;
    const int8_t *X;
    int M, N, K;
    static constexpr bool A16 = true, A_KFAST = false, B_KFAST = false;
    __device__ int rows() const { return N; }
    __device__ int cols() const { return K; }
    __device__ int red() const { return M; }
    __device__ int4 kdec(int kk) const { return make_int4(kk, kk < M, 0, 0); }
    __device__ int4 rowctx(int r) const { return make_int4(r, r < N, 0, 0); }
    __device__ int4 colctx(int c) const { return make_int4(c, c < K, 0, 0); }
    __device__ int fetchA(const int4 &r, const int4 &k, int z) const
    {
        return (r.y && k.y) ? (int)G16[(int64_t)k.x * N + r.x] : z;
    }
    __device__ int fetchB(const int4 &c, const int4 &k, int z) const
    {
        return (c.y && k.y) ? (int)X[(int64_t)k.x * K + c.x] : z;
    }
    __device__ int64_t out_index(int r, int c) const { return (int64_t)c * N + r; }
};

struct ConvGeom {
    int N, C, H, W, K, R, S, stride, pad, P, Q;
};

// conv forward: rows (b,p,q), cols kout, kk = (c,r,s)
struct ConvFwd {
    const int8_t *X, *Wt;
    ConvGeom g;
    static constexpr bool A16 = false, A_KFAST = false, B_KFAST = true;
    __device__ int rows() const { return g.N * g.P * g.Q; }
    __device__ int cols() const { return g.K; }
    __device__ int red() const { return g.C * g.R * g.S; }
    __device__ int4 kdec(int kk) const
    {
        const int rs = g.R * g.S;
        const int c = kk / rs, t = kk - c * rs, r = t / g.S, s = t - r * g.S;
        return make_int4(c, r, s, kk < g.C * rs);
    }
    __device__ int4 rowctx(int m) const
    {
        const int pq = g.P * g.Q;
        const int b = m / pq, t = m - b * pq, p = t / g.Q, q = t - p * g.Q;
        return make_int4(b, p * g.stride - g.pad, q * g.stride - g.pad, m < g.N * pq);
    }
    __device__ int4 colctx(int c) const { return make_int4(c, c < g.K, 0, 0); }
    __device__ int fetchA(const int4 &r, const int4 &k, int z) const
    {
        const int h = r.y + k.y, w = r.z + k.z;
        const bool ok = r.w && k.w && h >= 0 && h < g.H && w >= 0 && w < g.W;
        return ok ? (int)X[(((int64_t)r.x * g.C + k.x) * g.H + h) * g.W + w] : z;
    }
    __device__ int fetchB(const int4 &c, const int4 &k, int z) const
    {
        return (c.y && k.w) ? (int)Wt[(((int64_t)c.x * g.C + k.x) * g.R + k.y) * g.S + k.z] : z;
    }
    __device__ int64_t out_index(int m, int c) const
    {
        const int pq = g.P * g.Q;
        const int b = m / pq, t = m - b * pq;
        return ((int64_t)b * g.K + c) * pq + t;
    }
};

// conv layer gradient: rows (b,h,w), cols c, kk = (kout,r,s)
struct ConvDgrad {
    const int8_t *G, *Wt;
    ConvGeom g;
    static constexpr bool A16 = false, A_KFAST = false, B_KFAST = true;
    __device__ int rows() const { return g.N * g.H * g.W; }
    __device__ int cols() const { return g.C; }
    __device__ int red() const { return g.K * g.R * g.S; }
    __device__ int4 kdec(int kk) const
    {
        const int rs = g.R * g.S;
        const int k = kk / rs, t = kk - k * rs, r = t / g.S, s = t - r * g.S;
        return make_int4(k, r, s, kk < g.K * rs);
    }
    __device__ int4 rowctx(int m) const
    {
        const int hw = g.H * g.W;
        const int b = m / hw, t = m - b * hw, h = t / g.W, w = t - h * g.W;
        return make_int4(b, h + g.pad, w + g.pad, m < g.N * hw);
    }
    __device__ int4 colctx(int c) const { return make_int4(c, c < g.C, 0, 0); }
    __device__ int fetchA(const int4 &r, const int4 &k, int z) const
    {
        const int hp = r.y - k.y, wq = r.z - k.z;
        if (!(r.w && k.w) || hp < 0 || wq < 0) return z;
        const int p = hp / g.stride, q = wq / g.stride;
        if (p * g.stride != hp || q * g.stride != wq || p >= g.P || q >= g.Q) return z;
        return (int)G[(((int64_t)r.x * g.K + k.x) * g.P + p) * g.Q + q];
    }
    __device__ int fetchB(const int4 &c, const int4 &k, int z) const
    {
        return (c.y && k.w) ? (int)Wt[(((int64_t)k.x * g.C + c.x) * g.R + k.y) * g.S + k.z] : z;
    }
    __device__ int64_t out_index(int m, int c) const
    {
        const int hw = g.H * g.W;
        const int b = m / hw, t = m - b * hw;
        return ((int64_t)b * g.C + c) * hw + t;
    }
};

// conv weight gradient: rows kout, cols (c,r,s), kk = (b,p,q); A = 16-bit gradient copy
struct ConvWgrad {
    const int16_t *G16;
    const int8_t *X;
    ConvGeom g;
    static constexpr bool A16 = true, A_KFAST = true, B_KFAST = true;
    __device__ int rows() const { return g.K; }
    __device__ int cols() const { return g.C * g.R * g.S; }
    __device__ int red() const { return g.N * g.P * g.Q; }
    __device__ int4 kdec(int kk) const
    {
        const int pq = g.P * g.Q;
        const int b = kk / pq, t = kk - b * pq, p = t / g.Q, q = t - p * g.Q;
        return make_int4(b, p, q, kk < g.N * pq);
    }
    __device__ int4 rowctx(int r) const { return make_int4(r, r < g.K, 0, 0); }
    __device__ int4 colctx(int col) const
    {
        const int rs = g.R * g.S;
        const int c = col / rs, t = col - c * rs, r = t / g.S, s = t - r * g.S;
        return make_int4(c, r - g.pad, s - g.pad, col < g.C * rs);
    }
    __device__ int fetchA(const int4 &r, const int4 &k, int z) const
    {
        return (r.y && k.w) ? (int)G16[(((int64_t)k.x * g.K + r.x) * g.P + k.y) * g.Q + k.z] : z;
    }
    __device__ int fetchB(const int4 &c, const int4 &k, int z) const
    {
        const int h = k.y * g.stride + c.y, w = k.z * g.stride + c.z;
        const bool ok = c.w && k.w && h >= 0 && h < g.H && w >= 0 && w < g.W;
        return ok ? (int)X[(((int64_t)k.x * g.C + c.x) * g.H + h) * g.W + w] : z;
    }
    __device__ int64_t out_index(int r, int col) const { return (int64_t)r * cols() + col; }
};

// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t pack_bytes(int a, int b, int c, int d)
{
    return (uint32_t)(a & 255) | ((uint32_t)(b & 255) << 8) | ((uint32_t)(c & 255) << 16) |
           ((uint32_t)(d & 255) << 24);
}

// Output of one slice of the reduction.  splits == 1: final values are written directly.
// splits > 1: 64-bit partial accumulators go to `partial[z][rows*cols]` for the reduce kernel.
struct Sink {
    float *out_f;       // nullable
    void *out_acc;      // nullable; int32 (8-bit A) or int64 (16-bit A)
    int64_t *partial;   // used when splits > 1
    int splits;
    int slice_k;        // reduction elements per slice (multiple of BK)
};

template <class P>
__global__ __launch_bounds__(kThreads) void igemm_generic(P prob, const q8t_qparams *__restrict__ qpa,
                                                          const q8t_qparams *__restrict__ qpb, Sink sink)
{
    __shared__ __attribute__((aligned(16))) uint8_t As[2][BM * LDS_STRIDE];
    __shared__ __attribute__((aligned(16))) uint8_t Bs[BN * LDS_STRIDE];
    __shared__ int4 ktab[BK];
    __shared__ int rsum[2][BM];
    __shared__ int csum[BN];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
    const int za = qpa->zero_point - (1 << (qpa->bits - 1));
    const int zb = qpb->zero_point - (1 << (qpb->bits - 1));
    const float sc = qpa->scale * qpb->scale;

    const int red = prob.red();
    const int k_begin = blockIdx.z * sink.slice_k;
    const int k_end = min(red, k_begin + sink.slice_k);

    // which 16-byte chunk of the staged tiles this thread fills
    const int a_row = P::A_KFAST ? (tid >> 2) : (tid & 63), a_kc = P::A_KFAST ? (tid & 3) : (tid >> 6);
    const int b_col = P::B_KFAST ? (tid >> 2) : (tid & 63), b_kc = P::B_KFAST ? (tid & 3) : (tid >> 6);
    const int4 rctx = prob.rowctx(m0 + a_row);
    const int4 cctx = prob.colctx(n0 + b_col);

    if (tid < BM) { rsum[0][tid] = 0; rsum[1][tid] = 0; }
    if (tid < BN) csum[tid] = 0;

    v4i acc[2][2][2];  // [byte plane][mt][nt]
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[h][i][j] = (v4i){0, 0, 0, 0};

    int sumA0 = 0, sumA1 = 0, sumB = 0;
    int ksteps = 0;
    for (int kt = k_begin; kt < k_end; kt += BK, ++ksteps) {
        if (tid < BK) {
            int4 d = prob.kdec(kt + tid);
            if (kt + tid >= k_end) d = prob.kdec(red);  // beyond this slice: decode as "invalid"
            ktab[tid] = d;
        }
        __syncthreads();
        {   // stage A
            uint32_t w0[4], w1[4];
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                int v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = prob.fetchA(rctx, ktab[a_kc * 16 + e4 * 4 + e], za);
                if (P::A16) {
                    int hi[4], lo[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        hi[e] = v[e] >> 8;
                        lo[e] = (v[e] & 255) - 128;
                        sumA0 += hi[e];
                        sumA1 += lo[e];
                    }
                    w0[e4] = pack_bytes(hi[0], hi[1], hi[2], hi[3]);
                    w1[e4] = pack_bytes(lo[0], lo[1], lo[2], lo[3]);
                } else {
                    sumA0 += v[0] + v[1] + v[2] + v[3];
                    w0[e4] = pack_bytes(v[0], v[1], v[2], v[3]);
                }
            }
            *reinterpret_cast<uint4 *>(&As[0][a_row * LDS_STRIDE + a_kc * 16]) = make_uint4(w0[0], w0[1], w0[2], w0[3]);
            if (P::A16)
                *reinterpret_cast<uint4 *>(&As[1][a_row * LDS_STRIDE + a_kc * 16]) = make_uint4(w1[0], w1[1], w1[2], w1[3]);
        }
        {   // stage B
            uint32_t w0[4];
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                int v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = prob.fetchB(cctx, ktab[b_kc * 16 + e4 * 4 + e], zb);
                sumB += v[0] + v[1] + v[2] + v[3];
                w0[e4] = pack_bytes(v[0], v[1], v[2], v[3]);
            }
            *reinterpret_cast<uint4 *>(&Bs[b_col * LDS_STRIDE + b_kc * 16]) = make_uint4(w0[0], w0[1], w0[2], w0[3]);
        }
        __syncthreads();
        v4i bf[2];
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
            bf[nt] = *reinterpret_cast<const v4i *>(&Bs[(wn * 32 + nt * 16 + (lane & 15)) * LDS_STRIDE + (lane >> 4) * 16]);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            const int off = (wm * 32 + mt * 16 + (lane & 15)) * LDS_STRIDE + (lane >> 4) * 16;
            const v4i a0 = *reinterpret_cast<const v4i *>(&As[0][off]);
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
                acc[0][mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a0, bf[nt], acc[0][mt][nt], 0, 0, 0);
            if (P::A16) {
                const v4i a1 = *reinterpret_cast<const v4i *>(&As[1][off]);
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
                    acc[1][mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a1, bf[nt], acc[1][mt][nt], 0, 0, 0);
            }
        }
    }
    __syncthreads();
    atomicAdd(&rsum[0][a_row], sumA0);
    if (P::A16) atomicAdd(&rsum[1][a_row], sumA1);
    atomicAdd(&csum[b_col], sumB);
    __syncthreads();

    const int Kp = ksteps * BK;  // staged reduction length, padding included
    const int rows = prob.rows(), cols = prob.cols();
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int lr = wm * 32 + mt * 16 + (lane >> 4) * 4 + j, lc = wn * 32 + nt * 16 + (lane & 15);
                const int r = m0 + lr, c = n0 + lc;
                if (r >= rows || c >= cols) continue;
                int64_t v;
                if (P::A16) {
                    const int64_t ca = 128 - za;
                    v = 256 * (int64_t)acc[0][mt][nt][j] + (int64_t)acc[1][mt][nt][j] + ca * (int64_t)csum[lc] -
                        (int64_t)zb * (256 * (int64_t)rsum[0][lr] + (int64_t)rsum[1][lr] + ca * (int64_t)Kp);
                } else {
                    v = (int64_t)acc[0][mt][nt][j] - (int64_t)zb * rsum[0][lr] - (int64_t)za * csum[lc] +
                        (int64_t)Kp * za * zb;
                }
                const int64_t oi = prob.out_index(r, c);
                if (sink.splits > 1) {
                    sink.partial[(int64_t)blockIdx.z * rows * cols + oi] = v;
                } else if (P::A16) {
                    if (sink.out_acc) ((int64_t *)sink.out_acc)[oi] = v;
                    if (sink.out_f) sink.out_f[oi] = (float)((double)v * (double)sc);
                } else {
                    if (sink.out_acc) ((int32_t *)sink.out_acc)[oi] = (int32_t)v;
                    if (sink.out_f) sink.out_f[oi] = sc * (float)(int32_t)v;
                }
            }
}

// sums the slices in int64 and writes the final outputs
__global__ __launch_bounds__(kThreads) void splitk_reduce(const int64_t *__restrict__ partial, int splits,
                                                          int64_t count, const q8t_qparams *__restrict__ qpa,
                                                          const q8t_qparams *__restrict__ qpb, int a16,
                                                          float *__restrict__ out_f, void *__restrict__ out_acc)
{
    const float sc = qpa->scale * qpb->scale;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < count; i += stride) {
        int64_t v = 0;
        for (int z = 0; z < splits; ++z) v += partial[(int64_t)z * count + i];
        if (a16) {
            if (out_acc) ((int64_t *)out_acc)[i] = v;
            if (out_f) out_f[i] = (float)((double)v * (double)sc);
        } else {
            if (out_acc) ((int32_t *)out_acc)[i] = (int32_t)v;
            if (out_f) out_f[i] = sc * (float)(int32_t)v;
        }
    }
}

struct Plan {
    int splits, slice_k;
};

Plan plan_for(int64_t rows, int64_t cols, int64_t red)
{
    Plan p;
    const int64_t tiles = ((rows + BM - 1) / BM) * ((cols + BN - 1) / BN);
    int64_t want = 1;
    if (tiles < 512) want = (1024 + tiles - 1) / tiles;   // fill the chip when the output is small
    int64_t slice = (red + want - 1) / want;
    if (slice > kMaxSliceK) slice = kMaxSliceK;
    if (slice < 4 * BK) slice = 4 * BK;
    slice = (slice + BK - 1) / BK * BK;
    p.slice_k = (int)slice;
    p.splits = (int)((red + slice - 1) / slice);
    if (p.splits < 1) p.splits = 1;
    return p;
}

size_t ws_for(int64_t rows, int64_t cols, int64_t red)
{
    const Plan p = plan_for(rows, cols, red);
    return p.splits > 1 ? (size_t)p.splits * rows * cols * sizeof(int64_t) : 0;
}

template <class P>
int run(const P &prob, int64_t rows, int64_t cols, int64_t red, const q8t_qparams *qa, const q8t_qparams *qb,
        float *out_f, void *out_acc, void *ws, hipStream_t st)
{
    const Plan p = plan_for(rows, cols, red);
    if (p.splits > 1 && (!ws || !q8t_aligned(ws, 8))) return Q8T_ERR_WORKSPACE;
    Sink sink;
    sink.out_f = out_f;
    sink.out_acc = out_acc;
    sink.partial = (int64_t *)ws;
    sink.splits = p.splits;
    sink.slice_k = p.slice_k;
    const int64_t gy = (rows + BM - 1) / BM, gx = (cols + BN - 1) / BN;
    if (gy > 0x7fffffff || gx > 65535 || p.splits > 65535) return Q8T_ERR_SHAPE;
    hipLaunchKernelGGL((igemm_generic<P>), dim3((unsigned)gy, (unsigned)gx, (unsigned)p.splits), dim3(kThreads), 0,
                       st, prob, qa, qb, sink);
    Q8T_LAUNCH_CHECK();
    if (p.splits > 1) {
        const int64_t count = rows * cols;
        int64_t g = (count + kThreads - 1) / kThreads;
        if (g > 4096) g = 4096;
        hipLaunchKernelGGL(splitk_reduce, dim3((unsigned)g), dim3(kThreads), 0, st, (const int64_t *)ws, p.splits,
                           count, qa, qb, P::A16 ? 1 : 0, out_f, out_acc);
        Q8T_LAUNCH_CHECK();
    }
    return Q8T_OK;
}

constexpr int kMaxRed32 = 33025;  // 255*255*K < 2^31

bool geom_ok(const q8t_conv_desc *d, ConvGeom &g)
{
    if (!d) return false;
    if (d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0 ||
        d->stride <= 0 || d->pad < 0)
        return false;
    if (d->H + 2 * d->pad < d->R || d->W + 2 * d->pad < d->S) return false;
    g.N = d->N; g.C = d->C; g.H = d->H; g.W = d->W; g.K = d->K; g.R = d->R; g.S = d->S;
    g.stride = d->stride; g.pad = d->pad;
    g.P = (d->H + 2 * d->pad - d->R) / d->stride + 1;
    g.Q = (d->W + 2 * d->pad - d->S) / d->stride + 1;
    const int64_t lim = (int64_t)1 << 31;
    if ((int64_t)g.N * g.C * g.H * g.W >= lim || (int64_t)g.N * g.K * g.P * g.Q >= lim ||
        (int64_t)g.K * g.C * g.R * g.S >= lim)
        return false;
    return true;
}

}  // namespace

// entry points used by the dispatchers in api.hip
int q8t_generic_fc(int which, const void *a, const q8t_qparams *qa, const void *b, const q8t_qparams *qb, int M,
                   int N, int K, float *out_f, void *out_acc, void *ws, hipStream_t st)
{
    if (which == 0) {
        FcFwd p{(const int8_t *)a, (const int8_t *)b, M, N, K, nullptr, nullptr};
        return run(p, M, N, K, qa, qb, out_f, out_acc, ws, st);
    } else if (which == 1) {
        FcDgrad p{(const int8_t *)a, (const int8_t *)b, M, N, K};
        return run(p, M, K, N, qa, qb, out_f, out_acc, ws, st);
    }
    FcWgrad p{(const int16_t *)a, (const int8_t *)b, M, N, K};
    return run(p, N, K, M, qa, qb, out_f, out_acc, ws, st);
}

size_t q8t_generic_fc_ws(int which, int M, int N, int K)
{
    if (which == 0) return ws_for(M, N, K);
    if (which == 1) return ws_for(M, K, N);
    return ws_for(N, K, M);
}

int q8t_generic_conv(int which, const q8t_conv_desc *d, const void *a, const q8t_qparams *qa, const void *b,
                     const q8t_qparams *qb, float *out_f, void *out_acc, void *ws, hipStream_t st)
{
    ConvGeom g;
    if (!geom_ok(d, g)) return Q8T_ERR_SHAPE;
    if (which == 0) {
        ConvFwd p{(const int8_t *)a, (const int8_t *)b, g};
        return run(p, (int64_t)g.N * g.P * g.Q, g.K, (int64_t)g.C * g.R * g.S, qa, qb, out_f, out_acc, ws, st);
    } else if (which == 1) {
        ConvDgrad p{(const int8_t *)a, (const int8_t *)b, g};
        return run(p, (int64_t)g.N * g.H * g.W, g.C, (int64_t)g.K * g.R * g.S, qa, qb, out_f, out_acc, ws, st);
    }
    ConvWgrad p{(const int16_t *)a, (const int8_t *)b, g};
    return run(p, g.K, (int64_t)g.C * g.R * g.S, (int64_t)g.N * g.P * g.Q, qa, qb, out_f, out_acc, ws, st);
}

size_t q8t_generic_conv_ws(int which, const q8t_conv_desc *d)
{
    ConvGeom g;
    if (!geom_ok(d, g)) return 0;
    if (which == 0) return ws_for((int64_t)g.N * g.P * g.Q, g.K, (int64_t)g.C * g.R * g.S);
    if (which == 1) return ws_for((int64_t)g.N * g.H * g.W, g.C, (int64_t)g.K * g.R * g.S);
    return ws_for(g.K, (int64_t)g.C * g.R * g.S, (int64_t)g.N * g.P * g.Q);
}

int q8t_conv_reduction_check(int which, const q8t_conv_desc *d)
{
    ConvGeom g;
    if (!geom_ok(d, g)) return Q8T_ERR_SHAPE;
    if (which == 0 && (int64_t)g.C * g.R * g.S > kMaxRed32) return Q8T_ERR_OVERFLOW;
    if (which == 1 && (int64_t)g.K * g.R * g.S > kMaxRed32) return Q8T_ERR_OVERFLOW;
    return Q8T_OK;
}
