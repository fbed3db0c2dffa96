// Ternarized back-propagation pieces (appendix "Additional Experiments" of the paper): stochastic
// ternarization of a gradient, binarization, a product of +-1 matrices by XNOR + population count,
// and the weight gradient by multiple stochastic ternarization sampling (Algorithm 1).
//
// The paper names these operations without defining them; the readings are
//   StcTern(g)_i = sign(g_i) with probability |g_i| / max|g|, else 0   (times max|g|: unbiased)
//   binarized x  = +1 for x >= 0, -1 otherwise
// and the random draw is 16 bits of the library's counter-based generator keyed by (seed, flat
// index): kept iff fl32(fl32(|g_i| * fl32(1/max|g|)) * 65536) > r + 0.5.
#include "q8t_common.h"
#include "q8t_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kMaxPartials = 1024;
constexpr int64_t kMaxElements = (int64_t)1 << 34;

__device__ __forceinline__ float block_max(float v, float *smem)
{
    v = wave_reduce(v, OpMax());
    if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = smem[0];
    for (int w = 1; w < kThreads / 64; ++w) r = fmaxf(r, smem[w]);
    __syncthreads();
    return r;
}

// pass 1: max |x| per workgroup (every workgroup streams one contiguous slice)
__global__ __launch_bounds__(kThreads) void absmax_partials(const float *__restrict__ x, int64_t n, float *__restrict__ partials)
{
    __shared__ float smem[kThreads / 64];
    const int64_t per = (n + gridDim.x - 1) / gridDim.x;
    const int64_t lo = (int64_t)blockIdx.x * per, hi = min(n, lo + per);
    float mx = 0.0f;
    for (int64_t i = lo + threadIdx.x; i < hi; i += kThreads) mx = fmaxf(mx, fabsf(x[i]));
    mx = block_max(mx, smem);
    if (threadIdx.x == 0) partials[blockIdx.x] = mx;
}

__device__ __forceinline__ float fold_absmax(const float *__restrict__ partials, int np, float *smem)
{
    float mx = 0.0f;
    for (int i = threadIdx.x; i < np; i += kThreads) mx = fmaxf(mx, partials[i]);
    return block_max(mx, smem);
}

// code of one element: separate multiplies (the file is built without fp contraction)
__device__ __forceinline__ int tern_code(float x, float inv, uint32_t r16)
{
    const float p = fabsf(x) * inv;
    const float lhs = p * 65536.0f;
    const float rhs = (float)r16 + 0.5f;
    return lhs > rhs ? (x < 0.0f ? -1 : 1) : 0;
}

// pass 2: every workgroup folds the partial maxima itself (same value everywhere), then ternarizes
__global__ __launch_bounds__(kThreads) void ternarize_apply(const float *__restrict__ x, int64_t n, uint32_t seed_lo,
                                                            uint32_t seed_hi, const float *__restrict__ partials, int np,
                                                            int8_t *__restrict__ t, float *__restrict__ scale_out)
{
    __shared__ float smem[kThreads / 64];
    const float s = fold_absmax(partials, np, smem);
    if (blockIdx.x == 0 && threadIdx.x == 0) *scale_out = s;
    const float inv = s == 0.0f ? 0.0f : 1.0f / s;      // all-zero tensor: every code 0
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride)
        t[i] = (int8_t)tern_code(x[i], inv, rng_r16(i, seed_lo, seed_hi));
}

__global__ __launch_bounds__(kThreads) void binarize_kernel(const float *__restrict__ x, int64_t n, int8_t *__restrict__ codes)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride)
        codes[i] = (int8_t)(x[i] >= 0.0f ? 1 : -1);
}

// one thread per output word; nr bit rows of nc bits
__global__ __launch_bounds__(kThreads) void pack_bits_kernel(const int8_t *__restrict__ codes, int rows, int cols, int transpose,
                                                             uint32_t *__restrict__ out)
{
    const int nr = transpose ? cols : rows, nc = transpose ? rows : cols;
    const int words = (nc + 31) / 32;
    const int64_t total = (int64_t)nr * words;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t o = (int64_t)blockIdx.x * kThreads + threadIdx.x; o < total; o += stride) {
        // transposed: neighbouring threads take neighbouring matrix columns (coalesced reads)
        const int r = transpose ? (int)(o % nr) : (int)(o / words);
        const int w = transpose ? (int)(o / nr) : (int)(o % words);
        uint32_t v = 0;
        for (int j = 0; j < 32; ++j) {
            const int c = 32 * w + j;
            if (c >= nc) break;
            const int8_t code = transpose ? codes[(int64_t)c * cols + r] : codes[(int64_t)r * cols + c];
            if (code > 0) v |= 1u << j;
        }
        out[(int64_t)r * words + w] = v;
    }
}

// y[m][n] = sum_k a[m][k] w[n][k] over +-1 values = 2 * popcount(xnor) - K, pad bits (0 in both) taken off.
// 64 x 64 results per workgroup, 4 x 4 per thread, bit rows staged through LDS 32 words at a time.
constexpr int XT = 64, XW = 32;
__global__ __launch_bounds__(kThreads) void xnor_gemm_kernel(const uint32_t *__restrict__ a, const uint32_t *__restrict__ w, int M,
                                                             int N, int K, int32_t *__restrict__ y)
{
    __shared__ uint32_t sa[XT][XW + 1], sw[XT][XW + 1];
    const int words = (K + 31) / 32;
    const int m0 = blockIdx.y * XT, n0 = blockIdx.x * XT;
    const int tm = threadIdx.x >> 4, tn = threadIdx.x & 15;
    int acc[4][4] = {};
    for (int w0 = 0; w0 < words; w0 += XW) {
        for (int i = threadIdx.x; i < XT * XW; i += kThreads) {
            const int r = i / XW, c = i % XW;
            sa[r][c] = (m0 + r < M && w0 + c < words) ? a[(int64_t)(m0 + r) * words + w0 + c] : 0u;
            sw[r][c] = (n0 + r < N && w0 + c < words) ? w[(int64_t)(n0 + r) * words + w0 + c] : 0u;
        }
        __syncthreads();
        const int lim = min(XW, words - w0);
        for (int c = 0; c < lim; ++c) {
            uint32_t av[4], wv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                av[i] = sa[tm + 16 * i][c];
                wv[i] = sw[tn + 16 * i][c];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] += __popc(~(av[i] ^ wv[j]));
        }
        __syncthreads();
    }
    const int pad = 32 * words - K;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = m0 + tm + 16 * i, n = n0 + tn + 16 * j;
            if (m < M && n < N) y[(int64_t)m * N + n] = 2 * (acc[i][j] - pad) - K;
        }
}

// Algorithm 1 for a fully connected layer, one kernel: dW[k][n] = max|g| / S * sum_s sum_m a[m][k] * t_s[m][n].
// A workgroup owns 64 x 64 results; per sample and per 64 rows m it stages the codes of a (transposed:
// the reduction index must be contiguous per lane) and ternarizes its 64 x 64 patch of g on the way
// into LDS with the sample's seed, then multiplies on int8 MFMA (codes -1, 0, +1 are exact int8
// values); the int32 accumulators hold the sum over all samples (|acc| <= S * M).
constexpr int TW = 64;
constexpr int TPITCH = 80;   // LDS bytes per staged row of 64 codes (16-byte aligned, conflict-free fragment reads)
__global__ __launch_bounds__(kThreads) void tern_wgrad_multi_kernel(const float *__restrict__ g, const int8_t *__restrict__ a, int M,
                                                                    int N, int K, int S, uint32_t seed_lo, uint32_t seed_hi,
                                                                    const float *__restrict__ partials, int np,
                                                                    float *__restrict__ dw, int64_t *__restrict__ acc_out)
{
    __shared__ float smem[kThreads / 64];
    __shared__ __attribute__((aligned(16))) int8_t sa[TW * TPITCH], st[TW * TPITCH];   // [k][m], [n][m]
    const float s = fold_absmax(partials, np, smem);
    const float inv = s == 0.0f ? 0.0f : 1.0f / s;
    const int k0 = blockIdx.y * TW, n0 = blockIdx.x * TW;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, kb = lane >> 4;
    v4i acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = (v4i){0, 0, 0, 0};
    for (int smp = 0; smp < S; ++smp) {
        // seed + smp as a 64-bit sum
        const uint32_t lo = seed_lo + (uint32_t)smp, hi = seed_hi + (lo < seed_lo ? 1u : 0u);
        for (int m0 = 0; m0 < M; m0 += TW) {
            __syncthreads();
            for (int i = threadIdx.x; i < TW * TW; i += kThreads) {
                const int mm = i / TW, c = i % TW;          // neighbouring threads: neighbouring columns of a row (coalesced)
                const int m = m0 + mm;
                int8_t av = 0, tv = 0;
                if (m < M) {
                    if (k0 + c < K) av = a[(int64_t)m * K + k0 + c];
                    if (n0 + c < N) {
                        const int64_t idx = (int64_t)m * N + n0 + c;
                        tv = (int8_t)tern_code(g[idx], inv, rng_r16(idx, lo, hi));
                    }
                }
                sa[c * TPITCH + mm] = av;
                st[c * TPITCH + mm] = tv;
            }
            __syncthreads();
            const v4i fa = *reinterpret_cast<const v4i *>(&sa[(wave * 16 + l16) * TPITCH + kb * 16]);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const v4i fb = *reinterpret_cast<const v4i *>(&st[(j * 16 + l16) * TPITCH + kb * 16]);
                acc[j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa, fb, acc[j], 0, 0, 0);
            }
        }
    }
    // accumulator layout: lane (column l16, kb) holds rows 4*kb + i of its 16 x 16 tile
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int k = k0 + wave * 16 + kb * 4 + i, n = n0 + j * 16 + l16;
            if (k < K && n < N) {
                const int64_t v = acc[j][i];
                if (acc_out) acc_out[(int64_t)k * N + n] = v;
                if (dw) dw[(int64_t)k * N + n] = (float)((double)v * (double)s / (double)S);
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

int launch_absmax(const float *x, int64_t n, float *partials, hipStream_t st)
{
    if (n == 0) return 0;
    const int grid = grid_for(n, 16, kMaxPartials);
    hipLaunchKernelGGL(absmax_partials, dim3(grid), dim3(kThreads), 0, st, x, n, partials);
    return grid;
}

}  // namespace

extern "C" {

size_t q8t_ternarize_workspace_size(int64_t n)
{
    (void)n;
    return sizeof(float) * kMaxPartials;
}

int q8t_ternarize(const float *g, int64_t n, uint64_t seed, int8_t *t_out, float *scale_out, void *ws, void *stream)
{
    if (n < 0 || n > kMaxElements) return Q8T_ERR_SHAPE;
    if (!scale_out || (n > 0 && (!g || !t_out))) return Q8T_ERR_NULL;
    if (!ws || !q8t_aligned(ws, 4)) return Q8T_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const int np = launch_absmax(g, n, (float *)ws, st);
    Q8T_LAUNCH_CHECK();
    hipLaunchKernelGGL(ternarize_apply, dim3(grid_for(n, 8, 2048)), dim3(kThreads), 0, st, g, n, (uint32_t)seed,
                       (uint32_t)(seed >> 32), (const float *)ws, np, t_out, scale_out);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

int q8t_binarize(const float *x, int64_t n, int8_t *codes, void *stream)
{
    if (n < 0 || n > kMaxElements) return Q8T_ERR_SHAPE;
    if (n > 0 && (!x || !codes)) return Q8T_ERR_NULL;
    if (n == 0) return Q8T_OK;
    hipLaunchKernelGGL(binarize_kernel, dim3(grid_for(n, 8, 4096)), dim3(kThreads), 0, (hipStream_t)stream, x, n, codes);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

int q8t_pack_bits(const int8_t *codes, int rows, int cols, int transpose, uint32_t *out, void *stream)
{
    if (rows <= 0 || cols <= 0 || (int64_t)rows * cols >= ((int64_t)1 << 31)) return Q8T_ERR_SHAPE;
    if (!codes || !out) return Q8T_ERR_NULL;
    const int nr = transpose ? cols : rows, nc = transpose ? rows : cols;
    const int64_t total = (int64_t)nr * ((nc + 31) / 32);
    hipLaunchKernelGGL(pack_bits_kernel, dim3(grid_for(total, 1, 4096)), dim3(kThreads), 0, (hipStream_t)stream, codes, rows,
                       cols, transpose ? 1 : 0, out);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

int q8t_xnor_gemm(const uint32_t *a_bits, const uint32_t *w_bits, int M, int N, int K, int32_t *y, void *stream)
{
    if (M <= 0 || N <= 0 || K <= 0 || (int64_t)M * N >= ((int64_t)1 << 31)) return Q8T_ERR_SHAPE;
    if (!a_bits || !w_bits || !y) return Q8T_ERR_NULL;
    if ((N + XT - 1) / XT > 65535 || (M + XT - 1) / XT > 65535) return Q8T_ERR_SHAPE;
    hipLaunchKernelGGL(xnor_gemm_kernel, dim3((N + XT - 1) / XT, (M + XT - 1) / XT), dim3(kThreads), 0, (hipStream_t)stream,
                       a_bits, w_bits, M, N, K, y);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

size_t q8t_tern_wgrad_multi_workspace_size(int M, int N, int K)
{
    (void)M; (void)N; (void)K;
    return sizeof(float) * kMaxPartials;
}

int q8t_tern_wgrad_multi(const float *g, const int8_t *a_codes, int M, int N, int K, int S, uint64_t seed, float *dw,
                         int64_t *acc_out, void *ws, void *stream)
{
    if (M <= 0 || N <= 0 || K <= 0 || S <= 0) return Q8T_ERR_SHAPE;
    if ((int64_t)M * N >= ((int64_t)1 << 31) || (int64_t)M * K >= ((int64_t)1 << 31) || (int64_t)K * N >= ((int64_t)1 << 31))
        return Q8T_ERR_SHAPE;
    if ((int64_t)S * M >= ((int64_t)1 << 31)) return Q8T_ERR_OVERFLOW;   // |accumulator| <= S * M must fit 32 bits
    if ((N + TW - 1) / TW > 65535 || (K + TW - 1) / TW > 65535) return Q8T_ERR_SHAPE;
    if (!g || !a_codes || (!dw && !acc_out)) return Q8T_ERR_NULL;
    if (!ws || !q8t_aligned(ws, 4)) return Q8T_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const int np = launch_absmax(g, (int64_t)M * N, (float *)ws, st);
    Q8T_LAUNCH_CHECK();
    hipLaunchKernelGGL(tern_wgrad_multi_kernel, dim3((N + TW - 1) / TW, (K + TW - 1) / TW), dim3(kThreads), 0, st, g, a_codes, M,
                       N, K, S, (uint32_t)seed, (uint32_t)(seed >> 32), (const float *)ws, np, dw, acc_out);
    Q8T_LAUNCH_CHECK();
    return Q8T_OK;
}

}  // extern "C"
