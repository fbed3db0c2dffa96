/*
 * q8t_oracle.c -- plain, slow CPU oracle for the 8-bit training hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the arbiter of parity for the HIP
 * library; it shares no code, header, table or helper with it and must never
 * be called from the product path.  Only tests, the smoke check and the
 * benchmark's cpu-baseline leg load it.
 *
 * Every function follows one passage of the paper
 * ("Scalable Methods for 8-bit Training of Neural Networks"):
 *   - affine min/max quantization ............ Appendix B (GEMMLOWP scheme)
 *   - stochastic rounding of gradients ....... Section 4, "Quantization methods"
 *   - forward / layer-gradient / weight-gradient products
 *                                              Section 4, eqs. (grad_layer), (grad_weight)
 *   - 16-bit copy of g_l for the weight gradient  Section 1 / Section 7 ("Gradients Bifurcation")
 *   - Range BN forward ....................... Section 3, eq. (range), C(n) = 1/sqrt(2 ln n)
 *   - Range BN backward ...................... Section 7 (derivative of max/min is one at the
 *                                              coordinates attaining them, zero elsewhere)
 *   - stochastic ternarization, binarization, XNOR + population count product,
 *     multiple stochastic ternarization sampling   appendix "Additional Experiments", Algorithm 1
 *
 * Floating point: rounding decisions (the integer codes) are taken in fp32 with
 * a fixed operation order -- one rounding per written operation, no fused
 * multiply-add (build with -ffp-contract=off) -- because the codes are integers
 * that must match bit for bit.  All long sums are accumulated in fp64.
 * Integer products are accumulated in int64.
 *
 * Parity status: every function here is pinned by tests/test_oracle_*.py
 * against closed forms, brute force or invariants.  End-to-end accuracy figures
 * of the paper need its datasets: parity unpinned for those, out of scope.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    float vmin, vmax, scale, inv_scale;
    int32_t zero_point;
    int32_t bits;
} orc_qparams;

typedef struct {
    int N, C, H, W, K, R, S, stride, pad;
} orc_conv_desc;

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* Appendix B: clamping values are the tensor's minimum and maximum.   */
void orc_minmax(const float *x, int64_t n, float *vmin, float *vmax)
{
    float mn = INFINITY, mx = -INFINITY;
    for (int64_t i = 0; i < n; ++i) {
        if (x[i] < mn) mn = x[i];
        if (x[i] > mx) mx = x[i];
    }
    *vmin = mn;
    *vmax = mx;
}

/*
 * Appendix B: scale and zero point from [vmin, vmax] and the bit width M.
 * Readings: the range is widened to contain 0 so that the zero point is a
 * valid level; the highest level is 2^M - 1 so that vmax lands on a level
 * that fits M bits; the zero point is an integer; a constant-zero range
 * gives scale 1.
 */
void orc_qparams_from_range(float vmin, float vmax, int bits, orc_qparams *qp)
{
    if (vmin > 0.0f) vmin = 0.0f;
    if (vmax < 0.0f) vmax = 0.0f;
    int32_t qmax = (1 << bits) - 1;
    float span = vmax - vmin;
    float scale = span / (float)qmax;
    if (scale == 0.0f) scale = 1.0f;
    float inv_scale = 1.0f / scale;
    float negmin = -vmin;
    float zf = negmin * inv_scale;
    float zr = rintf(zf); /* round half to even */
    if (zr < 0.0f) zr = 0.0f;
    if (zr > (float)qmax) zr = (float)qmax;
    qp->vmin = vmin;
    qp->vmax = vmax;
    qp->scale = scale;
    qp->inv_scale = inv_scale;
    qp->zero_point = (int32_t)zr;
    qp->bits = bits;
}

/* ------------------------------------------------------------------ */
/* Counter-based generator for stochastic rounding.  Stateless, keyed  */
/* by (seed, logical flat element index).  All arithmetic is uint32.   */
static uint32_t orc_mix32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x6A09E667u;
    x ^= x >> 15;
    x *= 0xBB67AE85u;
    x ^= x >> 16;
    return x;
}

/* the two 32-bit words that serve the group of four elements 4g .. 4g+3 */
void orc_rng_words(uint64_t g, uint64_t seed, uint32_t *w0, uint32_t *w1)
{
    const uint32_t golden = 0x9E3779B9u;
    uint32_t g32 = (uint32_t)g;
    uint32_t h = orc_mix32(g32 * golden + (uint32_t)seed) ^ (uint32_t)(seed >> 32);
    *w0 = orc_mix32(h + golden);
    *w1 = orc_mix32(h + 2u * golden);
}

/* 16 random bits for element i */
uint32_t orc_r16(uint64_t i, uint64_t seed)
{
    uint32_t w0, w1;
    orc_rng_words(i >> 2, seed, &w0, &w1);
    uint32_t w = (i & 2) ? w1 : w0;
    return (w >> (16 * (unsigned)(i & 1))) & 0xFFFFu;
}

/* ------------------------------------------------------------------ */
/*
 * Appendix B: output = round(x / scale + zero_point), clamped to the M-bit
 * levels.  Returns the level in [0, 2^M - 1].  Nearest rounding is
 * round-half-to-even; stochastic rounding (Section 4) rounds up with
 * probability equal to the fractional part, using 16 random bits.
 */
static int32_t orc_level(float x, const orc_qparams *qp, int stochastic, uint64_t i, uint64_t seed)
{
    float qmax = (float)((1 << qp->bits) - 1);
    float u = x * qp->inv_scale;
    float t = u + (float)qp->zero_point;
    float q;
    if (!stochastic) {
        q = rintf(t);
    } else {
        float f = floorf(t);
        float frac = t - f;
        uint32_t r = orc_r16(i, seed);
        float lhs = frac * 65536.0f;
        float rhs = (float)r + 0.5f;
        q = (lhs > rhs) ? f + 1.0f : f;
    }
    /* saturate while still in float: a value far outside a supplied range must land on the
       nearest end level, whatever an out-of-range float-to-int conversion would do */
    if (q < 0.0f) q = 0.0f;
    if (q > qmax) q = qmax;
    return (int32_t)q;
}

/*
 * Quantize with a given range.  Levels are written as int32 (levels_out,
 * nullable) and in stored form level - 2^(M-1) as int8 (M <= 8) or int16
 * (stored_out, nullable).
 */
void orc_quantize_with_range(const float *x, int64_t n, int bits, int stochastic, uint64_t seed,
                             float vmin, float vmax, int32_t *levels_out, void *stored_out,
                             orc_qparams *qp_out)
{
    orc_qparams qp;
    orc_qparams_from_range(vmin, vmax, bits, &qp);
    int32_t half = 1 << (bits - 1);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        int32_t q = orc_level(x[i], &qp, stochastic, (uint64_t)i, seed);
        if (levels_out) levels_out[i] = q;
        if (stored_out) {
            if (bits <= 8)
                ((int8_t *)stored_out)[i] = (int8_t)(q - half);
            else
                ((int16_t *)stored_out)[i] = (int16_t)(q - half);
        }
    }
    if (qp_out) *qp_out = qp;
}

/* Quantize with the tensor's own minimum and maximum (Appendix B). */
void orc_quantize(const float *x, int64_t n, int bits, int stochastic, uint64_t seed,
                  int32_t *levels_out, void *stored_out, orc_qparams *qp_out)
{
    float mn, mx;
    if (n > 0) {
        orc_minmax(x, n, &mn, &mx);
    } else {
        mn = 0.0f;
        mx = 0.0f;
    }
    orc_quantize_with_range(x, n, bits, stochastic, seed, mn, mx, levels_out, stored_out, qp_out);
}

/* real value of a stored code: scale * (level - zero_point) */
void orc_dequantize(const void *stored, const orc_qparams *qp, int64_t n, float *out)
{
    int32_t half = 1 << (qp->bits - 1);
    for (int64_t i = 0; i < n; ++i) {
        int32_t s = (qp->bits <= 8) ? (int32_t)((const int8_t *)stored)[i]
                                    : (int32_t)((const int16_t *)stored)[i];
        int32_t q = s + half;
        out[i] = qp->scale * (float)(q - qp->zero_point);
    }
}

/* Sec. 5.1 (Problem Statement), eq. (1): cosine of the angle between a tensor and its quantized copy,
 * cos(theta) = (x . Q(x)) / (||x||_2 ||Q(x)||_2), with Q(x) the dequantized value of the stored
 * code (fp32, as orc_dequantize returns it).  All three sums in fp64, index order.
 * out[0] = x.Q(x), out[1] = ||x||^2, out[2] = ||Q(x)||^2, out[3] = cos(theta) (0 if a norm is 0). */
void orc_quant_angle(const float *x, const void *stored, const orc_qparams *qp, int64_t n, double *out)
{
    int32_t half = 1 << (qp->bits - 1);
    double dot = 0.0, nx = 0.0, nq = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        int32_t s = (qp->bits <= 8) ? (int32_t)((const int8_t *)stored)[i]
                                    : (int32_t)((const int16_t *)stored)[i];
        float xq = qp->scale * (float)(s + half - qp->zero_point);
        dot += (double)x[i] * (double)xq;
        nx += (double)x[i] * (double)x[i];
        nq += (double)xq * (double)xq;
    }
    out[0] = dot;
    out[1] = nx;
    out[2] = nq;
    out[3] = (nx > 0.0 && nq > 0.0) ? dot / sqrt(nx * nq) : 0.0;
}

/* App. B, clamping values of the activations: "the average of absolute maximum and minimum
 * values of K chunks".  The flat tensor is cut into K contiguous chunks of ceil(n/K) elements
 * (the last one may be shorter; when K does not divide n, chunks that would start past the end do
 * not exist and are not counted); vmax = mean over chunks of the chunk maximum, vmin = mean of the
 * chunk minimum.  The K values are summed in fp64 in chunk order and the mean is rounded
 * to fp32 once.  range_out[0] = vmin, range_out[1] = vmax. */
void orc_chunk_range(const float *x, int64_t n, int K, float *range_out)
{
    int64_t len = (n + K - 1) / K;
    double smin = 0.0, smax = 0.0;
    int used = 0;
    for (int k = 0; k < K; ++k) {
        int64_t lo = (int64_t)k * len, hi = lo + len < n ? lo + len : n;
        if (lo >= hi) break;
        float mn = x[lo], mx = x[lo];
        for (int64_t i = lo + 1; i < hi; ++i) {
            if (x[i] < mn) mn = x[i];
            if (x[i] > mx) mx = x[i];
        }
        smin += (double)mn;
        smax += (double)mx;
        ++used;
    }
    range_out[0] = (float)(smin / (double)used);
    range_out[1] = (float)(smax / (double)used);
}

/* stored code (int8 or int16) -> level minus zero point */
static inline int32_t orc_centered8(const int8_t *s, int64_t i, const orc_qparams *qp)
{
    return (int32_t)s[i] + (1 << (qp->bits - 1)) - qp->zero_point;
}
static inline int32_t orc_centered16(const int16_t *s, int64_t i, const orc_qparams *qp)
{
    return (int32_t)s[i] + (1 << (qp->bits - 1)) - qp->zero_point;
}

/* ------------------------------------------------------------------ */
/* Fully connected layer, row-major.                                   */
/* Forward: Y[M,N] = X[M,K] W[K,N] on the quantized operands, integer  */
/* accumulation, one float scale at the end (Section 7: forward pass   */
/* runs as 8-bit products).                                            */
void orc_qgemm_fwd(const int8_t *qx, const orc_qparams *px, const int8_t *qw, const orc_qparams *pw,
                   int M, int N, int K, float *y, int64_t *acc_out)
{
    float sc = px->scale * pw->scale;
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            int64_t acc = 0;
            for (int k = 0; k < K; ++k)
                acc += (int64_t)orc_centered8(qx, (int64_t)m * K + k, px) *
                       (int64_t)orc_centered8(qw, (int64_t)k * N + n, pw);
            if (acc_out) acc_out[(int64_t)m * N + n] = acc;
            if (y) y[(int64_t)m * N + n] = sc * (float)acc;
        }
}

/* Layer gradient, eq. (grad_layer): dX[M,K] = dY[M,N] W[K,N]^T. */
void orc_qgemm_dgrad(const int8_t *qdy, const orc_qparams *pg, const int8_t *qw, const orc_qparams *pw,
                     int M, int N, int K, float *dx, int64_t *acc_out)
{
    float sc = pg->scale * pw->scale;
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m)
        for (int k = 0; k < K; ++k) {
            int64_t acc = 0;
            for (int n = 0; n < N; ++n)
                acc += (int64_t)orc_centered8(qdy, (int64_t)m * N + n, pg) *
                       (int64_t)orc_centered8(qw, (int64_t)k * N + n, pw);
            if (acc_out) acc_out[(int64_t)m * K + k] = acc;
            if (dx) dx[(int64_t)m * K + k] = sc * (float)acc;
        }
}

/* Weight gradient, eq. (grad_weight): dW[K,N] = X[M,K]^T dY16[M,N], the  */
/* gradient operand kept at 16 bits, the layer input at 8 bits.           */
void orc_qgemm_wgrad(const int8_t *qx, const orc_qparams *px, const int16_t *qdy16,
                     const orc_qparams *pg, int M, int N, int K, float *dw, int64_t *acc_out)
{
    float sc = pg->scale * px->scale;
#pragma omp parallel for schedule(static)
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n) {
            int64_t acc = 0;
            for (int m = 0; m < M; ++m)
                acc += (int64_t)orc_centered8(qx, (int64_t)m * K + k, px) *
                       (int64_t)orc_centered16(qdy16, (int64_t)m * N + n, pg);
            if (acc_out) acc_out[(int64_t)k * N + n] = acc;
            if (dw) dw[(int64_t)k * N + n] = (float)((double)acc * (double)sc);
        }
}

/* ------------------------------------------------------------------ */
/* Convolution layer, NCHW activations, filter [K,C,R,S], zero padding */
/* (a padded tap contributes exactly nothing), no bias.                */
static inline int orc_out_dim(int in, int f, int stride, int pad)
{
    return (in + 2 * pad - f) / stride + 1;
}

void orc_qconv_fwd(const orc_conv_desc *d, const int8_t *qx, const orc_qparams *px, const int8_t *qw,
                   const orc_qparams *pw, float *y, int64_t *acc_out)
{
    const int P = orc_out_dim(d->H, d->R, d->stride, d->pad);
    const int Q = orc_out_dim(d->W, d->S, d->stride, d->pad);
    float sc = px->scale * pw->scale;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < d->N; ++n)
        for (int k = 0; k < d->K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    int64_t acc = 0;
                    for (int c = 0; c < d->C; ++c)
                        for (int r = 0; r < d->R; ++r) {
                            int h = p * d->stride + r - d->pad;
                            if (h < 0 || h >= d->H) continue;
                            for (int s = 0; s < d->S; ++s) {
                                int w = q * d->stride + s - d->pad;
                                if (w < 0 || w >= d->W) continue;
                                int64_t xi = (((int64_t)n * d->C + c) * d->H + h) * d->W + w;
                                int64_t wi = (((int64_t)k * d->C + c) * d->R + r) * d->S + s;
                                acc += (int64_t)orc_centered8(qx, xi, px) *
                                       (int64_t)orc_centered8(qw, wi, pw);
                            }
                        }
                    int64_t oi = (((int64_t)n * d->K + k) * P + p) * Q + q;
                    if (acc_out) acc_out[oi] = acc;
                    if (y) y[oi] = sc * (float)acc;
                }
}

/* dX[n,c,h,w] = sum over (k,r,s) and the output positions (p,q) that tap (h,w) */
void orc_qconv_dgrad(const orc_conv_desc *d, const int8_t *qdy, const orc_qparams *pg,
                     const int8_t *qw, const orc_qparams *pw, float *dx, int64_t *acc_out)
{
    const int P = orc_out_dim(d->H, d->R, d->stride, d->pad);
    const int Q = orc_out_dim(d->W, d->S, d->stride, d->pad);
    float sc = pg->scale * pw->scale;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < d->N; ++n)
        for (int c = 0; c < d->C; ++c)
            for (int h = 0; h < d->H; ++h)
                for (int w = 0; w < d->W; ++w) {
                    int64_t acc = 0;
                    for (int k = 0; k < d->K; ++k)
                        for (int r = 0; r < d->R; ++r) {
                            int hp = h + d->pad - r;
                            if (hp < 0 || hp % d->stride) continue;
                            int p = hp / d->stride;
                            if (p >= P) continue;
                            for (int s = 0; s < d->S; ++s) {
                                int wq = w + d->pad - s;
                                if (wq < 0 || wq % d->stride) continue;
                                int q = wq / d->stride;
                                if (q >= Q) continue;
                                int64_t gi = (((int64_t)n * d->K + k) * P + p) * Q + q;
                                int64_t wi = (((int64_t)k * d->C + c) * d->R + r) * d->S + s;
                                acc += (int64_t)orc_centered8(qdy, gi, pg) *
                                       (int64_t)orc_centered8(qw, wi, pw);
                            }
                        }
                    int64_t oi = (((int64_t)n * d->C + c) * d->H + h) * d->W + w;
                    if (acc_out) acc_out[oi] = acc;
                    if (dx) dx[oi] = sc * (float)acc;
                }
}

/* dW[k,c,r,s] = sum over (n,p,q) of g16[n,k,p,q] * x8[n,c,p*st+r-pad,q*st+s-pad] */
void orc_qconv_wgrad(const orc_conv_desc *d, const int8_t *qx, const orc_qparams *px,
                     const int16_t *qdy16, const orc_qparams *pg, float *dw, int64_t *acc_out)
{
    const int P = orc_out_dim(d->H, d->R, d->stride, d->pad);
    const int Q = orc_out_dim(d->W, d->S, d->stride, d->pad);
    float sc = pg->scale * px->scale;
#pragma omp parallel for collapse(2) schedule(static)
    for (int k = 0; k < d->K; ++k)
        for (int c = 0; c < d->C; ++c)
            for (int r = 0; r < d->R; ++r)
                for (int s = 0; s < d->S; ++s) {
                    int64_t acc = 0;
                    for (int n = 0; n < d->N; ++n)
                        for (int p = 0; p < P; ++p) {
                            int h = p * d->stride + r - d->pad;
                            if (h < 0 || h >= d->H) continue;
                            for (int q = 0; q < Q; ++q) {
                                int w = q * d->stride + s - d->pad;
                                if (w < 0 || w >= d->W) continue;
                                int64_t gi = (((int64_t)n * d->K + k) * P + p) * Q + q;
                                int64_t xi = (((int64_t)n * d->C + c) * d->H + h) * d->W + w;
                                acc += (int64_t)orc_centered16(qdy16, gi, pg) *
                                       (int64_t)orc_centered8(qx, xi, px);
                            }
                        }
                    int64_t oi = (((int64_t)k * d->C + c) * d->R + r) * d->S + s;
                    if (acc_out) acc_out[oi] = acc;
                    if (dw) dw[oi] = (float)((double)acc * (double)sc);
                }
}

/* ------------------------------------------------------------------ */
/* Range BN, Section 3.                                                */

/* C(n) = 1 / sqrt(2 ln n) */
double orc_range_bn_scale(int64_t n)
{
    return 1.0 / sqrt(2.0 * log((double)n));
}

/*
 * Per-channel statistics over the n = N*H*W values of channel c:
 * mean (fp64 sum, one rounding), minimum, maximum.
 * range(x - mu) = max(x) - min(x), so the raw extrema are what is kept.
 */
void orc_range_bn_stats(const float *x, int N, int C, int H, int W, float *stats /* [3][C] */)
{
    const int64_t HW = (int64_t)H * W;
    const int64_t n = (int64_t)N * HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        double sum = 0.0;
        float mn = INFINITY, mx = -INFINITY;
        for (int b = 0; b < N; ++b) {
            const float *p = x + ((int64_t)b * C + c) * HW;
            for (int64_t i = 0; i < HW; ++i) {
                float v = p[i];
                sum += (double)v;
                if (v < mn) mn = v;
                if (v > mx) mx = v;
            }
        }
        stats[c] = (float)(sum / (double)n);
        stats[C + c] = mn;
        stats[2 * C + c] = mx;
    }
}

/* 1 / (C(n) * (max - min) + eps), fp32, one rounding per operation */
static float orc_bn_inv(float mn, float mx, float cn, float eps)
{
    float range = mx - mn;
    float scaled = cn * range;
    float denom = scaled + eps;
    return 1.0f / denom;
}

/* the elementwise map of eq. (range) with optional affine, fp32, no fused ops */
static float orc_bn_apply(float x, float mu, float inv, float g, float b)
{
    float cen = x - mu;
    float xh = cen * inv;
    float sc = xh * g;
    return sc + b;
}

/*
 * Elementwise stage of the forward pass for GIVEN statistics.
 *  y        (nullable) fp32 output
 *  q_stored (nullable) 8-bit per-tensor quantized output; its range is taken
 *           from the images of each channel's extrema under the same map
 *           (Section 4: the normalizer already knows min and max, so no extra
 *           pass over the data is needed).
 */
void orc_range_bn_fwd_apply(const float *x, int N, int C, int H, int W, const float *gamma,
                            const float *beta, float eps, const float *stats, float *y,
                            int8_t *q_stored, orc_qparams *qp_out)
{
    const int64_t HW = (int64_t)H * W;
    const int64_t n = (int64_t)N * HW;
    const float cn = (float)orc_range_bn_scale(n);
    orc_qparams qp;
    memset(&qp, 0, sizeof qp);
    if (q_stored || qp_out) {
        float vmin = INFINITY, vmax = -INFINITY;
        for (int c = 0; c < C; ++c) {
            float g = gamma ? gamma[c] : 1.0f, b = beta ? beta[c] : 0.0f;
            float inv = orc_bn_inv(stats[C + c], stats[2 * C + c], cn, eps);
            float a = orc_bn_apply(stats[C + c], stats[c], inv, g, b);
            float z = orc_bn_apply(stats[2 * C + c], stats[c], inv, g, b);
            float lo = a < z ? a : z, hi = a < z ? z : a;
            if (lo < vmin) vmin = lo;
            if (hi > vmax) vmax = hi;
        }
        orc_qparams_from_range(vmin, vmax, 8, &qp);
        if (qp_out) *qp_out = qp;
    }
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < N; ++b)
        for (int c = 0; c < C; ++c) {
            float g = gamma ? gamma[c] : 1.0f, be = beta ? beta[c] : 0.0f;
            float mu = stats[c];
            float inv = orc_bn_inv(stats[C + c], stats[2 * C + c], cn, eps);
            int64_t base = ((int64_t)b * C + c) * HW;
            for (int64_t i = 0; i < HW; ++i) {
                float v = orc_bn_apply(x[base + i], mu, inv, g, be);
                if (y) y[base + i] = v;
                if (q_stored)
                    q_stored[base + i] = (int8_t)(orc_level(v, &qp, 0, 0, 0) - 128);
            }
        }
}

/* statistics + elementwise stage */
void orc_range_bn_fwd(const float *x, int N, int C, int H, int W, const float *gamma,
                      const float *beta, float eps, float *y, float *stats_out, int8_t *q_stored,
                      orc_qparams *qp_out)
{
    orc_range_bn_stats(x, N, C, H, W, stats_out);
    orc_range_bn_fwd_apply(x, N, C, H, W, gamma, beta, eps, stats_out, y, q_stored, qp_out);
}

/*
 * Per-channel sums of the backward pass for GIVEN forward statistics:
 *   sums[0][c] = sum dy          (= dbeta)
 *   sums[1][c] = sum dy * xhat   (= dgamma), xhat from the forward fp32 map
 * fp64 accumulation.
 */
void orc_range_bn_bwd_sums(const float *x, const float *dy, const float *stats, int N, int C, int H,
                           int W, float eps, double *sums /* [2][C] */)
{
    const int64_t HW = (int64_t)H * W;
    const int64_t n = (int64_t)N * HW;
    const float cn = (float)orc_range_bn_scale(n);
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        float mu = stats[c];
        float inv = orc_bn_inv(stats[C + c], stats[2 * C + c], cn, eps);
        double s0 = 0.0, s1 = 0.0;
        for (int b = 0; b < N; ++b) {
            int64_t base = ((int64_t)b * C + c) * HW;
            for (int64_t i = 0; i < HW; ++i) {
                float cen = x[base + i] - mu;
                float xh = cen * inv;
                s0 += (double)dy[base + i];
                s1 += (double)dy[base + i] * (double)xh;
            }
        }
        sums[c] = s0;
        sums[C + c] = s1;
    }
}

/*
 * Elementwise stage of the backward pass for GIVEN statistics and sums.
 * With g_j = gamma*dy_j, A = gamma*sum dy, B = gamma*sum dy*xhat,
 * s = C(n)(max-min)+eps, inv = 1/s:
 *   dx_j = inv*(g_j - A/n) - inv*C(n)*B*([x_j == max] - [x_j == min])
 * (chain rule through eq. (range); the max/min derivative follows Section 7,
 * every coordinate that attains the extremum receives the term).
 */
void orc_range_bn_bwd_apply(const float *x, const float *dy, const float *stats, const double *sums,
                            int N, int C, int H, int W, const float *gamma, float eps, float *dx,
                            float *dgamma, float *dbeta)
{
    const int64_t HW = (int64_t)H * W;
    const int64_t n = (int64_t)N * HW;
    const double cn_d = orc_range_bn_scale(n);
    const float cn = (float)cn_d;
    for (int c = 0; c < C; ++c) {
        if (dbeta) dbeta[c] = (float)sums[c];
        if (dgamma) dgamma[c] = (float)sums[C + c];
    }
    if (!dx) return;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < N; ++b)
        for (int c = 0; c < C; ++c) {
            float g = gamma ? gamma[c] : 1.0f;
            float mn = stats[C + c], mx = stats[2 * C + c];
            float inv = orc_bn_inv(mn, mx, cn, eps);
            double A = (double)g * sums[c];
            double B = (double)g * sums[C + c];
            float mean_g = (float)(A / (double)n);
            float kb = (float)((double)inv * (double)cn * B);
            int64_t base = ((int64_t)b * C + c) * HW;
            for (int64_t i = 0; i < HW; ++i) {
                float gh = g * dy[base + i];
                float t = gh - mean_g;
                float v = inv * t;
                float xv = x[base + i];
                if (xv == mx) v = v - kb;
                if (xv == mn) v = v + kb;
                dx[base + i] = v;
            }
        }
}

void orc_range_bn_bwd(const float *x, const float *dy, const float *stats, int N, int C, int H, int W,
                      const float *gamma, float eps, float *dx, float *dgamma, float *dbeta)
{
    double *sums = (double *)malloc(sizeof(double) * 2 * (size_t)C);
    orc_range_bn_bwd_sums(x, dy, stats, N, C, H, W, eps, sums);
    orc_range_bn_bwd_apply(x, dy, stats, sums, N, C, H, W, gamma, eps, dx, dgamma, dbeta);
    free(sums);
}

/*
 * Range BN followed by ReLU, for GIVEN statistics (a widening of Section 4's remark that the
 * normalizer already knows the extrema: the rectified output's range is known too).
 *   v = max(BN(x), 0), taken as (BN(x) > 0 ? BN(x) : +0)
 *  y        (nullable) fp32 output
 *  q_stored (nullable) 8-bit per-tensor codes of v; range = the images of every channel's extrema
 *           under the same map, rectified: [max(lo, 0), max(hi, 0)].
 */
void orc_range_bn_relu_fwd_apply(const float *x, int N, int C, int H, int W, const float *gamma,
                                 const float *beta, float eps, const float *stats, float *y,
                                 int8_t *q_stored, orc_qparams *qp_out)
{
    const int64_t HW = (int64_t)H * W;
    const int64_t n = (int64_t)N * HW;
    const float cn = (float)orc_range_bn_scale(n);
    orc_qparams qp;
    memset(&qp, 0, sizeof qp);
    if (q_stored || qp_out) {
        float vmin = INFINITY, vmax = -INFINITY;
        for (int c = 0; c < C; ++c) {
            float g = gamma ? gamma[c] : 1.0f, b = beta ? beta[c] : 0.0f;
            float inv = orc_bn_inv(stats[C + c], stats[2 * C + c], cn, eps);
            float a = orc_bn_apply(stats[C + c], stats[c], inv, g, b);
            float z = orc_bn_apply(stats[2 * C + c], stats[c], inv, g, b);
            float lo = a < z ? a : z, hi = a < z ? z : a;
            if (lo < vmin) vmin = lo;
            if (hi > vmax) vmax = hi;
        }
        vmin = vmin > 0.0f ? vmin : 0.0f;
        vmax = vmax > 0.0f ? vmax : 0.0f;
        orc_qparams_from_range(vmin, vmax, 8, &qp);
        if (qp_out) *qp_out = qp;
    }
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < N; ++b)
        for (int c = 0; c < C; ++c) {
            float g = gamma ? gamma[c] : 1.0f, be = beta ? beta[c] : 0.0f;
            float mu = stats[c];
            float inv = orc_bn_inv(stats[C + c], stats[2 * C + c], cn, eps);
            int64_t base = ((int64_t)b * C + c) * HW;
            for (int64_t i = 0; i < HW; ++i) {
                float v = orc_bn_apply(x[base + i], mu, inv, g, be);
                v = v > 0.0f ? v : 0.0f;
                if (y) y[base + i] = v;
                if (q_stored)
                    q_stored[base + i] = (int8_t)(orc_level(v, &qp, 0, 0, 0) - 128);
            }
        }
}

/*
 * Backward of the ReLU that follows a Range BN: the upstream gradient passes where the
 * (recomputed, fp32) BN output is positive and is zero elsewhere (derivative 0 at 0).
 * The Range BN backward then runs on the masked gradient.
 */
void orc_range_bn_relu_mask(const float *x, const float *dy, const float *stats, int N, int C, int H,
                            int W, const float *gamma, const float *beta, float eps, float *dy_masked)
{
    const int64_t HW = (int64_t)H * W;
    const int64_t n = (int64_t)N * HW;
    const float cn = (float)orc_range_bn_scale(n);
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < N; ++b)
        for (int c = 0; c < C; ++c) {
            float g = gamma ? gamma[c] : 1.0f, be = beta ? beta[c] : 0.0f;
            float inv = orc_bn_inv(stats[C + c], stats[2 * C + c], cn, eps);
            int64_t base = ((int64_t)b * C + c) * HW;
            for (int64_t i = 0; i < HW; ++i) {
                float v = orc_bn_apply(x[base + i], stats[c], inv, g, be);
                dy_masked[base + i] = v > 0.0f ? dy[base + i] : 0.0f;
            }
        }
}

/* ------------------------------------------------------------------ */
/* fp64 definitions, used only to pin the fp32 sequences above.        */

/* eq. (range) written out in double; x is [N,C,H,W] in double */
void orc_range_bn_fwd_f64(const double *x, int N, int C, int H, int W, const double *gamma,
                          const double *beta, double eps, double *y)
{
    const int64_t HW = (int64_t)H * W;
    const int64_t n = (int64_t)N * HW;
    const double cn = orc_range_bn_scale(n);
    for (int c = 0; c < C; ++c) {
        double sum = 0.0, mn = INFINITY, mx = -INFINITY;
        for (int b = 0; b < N; ++b)
            for (int64_t i = 0; i < HW; ++i) {
                double v = x[((int64_t)b * C + c) * HW + i];
                sum += v;
                if (v < mn) mn = v;
                if (v > mx) mx = v;
            }
        double mu = sum / (double)n;
        /* range of the centred values, as the equation states it */
        double range = (mx - mu) - (mn - mu);
        double s = cn * range + eps;
        double g = gamma ? gamma[c] : 1.0, be = beta ? beta[c] : 0.0;
        for (int b = 0; b < N; ++b)
            for (int64_t i = 0; i < HW; ++i) {
                int64_t j = ((int64_t)b * C + c) * HW + i;
                y[j] = g * ((x[j] - mu) / s) + be;
            }
    }
}

/* traditional batch norm, eq. (L2_BN_equation): (x - mu) / sqrt(Var) */
void orc_standard_bn_f64(const double *x, int N, int C, int H, int W, double *y)
{
    const int64_t HW = (int64_t)H * W;
    const int64_t n = (int64_t)N * HW;
    for (int c = 0; c < C; ++c) {
        double sum = 0.0;
        for (int b = 0; b < N; ++b)
            for (int64_t i = 0; i < HW; ++i) sum += x[((int64_t)b * C + c) * HW + i];
        double mu = sum / (double)n, ss = 0.0;
        for (int b = 0; b < N; ++b)
            for (int64_t i = 0; i < HW; ++i) {
                double dlt = x[((int64_t)b * C + c) * HW + i] - mu;
                ss += dlt * dlt;
            }
        double sd = sqrt(ss / (double)n);
        for (int b = 0; b < N; ++b)
            for (int64_t i = 0; i < HW; ++i) {
                int64_t j = ((int64_t)b * C + c) * HW + i;
                y[j] = (x[j] - mu) / sd;
            }
    }
}

/* ------------------------------------------------------------------ */
/* Ternarized back-propagation (appendix "Additional Experiments").     */
/* The paper names the operations (stochastic ternarization of the      */
/* gradient, binarized weights and activations, XNOR + population       */
/* count products, Algorithm 1) without defining them; the readings     */
/* are: StcTern(g)_i = sign(g_i) with probability |g_i| / max|g| and 0   */
/* otherwise (unbiased once multiplied by max|g|), the draw taken from  */
/* the same counter-based generator as the stochastic rounding; a       */
/* binarized value is +1 for x >= 0 and -1 otherwise.                   */

/* codes in {-1, 0, +1}; *scale = max |x| (0 for an all-zero tensor: every code is 0) */
void orc_ternarize(const float *x, int64_t n, uint64_t seed, int8_t *codes, float *scale)
{
    float s = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
        const float a = fabsf(x[i]);
        if (a > s) s = a;
    }
    *scale = s;
    if (s == 0.0f) {
        for (int64_t i = 0; i < n; ++i) codes[i] = 0;
        return;
    }
    const float inv = 1.0f / s;
    for (int64_t i = 0; i < n; ++i) {
        const float p = fabsf(x[i]) * inv;                 /* probability of a non-zero code */
        const float lhs = p * 65536.0f;
        const float rhs = (float)orc_r16((uint64_t)i, seed) + 0.5f;
        const int keep = lhs > rhs;
        codes[i] = (int8_t)(keep ? (x[i] < 0.0f ? -1 : 1) : 0);
    }
}

/* binarized value: +1 for x >= 0, -1 otherwise */
void orc_binarize(const float *x, int64_t n, int8_t *codes)
{
    for (int64_t i = 0; i < n; ++i) codes[i] = (int8_t)(x[i] >= 0.0f ? 1 : -1);
}

/* Bits of a [rows][cols] matrix of +-1 codes, bit = 1 for +1.  transpose = 0: one bit row per
 * matrix row, out[rows][ceil(cols/32)], bit j of word w = column 32w + j.  transpose = 1: one bit
 * row per matrix column, out[cols][ceil(rows/32)], bit j of word w = row 32w + j.  Bits past the
 * end of a bit row are 0. */
void orc_pack_bits(const int8_t *codes, int rows, int cols, int transpose, uint32_t *out)
{
    const int nr = transpose ? cols : rows, nc = transpose ? rows : cols;
    const int words = (nc + 31) / 32;
    for (int r = 0; r < nr; ++r)
        for (int w = 0; w < words; ++w) {
            uint32_t v = 0;
            for (int j = 0; j < 32; ++j) {
                const int c = 32 * w + j;
                if (c >= nc) break;
                const int8_t code = transpose ? codes[(int64_t)c * cols + r] : codes[(int64_t)r * cols + c];
                if (code > 0) v |= (uint32_t)1 << j;
            }
            out[(int64_t)r * words + w] = v;
        }
}

/* y[m][n] = sum_k a[m][k] * w[n][k] over +-1 values given as bit rows of K bits (what an XNOR +
 * population count computes: matches minus mismatches), written out from the definition */
void orc_xnor_gemm(const uint32_t *abits, const uint32_t *wbits, int M, int N, int K, int32_t *y)
{
    const int words = (K + 31) / 32;
#pragma omp parallel for
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            int32_t acc = 0;
            for (int k = 0; k < K; ++k) {
                const int a = (abits[(int64_t)m * words + k / 32] >> (k % 32)) & 1 ? 1 : -1;
                const int w = (wbits[(int64_t)n * words + k / 32] >> (k % 32)) & 1 ? 1 : -1;
                acc += a * w;
            }
            y[(int64_t)m * N + n] = acc;
        }
}

/* Algorithm 1 (multiple stochastic ternarization sampling) for a fully connected layer:
 * g [M][N] gradient, a [M][K] binarized layer input (+-1 codes), S samples;
 *   for s = 1..S: t = StcTern(g) (seed + s - 1);  acc[k][n] += sum_m a[m][k] * t[m][n]
 *   dW[k][n] = max|g| * acc[k][n] / S
 * acc (nullable) receives the integer sum over all samples. */
void orc_tern_wgrad_multi(const float *g, const int8_t *a, int M, int N, int K, int S, uint64_t seed,
                          float *dw, int64_t *acc_out)
{
    const int64_t n = (int64_t)M * N;
    int8_t *t = (int8_t *)malloc((size_t)(n > 0 ? n : 1));
    int64_t *acc = (int64_t *)calloc((size_t)K * N, sizeof(int64_t));
    float scale = 0.0f;
    for (int s = 0; s < S; ++s) {
        orc_ternarize(g, n, seed + (uint64_t)s, t, &scale);
#pragma omp parallel for
        for (int k = 0; k < K; ++k)
            for (int c = 0; c < N; ++c) {
                int64_t v = 0;
                for (int m = 0; m < M; ++m) v += (int64_t)a[(int64_t)m * K + k] * (int64_t)t[(int64_t)m * N + c];
                acc[(int64_t)k * N + c] += v;
            }
    }
    for (int64_t i = 0; i < (int64_t)K * N; ++i) {
        if (acc_out) acc_out[i] = acc[i];
        if (dw) dw[i] = (float)((double)acc[i] * (double)scale / (double)S);
    }
    free(acc);
    free(t);
}

/* ------------------------------------------------------------------ */
/* Network plumbing around the method (not from the paper): the stem of */
/* a ResNet follows its first Range BN + ReLU with a 3x3 / stride 2 /   */
/* pad 1 max pooling.  Pooling and the residual additions are plain      */
/* definitions; they are here so that the fused GPU forms have a         */
/* reference.                                                            */

/* out[n][c][p][q] = max over the window rows 2p-1..2p+1, cols 2q-1..2q+1 (inside the plane) of
 * v = relu(Range BN(x)) for given statistics; idx = position of the FIRST maximum inside the
 * window in row-major order (3*i + j), or 255 when the maximum is not positive (nothing passes
 * a gradient back through the rectifier then).  P = (H - 1)/2 + 1, Q = (W - 1)/2 + 1. */
void orc_range_bn_relu_maxpool_fwd(const float *x, int N, int C, int H, int W, const float *gamma,
                                   const float *beta, float eps, const float *stats, float *out,
                                   uint8_t *idx)
{
    const int64_t HW = (int64_t)H * W;
    const int P = (H - 1) / 2 + 1, Q = (W - 1) / 2 + 1;
    float *v = (float *)malloc(sizeof(float) * (size_t)N * C * HW);
    orc_range_bn_relu_fwd_apply(x, N, C, H, W, gamma, beta, eps, stats, v, NULL, NULL);
#pragma omp parallel for
    for (int64_t pl = 0; pl < (int64_t)N * C; ++pl)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q) {
                float best = -INFINITY;
                int where = 255;
                for (int i = 0; i < 3; ++i)
                    for (int j = 0; j < 3; ++j) {
                        const int h = 2 * p - 1 + i, w = 2 * q - 1 + j;
                        if (h < 0 || h >= H || w < 0 || w >= W) continue;
                        const float t = v[pl * HW + (int64_t)h * W + w];
                        if (t > best) {
                            best = t;
                            where = 3 * i + j;
                        }
                    }
                out[(pl * P + p) * Q + q] = best;
                idx[(pl * P + p) * Q + q] = (uint8_t)(best > 0.0f ? where : 255);
            }
    free(v);
}

/* gradient with respect to the Range BN output of the stem: every window hands its gradient to the
 * position idx names (none for 255); contributions of the (up to four) windows that share a position
 * are added in window order */
void orc_maxpool_relu_bwd(const float *gpool, const uint8_t *idx, int N, int C, int H, int W, float *dy)
{
    const int64_t HW = (int64_t)H * W;
    const int P = (H - 1) / 2 + 1, Q = (W - 1) / 2 + 1;
    memset(dy, 0, sizeof(float) * (size_t)N * C * HW);
#pragma omp parallel for
    for (int64_t pl = 0; pl < (int64_t)N * C; ++pl)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q) {
                const int k = idx[(pl * P + p) * Q + q];
                if (k == 255) continue;
                const int h = 2 * p - 1 + k / 3, w = 2 * q - 1 + k % 3;
                dy[pl * HW + (int64_t)h * W + w] += gpool[(pl * P + p) * Q + q];
            }
}

/* out = relu(a + b), elementwise; *vmax (nullable) = max of out (its min is 0 or positive: the
 * range of the rectified sum, widened to contain 0, is [0, vmax]) */
void orc_add_relu(const float *a, const float *b, int64_t n, float *out, float *vmax)
{
    float mx = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
        const float s = a[i] + b[i];
        const float r = s > 0.0f ? s : 0.0f;
        out[i] = r;
        if (r > mx) mx = r;
    }
    if (vmax) *vmax = mx;
}

/* tail of a residual block in one pass: out = relu(bn(x) + o), bn = the elementwise stage of Range BN from given
 * statistics (orc_range_bn_fwd_apply's arithmetic), o = other, or bn'(other) from its own statistics when
 * other_stats is given (a shortcut that is itself convolution + Range BN); *vmax (nullable) = max of out */
void orc_range_bn_add_relu(const float *x, const float *stats, const float *gamma, const float *beta,
                           const float *other, const float *other_stats, const float *other_gamma,
                           const float *other_beta, int N, int C, int H, int W, float eps, float *out, float *vmax)
{
    const int64_t HW = (int64_t)H * W;
    const float cn = (float)orc_range_bn_scale((int64_t)N * HW);
    float mx = 0.0f;
    for (int b = 0; b < N; ++b)
        for (int c = 0; c < C; ++c) {
            const float g = gamma ? gamma[c] : 1.0f, be = beta ? beta[c] : 0.0f;
            const float inv = orc_bn_inv(stats[C + c], stats[2 * C + c], cn, eps);
            float og = 1.0f, obe = 0.0f, oinv = 0.0f, omu = 0.0f;
            if (other_stats) {
                og = other_gamma ? other_gamma[c] : 1.0f;
                obe = other_beta ? other_beta[c] : 0.0f;
                oinv = orc_bn_inv(other_stats[C + c], other_stats[2 * C + c], cn, eps);
                omu = other_stats[c];
            }
            const int64_t base = ((int64_t)b * C + c) * HW;
            for (int64_t i = 0; i < HW; ++i) {
                const float v = orc_bn_apply(x[base + i], stats[c], inv, g, be);
                const float o = other_stats ? orc_bn_apply(other[base + i], omu, oinv, og, obe) : other[base + i];
                const float s = v + o;
                const float r = s > 0.0f ? s : 0.0f;
                out[base + i] = r;
                if (r > mx) mx = r;
            }
        }
    if (vmax) *vmax = mx;
}

/* gradient reaching a rectified tensor `out` from two consumers: (g1 + g2) where out > 0, else 0; out NULL: no
 * rectifier in between (plain sum); g2 NULL: nothing added */
void orc_relu_bwd_sum(const float *g1, const float *g2, const float *out, int64_t n, float *res)
{
    for (int64_t i = 0; i < n; ++i) {
        const float s = g2 ? g1[i] + g2[i] : g1[i];
        res[i] = (!out || out[i] > 0.0f) ? s : 0.0f;
    }
}

/* the same where the second gradient lives on a lattice: g2s [N,C,ceil(H/s),ceil(W/s)] is the gradient of a tensor
 * that was read at every s-th row and column only (a 1x1 convolution with stride s and no padding), so it reaches
 * position (h, w) of the [N,C,H,W] tensor only where h and w are multiples of s; elsewhere 0 is added */
void orc_relu_bwd_sum_lattice(const float *g1, const float *g2s, const float *out, int N, int C, int H, int W, int s,
                              float *res)
{
    const int Hs = (H + s - 1) / s, Ws = (W + s - 1) / s;
    for (int64_t pl = 0; pl < (int64_t)N * C; ++pl)
        for (int h = 0; h < H; ++h)
            for (int w = 0; w < W; ++w) {
                const int64_t i = (pl * H + h) * W + w;
                const float t = (h % s == 0 && w % s == 0) ? g2s[(pl * Hs + h / s) * Ws + w / s] : 0.0f;
                const float sum = g1[i] + t;
                res[i] = (!out || out[i] > 0.0f) ? sum : 0.0f;
            }
}

/* backward of out = relu(.): g passes where out > 0; with `other` (nullable) added to it */
void orc_relu_bwd_add(const float *g, const float *out, const float *other, int64_t n, float *res)
{
    for (int64_t i = 0; i < n; ++i) {
        const float m = out[i] > 0.0f ? g[i] : 0.0f;
        res[i] = other ? m + other[i] : m;
    }
}
