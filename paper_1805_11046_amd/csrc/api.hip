// C-ABI entry points of the product calls: argument checks on the host, then dispatch to the
// specialised kernel for the shape if there is one, else to the general kernel.
#include "q8t_common.h"
#include <vector>

#include "q8t_internal.h"
#include "repack.h"

namespace {

constexpr int kMaxRed32 = 33025;  // 255*255*K < 2^31  (32-bit accumulator contract of fwd / dgrad)

int fc_check(int M, int N, int K, const void *a, const void *qa, const void *b, const void *qb, const void *o1,
             const void *o2)
{
    if (M <= 0 || N <= 0 || K <= 0) return Q8T_ERR_SHAPE;
    if ((int64_t)M * N >= ((int64_t)1 << 31) || (int64_t)M * K >= ((int64_t)1 << 31) ||
        (int64_t)K * N >= ((int64_t)1 << 31))
        return Q8T_ERR_SHAPE;
    if (!a || !qa || !b || !qb || (!o1 && !o2)) return Q8T_ERR_NULL;
    return Q8T_OK;
}

// the im2col + GEMM form of a forward with few input channels pays off once the product is not tiny
bool smallc_wanted(int which, const q8t_conv_desc *d)
{
    if (!q8t_smallc_conv_supported(which, d)) return false;
    const int P = (d->H + 2 * d->pad - d->R) / d->stride + 1, Q = (d->W + 2 * d->pad - d->S) / d->stride + 1;
    return (double)d->K * d->C * d->R * d->S * d->N * P * Q >= 4194304.0;
}

// the GEMM form of the weight gradient pays off once the product is not tiny
bool wgrad_wants_gemm(const q8t_conv_desc *d)
{
    if (!q8t_gemm_wgrad_supported(d)) return false;
    const int P = (d->H + 2 * d->pad - d->R) / d->stride + 1, Q = (d->W + 2 * d->pad - d->S) / d->stride + 1;
    return (double)d->K * d->C * d->R * d->S * d->N * P * Q >= 4194304.0;
}

// bytes of partial statistics that the forward kernel for this shape writes from its epilogue (0: none there)
size_t stats_in_epilogue_ws(const q8t_conv_desc *d)
{
    if (q8t_nhwc_conv_supported(0, d)) return q8t_nhwc_conv_stats_ws(d);
    size_t s = smallc_wanted(0, d) ? q8t_smallc_conv_stats_ws(d) : 0;
    const size_t f = q8t_first_conv_stats_ws(d);   // which of the two runs also depends on the pointers
    return f > s ? f : s;
}

// A 1x1 convolution with a stride and no padding is the stride-1 layer on the positions it reads: where the
// register-tile kernel takes that reduced shape, the forward product gathers those codes into the workspace
// (a quarter of the operand at stride 2) and runs there, instead of rewriting the whole operand channel-contiguous
// for the general strided path.
bool lattice_forward(const q8t_conv_desc *d, q8t_conv_desc *sub)
{
    if (d->R != 1 || d->S != 1 || d->pad != 0 || d->stride < 2 || d->H < 1 || d->W < 1) return false;
    *sub = *d;
    sub->H = (d->H - 1) / d->stride + 1;
    sub->W = (d->W - 1) / d->stride + 1;
    sub->stride = 1;
    return q8t_fast_conv_ws(0, sub) != 0;   // the shape is one the register-tile kernel takes
}
size_t lattice_codes_bytes(const q8t_conv_desc *sub) { return ((size_t)sub->N * sub->C * sub->H * sub->W + 255) & ~(size_t)255; }

// The layout (repack.h) in which the forward (which = 0) or layer-gradient (1) product of this shape reads its filter
// when its operands are aligned, decided by the shape alone and in the order the products route; Q8T_PACK_NONE: the
// path that serves the shape has no filter pre-pass to take out.
int pack_layout(const q8t_conv_desc *d, int which)
{
    if (!d || which < 0 || which > 1 || q8t_conv_reduction_check(which, d)) return Q8T_PACK_NONE;
    q8t_conv_desc sub;
    if (which == 0 && lattice_forward(d, &sub)) return Q8T_PACK_TILE64;   // the same filter layout as on the full shape
    const int w = q8t_wide_conv_pack_layout(which, d);
    if (w != Q8T_PACK_NONE) return w;
    return q8t_fast_conv_ws(which, d) ? Q8T_PACK_TILE64 : Q8T_PACK_NONE;
}
// the packed filter for a branch that reads layout `want`, if the caller's buffer holds that one
// the caller's packed filter for the register-tile kernel / for the wide-tile kernel, if it holds that layout
const void *packed_tile64(const void *packed, const q8t_conv_desc *d, int which)
{
    return packed && pack_layout(d, which) == Q8T_PACK_TILE64 ? packed : nullptr;
}
const void *packed_wide(const void *packed, const q8t_conv_desc *d, int which)
{
    const int l = packed ? pack_layout(d, which) : Q8T_PACK_NONE;
    return l == Q8T_PACK_WIDE256 || l == Q8T_PACK_WIDE128 ? packed : nullptr;
}

}  // namespace

extern "C" {

const char *q8t_version(void) { return "q8t 0.1 (gfx950)"; }

size_t q8t_qgemm_workspace_size(int M, int N, int K, int which)
{
    if (M <= 0 || N <= 0 || K <= 0 || which < 0 || which > 2) return 0;
    return q8t_generic_fc_ws(which, M, N, K);
}

int q8t_qgemm_fwd(const int8_t *qx, const q8t_qparams *px, const int8_t *qw, const q8t_qparams *pw, int M, int N,
                  int K, float *y, int32_t *acc_out, void *ws, void *stream)
{
    const int rc = fc_check(M, N, K, qx, px, qw, pw, y, acc_out);
    if (rc) return rc;
    if (K > kMaxRed32) return Q8T_ERR_OVERFLOW;
    return q8t_generic_fc(0, qx, px, qw, pw, M, N, K, y, acc_out, ws, (hipStream_t)stream);
}

int q8t_qgemm_dgrad(const int8_t *qdy, const q8t_qparams *pg, const int8_t *qw, const q8t_qparams *pw, int M,
                    int N, int K, float *dx, int32_t *acc_out, void *ws, void *stream)
{
    const int rc = fc_check(M, N, K, qdy, pg, qw, pw, dx, acc_out);
    if (rc) return rc;
    if (N > kMaxRed32) return Q8T_ERR_OVERFLOW;
    return q8t_generic_fc(1, qdy, pg, qw, pw, M, N, K, dx, acc_out, ws, (hipStream_t)stream);
}

int q8t_qgemm_wgrad(const int8_t *qx, const q8t_qparams *px, const int16_t *qdy16, const q8t_qparams *pg16, int M,
                    int N, int K, float *dw, int64_t *acc_out, void *ws, void *stream)
{
    const int rc = fc_check(M, N, K, qx, px, qdy16, pg16, dw, acc_out);
    if (rc) return rc;
    return q8t_generic_fc(2, qdy16, pg16, qx, px, M, N, K, dw, acc_out, ws, (hipStream_t)stream);
}

size_t q8t_qconv_workspace_size(const q8t_conv_desc *desc, int which)
{
    if (!desc || which < 0 || which > 2) return 0;
    size_t g = q8t_generic_conv_ws(which, desc);
    size_t f = q8t_fast_conv_ws(which, desc);
    if (which < 2) {
        const size_t wd = q8t_wide_conv_ws(which, desc);
        if (wd > f) f = wd;
    }
    if (which == 2) {
        f = q8t_fast_wgrad_ws(desc);
        const size_t pw = q8t_planes_wgrad_ws(desc);
        if (pw > f) f = pw;
    }
    size_t h = which < 2 ? q8t_nhwc_conv_ws(which, desc) : (wgrad_wants_gemm(desc) ? q8t_gemm_wgrad_ws(desc) : 0);
    if (smallc_wanted(which, desc)) h = q8t_smallc_conv_ws(which, desc);
    if (which == 0 && q8t_first_conv_ws(desc) > h) h = q8t_first_conv_ws(desc);
    q8t_conv_desc sub;
    if (which == 0 && lattice_forward(desc, &sub)) {
        const size_t l = lattice_codes_bytes(&sub) + q8t_fast_conv_ws(0, &sub);
        if (l > h) h = l;
    }
    if (h > g) g = h;
    return g > f ? g : f;
}

static int qconv_fwd_impl(const q8t_conv_desc *desc, const int8_t *qx, const q8t_qparams *px, const int8_t *qw,
                          const q8t_qparams *pw, float *y, int32_t *acc_out, void *ws, void *stream, const void *packed)
{
    if (!desc || !qx || !px || !qw || !pw || (!y && !acc_out)) return Q8T_ERR_NULL;
    const int rc = q8t_conv_reduction_check(0, desc);
    if (rc) return rc;
    q8t_conv_desc sub;
    if (lattice_forward(desc, &sub) && ws && q8t_aligned(ws, 16)) {
        int8_t *codes = (int8_t *)ws;
        void *ws2 = (char *)ws + lattice_codes_bytes(&sub);
        if (q8t_fast_conv_supported(0, &sub, codes, qw, y, acc_out)) {
            const int rs = q8t_subsample_codes(qx, desc->N, desc->C, desc->H, desc->W, desc->stride, codes, (hipStream_t)stream);
            if (rs) return rs;
            return q8t_fast_conv(0, &sub, codes, px, qw, pw, y, acc_out, nullptr, ws2, (hipStream_t)stream, nullptr,
                                 packed_tile64(packed, desc, 0));
        }
    }
    if (q8t_wide_conv_supported(0, desc, qx, y, acc_out))
        return q8t_wide_conv(0, desc, qx, px, qw, pw, y, acc_out, nullptr, ws, (hipStream_t)stream, packed_wide(packed, desc, 0));
    if (q8t_fast_conv_supported(0, desc, qx, qw, y, acc_out))
        return q8t_fast_conv(0, desc, qx, px, qw, pw, y, acc_out, nullptr, ws, (hipStream_t)stream, nullptr,
                             packed_tile64(packed, desc, 0));
    if (q8t_nhwc_conv_supported(0, desc))
        return q8t_nhwc_conv(0, desc, qx, px, qw, pw, y, acc_out, nullptr, nullptr, ws, (hipStream_t)stream);
    if (q8t_first_conv_supported(desc, qx, y, acc_out))
        return q8t_first_conv(desc, qx, px, qw, pw, y, acc_out, nullptr, nullptr, ws, (hipStream_t)stream);
    if (smallc_wanted(0, desc)) return q8t_smallc_conv(desc, qx, px, qw, pw, y, acc_out, nullptr, nullptr, ws, (hipStream_t)stream);
    return q8t_generic_conv(0, desc, qx, px, qw, pw, y, acc_out, ws, (hipStream_t)stream);
}

int q8t_qconv_fwd(const q8t_conv_desc *desc, const int8_t *qx, const q8t_qparams *px, const int8_t *qw,
                  const q8t_qparams *pw, float *y, int32_t *acc_out, void *ws, void *stream)
{
    return qconv_fwd_impl(desc, qx, px, qw, pw, y, acc_out, ws, stream, nullptr);
}

size_t q8t_qconv_fwd_bn_stats_workspace_size(const q8t_conv_desc *desc)
{
    if (!desc || desc->stride < 1) return 0;
    const int P = (desc->H + 2 * desc->pad - desc->R) / desc->stride + 1, Q = (desc->W + 2 * desc->pad - desc->S) / desc->stride + 1;
    const size_t c = (q8t_qconv_workspace_size(desc, 0) + 255) & ~(size_t)255;
    // behind the product's own workspace: the partial statistics of its epilogue, or the workspace of a
    // statistics pass over the result where the kernel for this shape gathers none
    size_t s = q8t_range_bn_workspace_size(desc->N, desc->K, P, Q);
    const size_t e = stats_in_epilogue_ws(desc);
    if (e > s) s = e;
    return c + s;
}

static int qconv_fwd_bn_stats_impl(const q8t_conv_desc *desc, const int8_t *qx, const q8t_qparams *px, const int8_t *qw,
                                   const q8t_qparams *pw, float *y, int32_t *acc_out, float *stats_out, void *ws, void *stream,
                                   const void *packed)
{
    if (!desc || !qx || !px || !qw || !pw || !y || !stats_out) return Q8T_ERR_NULL;
    const int rc = q8t_conv_reduction_check(0, desc);
    if (rc) return rc;
    if (!ws || !q8t_aligned(ws, 16)) return Q8T_ERR_WORKSPACE;
    q8t_conv_desc sub;
    if (lattice_forward(desc, &sub)) {
        int8_t *codes = (int8_t *)ws;
        void *ws2 = (char *)ws + lattice_codes_bytes(&sub);
        if (q8t_fast_conv_supported(0, &sub, codes, qw, y, acc_out)) {
            const int rs = q8t_subsample_codes(qx, desc->N, desc->C, desc->H, desc->W, desc->stride, codes, (hipStream_t)stream);
            if (rs) return rs;
            return q8t_fast_conv(0, &sub, codes, px, qw, pw, y, acc_out, stats_out, ws2, (hipStream_t)stream, nullptr,
                                 packed_tile64(packed, desc, 0));
        }
    }
    // the specialised kernel gathers the statistics in its epilogue; other shapes run the product
    // and then the statistics pass of the Range BN over its result
    if (q8t_wide_conv_supported(0, desc, qx, y, acc_out))
        return q8t_wide_conv(0, desc, qx, px, qw, pw, y, acc_out, stats_out, ws, (hipStream_t)stream, packed_wide(packed, desc, 0));
    if (q8t_fast_conv_supported(0, desc, qx, qw, y, acc_out))
        return q8t_fast_conv(0, desc, qx, px, qw, pw, y, acc_out, stats_out, ws, (hipStream_t)stream, nullptr,
                             packed_tile64(packed, desc, 0));
    void *sws = (char *)ws + ((q8t_qconv_workspace_size(desc, 0) + 255) & ~(size_t)255);
    if (q8t_nhwc_conv_supported(0, desc))
        return q8t_nhwc_conv(0, desc, qx, px, qw, pw, y, acc_out, stats_out, sws, ws, (hipStream_t)stream);
    if (q8t_first_conv_supported(desc, qx, y, acc_out))
        return q8t_first_conv(desc, qx, px, qw, pw, y, acc_out, stats_out, sws, ws, (hipStream_t)stream);
    if (smallc_wanted(0, desc) && q8t_smallc_conv_stats_ws(desc))
        return q8t_smallc_conv(desc, qx, px, qw, pw, y, acc_out, stats_out, sws, ws, (hipStream_t)stream);
    const int rc2 = qconv_fwd_impl(desc, qx, px, qw, pw, y, acc_out, ws, stream, packed);
    if (rc2) return rc2;
    const int P = (desc->H + 2 * desc->pad - desc->R) / desc->stride + 1, Q = (desc->W + 2 * desc->pad - desc->S) / desc->stride + 1;
    void *bnws = (char *)ws + ((q8t_qconv_workspace_size(desc, 0) + 255) & ~(size_t)255);
    return q8t_range_bn_stats(y, desc->N, desc->K, P, Q, stats_out, bnws, (hipStream_t)stream);
}

int q8t_qconv_fwd_bn_stats(const q8t_conv_desc *desc, const int8_t *qx, const q8t_qparams *px, const int8_t *qw,
                           const q8t_qparams *pw, float *y, int32_t *acc_out, float *stats_out, void *ws, void *stream)
{
    return qconv_fwd_bn_stats_impl(desc, qx, px, qw, pw, y, acc_out, stats_out, ws, stream, nullptr);
}

static int qconv_dgrad_impl(const q8t_conv_desc *desc, const int8_t *qdy, const q8t_qparams *pg, const int8_t *qw,
                            const q8t_qparams *pw, float *dx, int32_t *acc_out, void *ws, void *stream, const void *packed)
{
    if (!desc || !qdy || !pg || !qw || !pw || (!dx && !acc_out)) return Q8T_ERR_NULL;
    const int rc = q8t_conv_reduction_check(1, desc);
    if (rc) return rc;
    if (q8t_wide_conv_supported(1, desc, qdy, dx, acc_out))
        return q8t_wide_conv(1, desc, qdy, pg, qw, pw, dx, acc_out, nullptr, ws, (hipStream_t)stream, packed_wide(packed, desc, 1));
    if (q8t_fast_conv_supported(1, desc, qdy, qw, dx, acc_out))
        return q8t_fast_conv(1, desc, qdy, pg, qw, pw, dx, acc_out, nullptr, ws, (hipStream_t)stream, nullptr,
                             packed_tile64(packed, desc, 1));
    if (q8t_nhwc_conv_supported(1, desc))
        return q8t_nhwc_conv(1, desc, qdy, pg, qw, pw, dx, acc_out, nullptr, nullptr, ws, (hipStream_t)stream);
    return q8t_generic_conv(1, desc, qdy, pg, qw, pw, dx, acc_out, ws, (hipStream_t)stream);
}

int q8t_qconv_dgrad(const q8t_conv_desc *desc, const int8_t *qdy, const q8t_qparams *pg, const int8_t *qw,
                    const q8t_qparams *pw, float *dx, int32_t *acc_out, void *ws, void *stream)
{
    return qconv_dgrad_impl(desc, qdy, pg, qw, pw, dx, acc_out, ws, stream, nullptr);
}

static int qconv_dgrad_relu_sum_impl(const q8t_conv_desc *desc, const int8_t *qdy, const q8t_qparams *pg, const int8_t *qw,
                                     const q8t_qparams *pw, const float *other, const float *act, float *dx, void *ws,
                                     void *stream, const void *packed)
{
    if (!desc || !qdy || !pg || !qw || !pw || !act || !dx) return Q8T_ERR_NULL;
    const int rc = q8t_conv_reduction_check(1, desc);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    const Q8tReluSum rs = {other, act};
    const bool al = q8t_aligned(other, 16) && q8t_aligned(act, 16) && q8t_aligned(dx, 16);
    // The register-tile kernel of the large planes finishes the block's gradient in its epilogue.  Measured on the
    // other kernels (stride-2 pairs, wide tiles on 14x14 / 7x7 planes): the two extra operands cost their exposed
    // write-out more than the separate pass does, so those shapes, like every other one, run the product and then
    // the plumbing pass in place.
    if (al && !q8t_wide_conv_supported(1, desc, qdy, dx, nullptr) && q8t_fast_conv_supported(1, desc, qdy, qw, dx, nullptr))
        return q8t_fast_conv(1, desc, qdy, pg, qw, pw, dx, nullptr, nullptr, ws, st, &rs, packed_tile64(packed, desc, 1));
    const int r2 = qconv_dgrad_impl(desc, qdy, pg, qw, pw, dx, nullptr, ws, stream, packed);
    if (r2) return r2;
    return q8t_relu_bwd_sum(dx, other, act, (int64_t)desc->N * desc->C * desc->H * desc->W, dx, stream);
}

int q8t_qconv_dgrad_relu_sum(const q8t_conv_desc *desc, const int8_t *qdy, const q8t_qparams *pg, const int8_t *qw,
                             const q8t_qparams *pw, const float *other, const float *act, float *dx, void *ws, void *stream)
{
    return qconv_dgrad_relu_sum_impl(desc, qdy, pg, qw, pw, other, act, dx, ws, stream, nullptr);
}

// ---- filters packed ahead of the products ----
size_t q8t_qconv_pack_size(const q8t_conv_desc *desc, int which)
{
    return pack_layout(desc, which) == Q8T_PACK_NONE ? 0 : q8t_pack_bytes(which, desc);
}

int q8t_qconv_pack_multi(int n, const q8t_conv_desc *descs, const int *which, const int8_t *const *qw, void *const *packed,
                         void *stream)
{
    if (n < 0 || (n > 0 && (!descs || !which || !qw || !packed))) return Q8T_ERR_NULL;
    std::vector<Q8tPackJob> jobs;
    jobs.reserve((size_t)n);
    for (int i = 0; i < n; ++i) {
        const int lay = pack_layout(&descs[i], which[i]);
        if (lay == Q8T_PACK_NONE || !packed[i]) continue;   // nothing to pack ahead for this product
        if (!qw[i]) return Q8T_ERR_NULL;
        if (!q8t_aligned(packed[i], 16)) return Q8T_ERR_WORKSPACE;
        Q8tPackJob j;
        j.w = qw[i];
        j.out = (int8_t *)packed[i];
        j.colsum = (int *)((char *)packed[i] + q8t_pack_colsum_offset(&descs[i]));
        j.Kf = descs[i].K;
        j.Cf = descs[i].C;
        j.R = descs[i].R;
        j.S = descs[i].S;
        j.dgrad = which[i];
        j.layout = lay;
        j.first_block = 0;
        jobs.push_back(j);
    }
    return q8t_pack_launch(jobs.data(), (int)jobs.size(), (hipStream_t)stream);
}

int q8t_qconv_fwd_bn_stats_packed(const q8t_conv_desc *desc, const int8_t *qx, const q8t_qparams *px, const int8_t *qw,
                                  const q8t_qparams *pw, const void *packed, float *y, int32_t *acc_out, float *stats_out,
                                  void *ws, void *stream)
{
    return qconv_fwd_bn_stats_impl(desc, qx, px, qw, pw, y, acc_out, stats_out, ws, stream, packed);
}

int q8t_qconv_dgrad_packed(const q8t_conv_desc *desc, const int8_t *qdy, const q8t_qparams *pg, const int8_t *qw,
                           const q8t_qparams *pw, const void *packed, float *dx, int32_t *acc_out, void *ws, void *stream)
{
    return qconv_dgrad_impl(desc, qdy, pg, qw, pw, dx, acc_out, ws, stream, packed);
}

int q8t_qconv_dgrad_relu_sum_packed(const q8t_conv_desc *desc, const int8_t *qdy, const q8t_qparams *pg, const int8_t *qw,
                                    const q8t_qparams *pw, const void *packed, const float *other, const float *act, float *dx,
                                    void *ws, void *stream)
{
    return qconv_dgrad_relu_sum_impl(desc, qdy, pg, qw, pw, other, act, dx, ws, stream, packed);
}

int q8t_qconv_wgrad(const q8t_conv_desc *desc, const int8_t *qx, const q8t_qparams *px, const int16_t *qdy16,
                    const q8t_qparams *pg16, float *dw, int64_t *acc_out, void *ws, void *stream)
{
    if (!desc || !qx || !px || !qdy16 || !pg16 || (!dw && !acc_out)) return Q8T_ERR_NULL;
    const int rc = q8t_conv_reduction_check(2, desc);
    if (rc) return rc;
    if (q8t_planes_wgrad_supported(desc, qdy16, qx, dw, acc_out))
        return q8t_planes_wgrad(desc, qdy16, pg16, qx, px, dw, acc_out, ws, (hipStream_t)stream);
    if (q8t_fast_wgrad_supported(desc, qdy16, qx, dw, acc_out))
        return q8t_fast_wgrad(desc, qdy16, pg16, qx, px, dw, acc_out, ws, (hipStream_t)stream);
    if (wgrad_wants_gemm(desc))
        return q8t_gemm_wgrad(desc, qdy16, pg16, qx, px, dw, acc_out, ws, (hipStream_t)stream);
    return q8t_generic_conv(2, desc, qdy16, pg16, qx, px, dw, acc_out, ws, (hipStream_t)stream);
}

}  // extern "C"
