/*
 * q8t.h -- C ABI of libq8t: the quantized back-propagation step of a conv/FC layer plus
 * Range Batch-Norm, as hand-written HIP kernels for gfx950 (MI355X).
 *
 * Method: "Scalable Methods for 8-bit Training of Neural Networks" (Banner, Hubara, Hoffer,
 * Soudry).  Each entry point cites the passage that defines its operation.
 *
 * Conventions (all entry points)
 *  - Every pointer is a DEVICE pointer unless the comment says "host".  The caller owns every
 *    buffer, including the workspace `ws` (size from the matching *_workspace_size query, 256-byte
 *    aligned; contents on entry are irrelevant, contents on return are unspecified).
 *  - The library allocates nothing and never synchronizes the host: all work is enqueued on
 *    `stream` (a hipStream_t passed as void*; NULL = the default stream).  The only state it keeps
 *    between calls is, per device, the address of the static scratch array of q8t_quantize_noalloc
 *    (looked up once, under a mutex); results never depend on earlier calls.
 *  - Float tensors are contiguous NCHW (conv / Range BN) or row-major (FC).
 *  - Quantized payloads are SIGNED: an M-bit level q in [0, 2^M-1] is stored as q - 2^(M-1),
 *    int8 for M <= 8 and int16 for 8 < M <= 16, in the same logical layout as the float source.
 *  - Return value: Q8T_OK or a negative error code.  Shapes, bit widths and pointers are checked
 *    on the host before anything is launched; on error nothing has been enqueued.
 */
#ifndef Q8T_H
#define Q8T_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    Q8T_OK = 0,
    Q8T_ERR_NULL = -1,      /* a required pointer is NULL */
    Q8T_ERR_SHAPE = -2,     /* a dimension is <= 0 or beyond what index arithmetic supports */
    Q8T_ERR_BITS = -3,      /* bit width outside [2,16] (or not 8 / 16 where fixed) */
    Q8T_ERR_OVERFLOW = -4,  /* reduction length too large for the 32-bit accumulator contract */
    Q8T_ERR_WORKSPACE = -5, /* ws is NULL or misaligned although the call needs one */
    Q8T_ERR_HIP = -6        /* a launch was rejected by the runtime */
};

/* Affine quantization parameters (Appendix B).  Device-resident: written by the quantize calls,
 * read by the product calls, never touched by the host inside the library.
 *   real value = scale * (level - zero_point),  level = stored + 2^(bits-1).                  */
typedef struct {
    float vmin, vmax;      /* clamping range after it was widened to contain 0 */
    float scale;           /* (vmax - vmin) / (2^bits - 1); 1 for an all-zero tensor */
    float inv_scale;       /* fl32(1 / scale) */
    int32_t zero_point;    /* level of the real value 0, in [0, 2^bits - 1] */
    int32_t bits;
} q8t_qparams;

/* Convolution geometry: input [N,C,H,W], filter [K,C,R,S], output [N,K,P,Q] with
 * P = (H + 2*pad - R)/stride + 1 (Q likewise); zero padding, no bias, no dilation, no groups. */
typedef struct {
    int N, C, H, W, K, R, S, stride, pad;
} q8t_conv_desc;

/* ---------------------------------------------------------------------------------------------
 * Quantization (Appendix B; Section 4 "Quantization methods").
 *
 *   vmin = min(min_i x_i, 0), vmax = max(max_i x_i, 0)
 *   scale = (vmax - vmin)/(2^M - 1), zero_point = round(-vmin/scale) clamped to [0, 2^M - 1]
 *   level_i = clamp(round(x_i * inv_scale + zero_point), 0, 2^M - 1)
 * evaluated in fp32 with one rounding per operation (no fused multiply-add); round is
 * round-half-to-even.  With stochastic != 0 (Section 4: required for gradients) the level is
 * floor(t) + [frac(t)*65536 > r + 0.5] where r are 16 bits of a stateless counter-based generator
 * keyed by (seed, flat element index).
 *
 * x: n floats.  q_out: n int8 (bits <= 8) or n int16.  qp_out: one q8t_qparams.  n may be 0
 * (then qp_out describes the range [0,0]).  n <= 2^34.
 */
size_t q8t_quantize_workspace_size(int64_t n);
int q8t_quantize(const float *x, int64_t n, int bits, int stochastic, uint64_t seed, void *q_out,
                 q8t_qparams *qp_out, void *ws, void *stream);

/* For callers that cannot allocate device memory or carry a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): q8t_quantize with the (min,max) pairs of
 * its first pass kept in a file-scope `static __device__` array of the library (8 KiB; every GPU the
 * library runs on holds its own copy until the process ends) instead of a caller workspace.  Same
 * arguments, checks and results as q8t_quantize, bit for bit.  Calls no hipMalloc / hipFree and no
 * allocating routine.  n <= Q8T_NOALLOC_MAX_ELEMENTS, else Q8T_ERR_SHAPE (the scratch does not grow
 * with n; the limit is that of the 32-bit group counter of the generator, as for q8t_quantize).
 * The device that `stream` belongs to must be the current device.  All calls on one GPU share that
 * GPU's array: the pairs a call reads are the ones it has just written (nothing needs to start at
 * zero), but two calls that overlap in time on one GPU (different streams) race on it.
 * q8t_init() looks up the array's device address for the current device (what the first call on a
 * device does by itself); call it once per device before stream capture.  Returns Q8T_OK or
 * Q8T_ERR_HIP. */
#define Q8T_NOALLOC_MAX_ELEMENTS ((int64_t)1 << 34)
int q8t_init(void);
int q8t_quantize_noalloc(const float *x, int64_t n, int bits, int stochastic, uint64_t seed, void *q_out,
                         q8t_qparams *qp_out, void *stream);

/* Several tensors at once (the weights of a network at the start of a step: dozens of small tensors, each of
 * which would otherwise cost one or two launches of its own).  x, n, q_out, qp_out: HOST arrays of `count`
 * entries; x[t], q_out[t], qp_out[t] are device pointers, n[t] the element count of tensor t.  Nearest rounding,
 * bits <= 8, every tensor with its own range: the result for tensor t is that of
 * q8t_quantize(x[t], n[t], bits, 0, ...), bit for bit.  Two launches per 32 tensors.
 * ws: q8t_quantize_multi_workspace_size(count, n) bytes (n: the same host array). */
size_t q8t_quantize_multi_workspace_size(int count, const int64_t *n);
int q8t_quantize_multi(int count, const float *const *x, const int64_t *n, int bits, int8_t *const *q_out,
                       q8t_qparams *const *qp_out, void *ws, void *stream);

/* Same, with the range supplied instead of searched: vmin_vmax points to 2 device floats
 * (Section 4: the range of an activation is already known to the preceding Range BN).  Values
 * outside the range saturate.  Needs no workspace. */
int q8t_quantize_with_range(const float *x, int64_t n, int bits, int stochastic, uint64_t seed,
                            const float *vmin_vmax, void *q_out, q8t_qparams *qp_out, void *stream);

/* Clamping range of an activation tensor averaged over chunks (Appendix B, "Quantization methods":
 * the clamping values of the activations are the average of the maximum and of the minimum over K
 * chunks).  The flat tensor is cut into K contiguous chunks of ceil(n/K) elements (the last may be
 * shorter; chunks that would start past the end do not exist and are not counted).
 * range_out: 2 device floats {vmin, vmax} = fp32(mean of the chunk minima), fp32(mean of the chunk
 * maxima), each mean taken in fp64 in chunk order.  Feed it to q8t_quantize_with_range: values
 * outside saturate.  1 <= K <= min(n, 65535).  Workspace: device,
 * q8t_chunk_range_workspace_size(n, K) bytes, 8-byte aligned.
 * Errors: Q8T_ERR_SHAPE (n, K), Q8T_ERR_NULL, Q8T_ERR_WORKSPACE, Q8T_ERR_HIP. */
size_t q8t_chunk_range_workspace_size(int64_t n, int K);
int q8t_chunk_range(const float *x, int64_t n, int K, float *range_out, void *ws, void *stream);

/* Angle between a tensor and its quantized copy (Section 5.1 (Problem Statement), eq. (1)):
 * cos(theta) = (x . Q(x)) / (||x||_2 ||Q(x)||_2), Q(x) = scale * (level - zero_point) of the stored
 * codes q (int8 for qp->bits <= 8, else int16; as q8t_dequantize returns them).
 * out: 4 device doubles { x.Q(x), ||x||^2, ||Q(x)||^2, cos(theta) } (cos = 0 if a norm is 0); sums
 * in fp64.  Workspace: device, q8t_quant_angle_workspace_size(n) bytes, 8-byte aligned.
 * Errors: Q8T_ERR_SHAPE, Q8T_ERR_NULL, Q8T_ERR_WORKSPACE, Q8T_ERR_HIP. */
size_t q8t_quant_angle_workspace_size(int64_t n);
int q8t_quant_angle(const float *x, const void *q, const q8t_qparams *qp, int64_t n, double *out, void *ws,
                    void *stream);

/* Gradient bifurcation (Section 1; Section 7): one pass over g yields the 8-bit copy that feeds
 * the layer gradient and the 16-bit copy that feeds the weight gradient.  Both share g's min/max
 * and use stochastic rounding with their own seeds.  ws: q8t_quantize_workspace_size(n). */
int q8t_quantize_bifurcate(const float *g, int64_t n, uint64_t seed8, uint64_t seed16, int8_t *q8_out,
                           q8t_qparams *qp8_out, int16_t *q16_out, q8t_qparams *qp16_out, void *ws,
                           void *stream);

/* out_i = scale * (level_i - zero_point).  q holds int8 or int16 according to qp->bits. */
int q8t_dequantize(const void *q, const q8t_qparams *qp, int64_t n, float *out, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Fully connected layer, row-major (Section 4, eqs. (grad_layer) and (grad_weight)).
 *   fwd  : Y [M,N] = X[M,K]  * W[K,N]
 *   dgrad: dX[M,K] = dY[M,N] * W[K,N]^T           (8-bit copy of dY, stochastic)
 *   wgrad: dW[K,N] = X[M,K]^T * dY16[M,N]         (16-bit copy of dY, 8-bit layer input)
 * Operands are stored codes with their device-resident parameters.  The integer accumulator is
 *   acc = sum_k (level_a - zero_a) * (level_b - zero_b)
 * exact, and the float result is fl32(scale_a*scale_b) * (float)acc for fwd/dgrad and
 * (float)((double)acc * (double)fl32(scale_a*scale_b)) for wgrad.  `acc_out` (nullable) receives
 * the accumulator itself: int32 for fwd/dgrad, int64 for wgrad.  The float output is nullable too.
 * fwd/dgrad require a reduction length <= 33025 (so that |acc| < 2^31), else Q8T_ERR_OVERFLOW;
 * wgrad accepts any M (partial sums are reduced in 64 bits).
 * which: 0 fwd, 1 dgrad, 2 wgrad.
 */
size_t q8t_qgemm_workspace_size(int M, int N, int K, int which);
int q8t_qgemm_fwd(const int8_t *qx, const q8t_qparams *px, const int8_t *qw, const q8t_qparams *pw,
                  int M, int N, int K, float *y, int32_t *acc_out, void *ws, void *stream);
int q8t_qgemm_dgrad(const int8_t *qdy, const q8t_qparams *pg, const int8_t *qw, const q8t_qparams *pw,
                    int M, int N, int K, float *dx, int32_t *acc_out, void *ws, void *stream);
int q8t_qgemm_wgrad(const int8_t *qx, const q8t_qparams *px, const int16_t *qdy16,
                    const q8t_qparams *pg16, int M, int N, int K, float *dw, int64_t *acc_out,
                    void *ws, void *stream);

/* Forward convolution that also returns the Range BN statistics of its result (Sec. 3: mean, min
 * and max per output channel; Sec. 4: the range is known to the normalizer, no extra pass).
 * Same arguments as q8t_qconv_fwd, y required; stats_out: device, [3][K] floats = mean, min, max
 * over the N*P*Q values of each output channel -- what q8t_range_bn_fwd would write into its
 * stats_out for y.  min/max are exact; the mean is taken from the exact integer sum of the
 * accumulators (differs from a float scan of y by rounding only).  Workspace: device,
 * q8t_qconv_fwd_bn_stats_workspace_size(desc) bytes, 16-byte aligned.  Errors as q8t_qconv_fwd. */
size_t q8t_qconv_fwd_bn_stats_workspace_size(const q8t_conv_desc *desc);
int q8t_qconv_fwd_bn_stats(const q8t_conv_desc *desc, const int8_t *qx, const q8t_qparams *px, const int8_t *qw,
                           const q8t_qparams *pw, float *y, int32_t *acc_out, float *stats_out, void *ws, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Convolution layer, NCHW (same three products, Section 4).  A padded tap contributes nothing.
 *   fwd  : Y [n,k,p,q] = sum_{c,r,s} X[n,c,p*st+r-pad,q*st+s-pad] * W[k,c,r,s]
 *   dgrad: dX[n,c,h,w] = sum_{k,r,s} dY[n,k,p,q] * W[k,c,r,s]   over p*st+r-pad = h, q*st+s-pad = w
 *   wgrad: dW[k,c,r,s] = sum_{n,p,q} dY16[n,k,p,q] * X[n,c,p*st+r-pad,q*st+s-pad]
 * Same accumulator / scaling / acc_out contract as the FC calls (reduction lengths C*R*S, K*R*S
 * and N*P*Q respectively).
 */
size_t q8t_qconv_workspace_size(const q8t_conv_desc *desc /* host */, int which);
int q8t_qconv_fwd(const q8t_conv_desc *desc /* host */, const int8_t *qx, const q8t_qparams *px,
                  const int8_t *qw, const q8t_qparams *pw, float *y, int32_t *acc_out, void *ws,
                  void *stream);
int q8t_qconv_dgrad(const q8t_conv_desc *desc /* host */, const int8_t *qdy, const q8t_qparams *pg,
                    const int8_t *qw, const q8t_qparams *pw, float *dx, int32_t *acc_out, void *ws,
                    void *stream);
int q8t_qconv_wgrad(const q8t_conv_desc *desc /* host */, const int8_t *qx, const q8t_qparams *px,
                    const int16_t *qdy16, const q8t_qparams *pg16, float *dw, int64_t *acc_out,
                    void *ws, void *stream);

/* The layer gradient of the first convolution of a residual block (Section 4, eq. (grad_layer): the dgrad
 * product above) together with the plumbing that ends the block's backward pass:
 *   dx[i] = act[i] > 0 ? dgrad[i] + other[i] : 0
 * with dgrad the float result q8t_qconv_dgrad would store, other [N,C,H,W] the gradient of the block's other
 * branch (nullable: nothing is added) and act [N,C,H,W] the block's input, through whose rectifier the
 * gradient passes.  Bit-identical to q8t_qconv_dgrad followed by q8t_relu_bwd_sum; where the kernel for the
 * shape has the step in its epilogue (3x3 / 1x1 stride-1 layers on large planes; other, act and dx
 * 16-byte aligned) the product's result never makes the round trip through memory (12 instead of 20
 * bytes per element); other shapes run the two steps one after the other, the second in place.  ws: q8t_qconv_workspace_size(desc, 1).  Errors as q8t_qconv_dgrad. */
int q8t_qconv_dgrad_relu_sum(const q8t_conv_desc *desc /* host */, const int8_t *qdy, const q8t_qparams *pg,
                             const int8_t *qw, const q8t_qparams *pw, const float *other, const float *act,
                             float *dx, void *ws, void *stream);

/* Filters packed ahead of the products.  The forward and the layer-gradient product (Section 4, eqs. (forward),
 * (grad_layer)) of most layer shapes read the 8-bit filter in a kernel-specific order and need the sum of every
 * output channel's codes for the zero-point correction; by default each product call makes both in a small launch of
 * its own in front of the product.  The weights of a training step are quantized once, so a caller can have the
 * filters of all its layers packed by ONE launch, right after the weights are quantized, and hand each product its
 * packed filter.  Results are bit-identical with and without.
 *   q8t_qconv_pack_size(desc, which): bytes of the packed filter for the forward (which = 0) or layer-gradient (1)
 *     product of this shape; 0 where the kernel that serves the shape packs nothing ahead (then pass packed = NULL).
 *   q8t_qconv_pack_multi: n jobs; descs / which: host arrays; qw[i]: device, the layer's codes [K,C,R,S]; packed[i]:
 *     device buffer of q8t_qconv_pack_size(&descs[i], which[i]) bytes, 16-byte aligned, owned by the caller and left
 *     alone by the library after the call; jobs with a size of 0 or packed[i] = NULL are skipped.
 *   the _packed products: as their namesakes, with packed = the buffer made for the same desc, which and codes (or
 *     NULL: behave exactly like the namesake).  Where the operands' alignment sends a call down another kernel than the
 *     shape alone would, the buffer is ignored and the filter is packed in the workspace as usual.  ws as for the
 *     namesake.  A buffer made from other codes or another shape gives wrong results without an error.
 * Errors: Q8T_ERR_NULL, Q8T_ERR_WORKSPACE (misaligned packed buffer), and those of the namesakes. */
size_t q8t_qconv_pack_size(const q8t_conv_desc *desc /* host */, int which);
int q8t_qconv_pack_multi(int n, const q8t_conv_desc *descs /* host */, const int *which /* host */,
                         const int8_t *const *qw /* host array of device pointers */,
                         void *const *packed /* host array of device pointers */, void *stream);
int q8t_qconv_fwd_bn_stats_packed(const q8t_conv_desc *desc /* host */, const int8_t *qx, const q8t_qparams *px,
                                  const int8_t *qw, const q8t_qparams *pw, const void *packed, float *y,
                                  int32_t *acc_out, float *stats_out, void *ws, void *stream);
int q8t_qconv_dgrad_packed(const q8t_conv_desc *desc /* host */, const int8_t *qdy, const q8t_qparams *pg,
                           const int8_t *qw, const q8t_qparams *pw, const void *packed, float *dx,
                           int32_t *acc_out, void *ws, void *stream);
int q8t_qconv_dgrad_relu_sum_packed(const q8t_conv_desc *desc /* host */, const int8_t *qdy, const q8t_qparams *pg,
                                    const int8_t *qw, const q8t_qparams *pw, const void *packed, const float *other,
                                    const float *act, float *dx, void *ws, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Range Batch-Norm over NCHW (Section 3, eq. (range); FC activations: H = W = 1).
 * Per channel c over its n = N*H*W values:
 *   mu = mean(x), range = max(x) - min(x), C(n) = 1/sqrt(2 ln n)
 *   y = gamma_c * (x - mu) / (C(n)*range + eps) + beta_c
 * fp32 elementwise arithmetic, one rounding per operation; the mean is accumulated in fp64.
 * gamma / beta nullable (1 / 0).  stats_out: [3][C] floats = mean, min, max (kept for backward).
 * y is nullable.  If q_out != NULL the output is also emitted as 8-bit codes quantized per tensor,
 * the range taken from the images of each channel's min and max (Section 4: no extra pass over the
 * data), with parameters in qp_out.  Requires n >= 2.
 */
size_t q8t_range_bn_workspace_size(int N, int C, int H, int W);
int q8t_range_bn_fwd(const float *x, int N, int C, int H, int W, const float *gamma,
                     const float *beta, float eps, float *y, float *stats_out, int8_t *q_out,
                     q8t_qparams *qp_out, void *ws, void *stream);

/* Range BN forward with ready-made statistics (Sec. 3, eq. (range)): the normalization pass of
 * q8t_range_bn_fwd alone.  stats: device, [3][C] = mean, min, max (e.g. from
 * q8t_qconv_fwd_bn_stats); y and / or q_out + qp_out as in q8t_range_bn_fwd (at least one output).
 * No workspace.  Errors: Q8T_ERR_SHAPE, Q8T_ERR_NULL, Q8T_ERR_HIP. */
int q8t_range_bn_fwd_apply(const float *x, int N, int C, int H, int W, const float *gamma, const float *beta, float eps,
                           const float *stats, float *y, int8_t *q_out, q8t_qparams *qp_out, void *stream);

/* Backward of the above (Section 7: the derivative of max / min is one at every coordinate that
 * attains it and zero elsewhere).  With g_j = gamma*dy_j, s = C(n)*range + eps:
 *   dbeta = sum dy,  dgamma = sum dy * xhat
 *   dx_j = (g_j - mean(g))/s - C(n)*(sum_i g_i*xhat_i)/s * ([x_j == max] - [x_j == min])
 * stats: the [3][C] array written by the forward call.  dx, dgamma, dbeta are each nullable. */
int q8t_range_bn_bwd(const float *x, const float *dy, const float *stats, int N, int C, int H, int W,
                     const float *gamma, float eps, float *dx, float *dgamma, float *dbeta, void *ws,
                     void *stream);

/* Range BN backward together with the bifurcated quantization of its result (Section 7 for the
 * backward rule; Sections 1 and 4 for the 8-bit / 16-bit stochastic copies of the layer gradient).
 * Inside a channel dx is a monotone function of dy, apart from the -/+ term at the coordinates that
 * attain the channel's max / min; the pass that takes the sums therefore also yields the exact range
 * of dx (from the extremes of dy per kind of coordinate), and the second pass quantizes dx where it
 * is computed: 8 + 8 + 3 bytes per element (+4 if dx is wanted) against 20 + 11 for
 * q8t_range_bn_bwd followed by q8t_quantize_bifurcate, with bit-identical results.
 * dx is nullable (the codes are all the rest of the backward pass consumes); q16_out and qp16_out are
 * required; q8_out is nullable, with qp8_out (the first layer of a network: its input needs no gradient,
 * so only the weight gradient's 16-bit operand is wanted); dgamma / dbeta stay nullable.
 * ws: q8t_range_bn_bwd_bifurcate_workspace_size. */
size_t q8t_range_bn_bwd_bifurcate_workspace_size(int N, int C, int H, int W);
int q8t_range_bn_bwd_bifurcate(const float *x, const float *dy, const float *stats, int N, int C, int H, int W,
                               const float *gamma, float eps, float *dx, float *dgamma, float *dbeta,
                               uint64_t seed8, uint64_t seed16, int8_t *q8_out, q8t_qparams *qp8_out,
                               int16_t *q16_out, q8t_qparams *qp16_out, void *ws, void *stream);

/* Range BN followed by ReLU in one pass (eq. (range) of Section 3, then max(., 0); the 8-bit
 * output follows Section 4's remark that the normalizer already knows the extrema: the range of
 * the rectified output is [max(lo, 0), max(hi, 0)] with lo / hi the images of the channel
 * extrema, so zero is always a code).  Arguments as q8t_range_bn_fwd_apply; with q_out the codes
 * are ready to be the next layer's 8-bit operand and y may be NULL, which leaves 5 bytes per
 * element of traffic where normalization, rectification and quantization as separate passes
 * move 25. */
int q8t_range_bn_relu_fwd_apply(const float *x, int N, int C, int H, int W, const float *gamma, const float *beta,
                                float eps, const float *stats, float *y, int8_t *q_out, q8t_qparams *qp_out,
                                void *stream);

/* Backward of the above fused with the bifurcated quantization: dy is the gradient with respect
 * to the rectified output; it passes where the forward output gamma*xhat + beta (recomputed from
 * x and stats in the forward's fp32 arithmetic) is positive and counts as zero elsewhere
 * (derivative 0 at 0), then the rule of q8t_range_bn_bwd_bifurcate applies, dgamma / dbeta
 * included.  beta and dx are nullable.  Same workspace as q8t_range_bn_bwd_bifurcate. */
int q8t_range_bn_relu_bwd_bifurcate(const float *x, const float *dy, const float *stats, int N, int C, int H, int W,
                                    const float *gamma, const float *beta, float eps, float *dx, float *dgamma,
                                    float *dbeta, uint64_t seed8, uint64_t seed16, int8_t *q8_out,
                                    q8t_qparams *qp8_out, int16_t *q16_out, q8t_qparams *qp16_out, void *ws,
                                    void *stream);

/* C(n) = 1/sqrt(2 ln n) (Section 3), host arithmetic in double.  n >= 2. */
double q8t_range_bn_scale(int64_t n);

/* ---------------------------------------------------------------------------------------------
 * Ternarized back-propagation (appendix "Additional Experiments": gradients ternarized
 * stochastically, weights and activations binarized, products by XNOR + population count, and
 * Algorithm 1, multiple stochastic ternarization sampling, for the weight gradient).  The paper
 * names these operations without defining them; the readings are
 *   StcTern(g)_i = sign(g_i) with probability |g_i| / max|g|, else 0 (unbiased once scaled by max|g|),
 *                  kept iff fl32(fl32(|g_i| * fl32(1/max|g|)) * 65536) > r + 0.5 with r the 16 bits of
 *                  the generator of q8t_quantize for (seed, flat index i);
 *   binarized x  = +1 for x >= 0, -1 otherwise.
 *
 * q8t_ternarize: g: n floats -> t_out: n int8 codes in {-1, 0, +1}; scale_out: 1 device float =
 * max|g| (0 for an all-zero tensor, whose codes are all 0).  ws: q8t_ternarize_workspace_size(n)
 * bytes, 4-byte aligned.  n <= 2^34.
 * q8t_binarize: x: n floats -> codes: n int8 in {-1, +1}.
 * q8t_pack_bits: codes [rows][cols] (+-1, row-major) -> bit rows of uint32 words, bit = 1 for +1.
 *   transpose = 0: out[rows][ceil(cols/32)], bit j of word w = column 32w + j;
 *   transpose = 1: out[cols][ceil(rows/32)], bit j of word w = row 32w + j (a bit row per column).
 *   Bits past the end of a bit row are 0.
 * q8t_xnor_gemm: y[m][n] = sum_k a[m][k] * w[n][k] over +-1 values, from bit rows a_bits
 *   [M][ceil(K/32)] and w_bits [N][ceil(K/32)] (the forward product of a binarized layer:
 *   matches minus mismatches = 2 * popcount(xnor) - K).  y: M*N int32, row-major.
 * q8t_tern_wgrad_multi: Algorithm 1 for a fully connected layer.  g [M][N]: gradient (floats),
 *   a_codes [M][K]: binarized layer input (+-1 int8), S >= 1 samples, sample s drawn with seed + s:
 *     acc[k][n] = sum_{s<S} sum_m a[m][k] * StcTern_s(g)[m][n]      (exact, S*M < 2^31 else
 *     Q8T_ERR_OVERFLOW);   dW[k][n] = (float)((double)acc * (double)max|g| / (double)S).
 *   dw [K][N] floats and acc_out [K][N] int64 are each nullable (not both).  ws:
 *   q8t_tern_wgrad_multi_workspace_size bytes, 4-byte aligned.
 * Errors: Q8T_ERR_SHAPE, Q8T_ERR_NULL, Q8T_ERR_WORKSPACE, Q8T_ERR_OVERFLOW, Q8T_ERR_HIP. */
size_t q8t_ternarize_workspace_size(int64_t n);
int q8t_ternarize(const float *g, int64_t n, uint64_t seed, int8_t *t_out, float *scale_out, void *ws, void *stream);
int q8t_binarize(const float *x, int64_t n, int8_t *codes, void *stream);
int q8t_pack_bits(const int8_t *codes, int rows, int cols, int transpose, uint32_t *out, void *stream);
int q8t_xnor_gemm(const uint32_t *a_bits, const uint32_t *w_bits, int M, int N, int K, int32_t *y, void *stream);
size_t q8t_tern_wgrad_multi_workspace_size(int M, int N, int K);
int q8t_tern_wgrad_multi(const float *g, const int8_t *a_codes, int M, int N, int K, int S, uint64_t seed, float *dw,
                         int64_t *acc_out, void *ws, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Network plumbing around the method (not from the paper; what a ResNet training step needs between
 * the calls above), fused with its neighbours so that the large activation tensors cross HBM once.
 *
 * q8t_range_bn_relu_maxpool_fwd: relu(Range BN(x)) for given statistics (as
 *   q8t_range_bn_relu_fwd_apply) followed by 3x3 / stride 2 / pad 1 max pooling, without writing the
 *   normalized tensor.  x [N,C,H,W]; stats [3][C]; out [N,C,P,Q] floats with P = (H-1)/2 + 1,
 *   Q = (W-1)/2 + 1; idx [N,C,P,Q] bytes: position 3*i + j of the first maximum inside its window
 *   (row-major), 255 where the maximum is not positive (the rectifier passes no gradient there).
 * q8t_maxpool_relu_bwd: gradient with respect to the Range BN output: dy [N,C,H,W] receives, at
 *   every position, the sum of gpool over the windows whose idx names it (0 elsewhere).  Feed it to
 *   q8t_range_bn_bwd / q8t_range_bn_bwd_bifurcate (not the ReLU variants: the mask is in idx).
 * q8t_maxpool_range_bn_bwd_bifurcate: q8t_maxpool_relu_bwd followed by q8t_range_bn_bwd_bifurcate (Section 7's
 *   backward rule, Sections 1 and 4 for the copies) with bit-identical codes, parameters, dgamma and dbeta, but
 *   without the unpooled gradient ever being written: both passes gather it from gpool and idx, one pooled plane at a
 *   time.  x [N,C,H,W]: the Range BN input; gpool, idx [N,C,P,Q]; no dx output; q8_out / qp8_out nullable as above.
 *   Planes of at least 1024 positions with W a multiple of 4, (P*Q) a multiple of 16 and P*Q <= 12288 are served
 *   directly and need x, gpool, idx 16-byte aligned (q8_out 4, q16_out 8), else Q8T_ERR_SHAPE; for every other
 *   shape the unpooled gradient goes through the workspace.  ws:
 *   q8t_maxpool_range_bn_bwd_bifurcate_workspace_size bytes, 16-byte aligned.
 * q8t_relu_bwd_sum_lattice: q8t_relu_bwd_sum where the second gradient is that of a tensor read at every
 *   stride-th row and column only (the input of a 1x1 convolution with that stride and no padding: its layer
 *   gradient is the stride-1 product on the sampled positions and zero elsewhere): g1, out, res [N,C,H,W],
 *   g2s [N,C,ceil(H/stride),ceil(W/stride)]; res = out > 0 ? g1 + t : 0 with t = g2s[h/stride][w/stride] where h
 *   and w are multiples of stride, else 0; bit-identical to the plain call with the zero-filled gradient, which
 *   then never has to be written or read (out nullable: no mask).
 * q8t_add_relu_quantize: out = relu(a + b) (n floats each) and, if q_out != NULL, its 8-bit codes
 *   and parameters exactly as q8t_quantize(out, n, 8, 0, ...) would give them: the first pass leaves
 *   the maximum behind (the minimum of the rectified sum, widened to contain 0, is 0), so only the
 *   second pass of the quantization runs.  ws: q8t_add_relu_quantize_workspace_size(n) bytes,
 *   8-byte aligned.
 * q8t_range_bn_add_relu_quantize: the tail of a residual block in one pass: out = relu(bn(x) + o) with bn the
 *   elementwise stage of Range BN from given statistics (q8t_range_bn_fwd_apply's arithmetic, eq. (range) of
 *   Section 3) and o = other, or bn'(other) from other_stats / other_gamma / other_beta when other_stats != NULL
 *   (a shortcut that is itself convolution + Range BN); 8-bit codes as for q8t_add_relu_quantize.  x, other, out:
 *   [N,C,H,W]; stats, other_stats: [3][C]; gamma / beta pointers nullable.  The normalized tensors are never
 *   written: 12 (+5 for the codes) bytes per element instead of 20 (+5).  ws: q8t_add_relu_quantize_workspace_size.
 * q8t_relu_bwd_add: res = (out > 0 ? g : 0) + other (other nullable: nothing added).
 * q8t_relu_bwd_sum: the gradient that reaches a rectified tensor `out` from its two consumers (a residual
 *   block's convolutions and its shortcut): res = out > 0 ? g1 + g2 : 0 in one pass, instead of a sum and a
 *   masking pass.  out nullable: plain sum; g2 nullable: nothing added.
 * Errors: Q8T_ERR_SHAPE, Q8T_ERR_NULL, Q8T_ERR_WORKSPACE, Q8T_ERR_HIP. */
int q8t_range_bn_relu_maxpool_fwd(const float *x, int N, int C, int H, int W, const float *gamma, const float *beta, float eps,
                                  const float *stats, float *out, uint8_t *idx, void *stream);
int q8t_maxpool_relu_bwd(const float *gpool, const uint8_t *idx, int N, int C, int H, int W, float *dy, void *stream);
size_t q8t_maxpool_range_bn_bwd_bifurcate_workspace_size(int N, int C, int H, int W);
int q8t_maxpool_range_bn_bwd_bifurcate(const float *x, const float *gpool, const uint8_t *idx, const float *stats, int N, int C,
                                       int H, int W, const float *gamma, float eps, float *dgamma, float *dbeta, uint64_t seed8,
                                       uint64_t seed16, int8_t *q8_out, q8t_qparams *qp8_out, int16_t *q16_out,
                                       q8t_qparams *qp16_out, void *ws, void *stream);
size_t q8t_add_relu_quantize_workspace_size(int64_t n);
int q8t_add_relu_quantize(const float *a, const float *b, int64_t n, float *out, int8_t *q_out, q8t_qparams *qp_out, void *ws,
                          void *stream);
int q8t_range_bn_add_relu_quantize(const float *x, const float *stats, const float *gamma, const float *beta,
                                   const float *other, const float *other_stats, const float *other_gamma,
                                   const float *other_beta, int N, int C, int H, int W, float eps, float *out, int8_t *q_out,
                                   q8t_qparams *qp_out, void *ws, void *stream);
int q8t_relu_bwd_add(const float *g, const float *out, const float *other, int64_t n, float *res, void *stream);
int q8t_relu_bwd_sum(const float *g1, const float *g2, const float *out, int64_t n, float *res, void *stream);
int q8t_relu_bwd_sum_lattice(const float *g1, const float *g2s, const float *out, int N, int C, int H, int W, int stride,
                             float *res, void *stream);

/* Measurement aid, not a step of the method: a plain streaming kernel of known traffic with the access
 * shape of the library's HBM-bound calls (every workgroup streams one contiguous slice, four 16-byte
 * accesses in flight per lane).  mode 0: dst = src (bytes read and bytes written); mode 1: src is
 * read only (dst receives checksums, at most 64 KiB: size it >= 64 KiB); mode 2: dst is
 * filled with zeros.  bytes: multiple of 16, >= 65536; src / dst: device, 16-byte aligned, must not
 * overlap.  Errors: Q8T_ERR_SHAPE, Q8T_ERR_NULL, Q8T_ERR_HIP. */
int q8t_probe_stream(int mode, const void *src, void *dst, int64_t bytes, void *stream);

/* Library version string (host pointer, static storage). */
const char *q8t_version(void);

#ifdef __cplusplus
}
#endif
#endif /* Q8T_H */
