// Internal (non-exported) interfaces between the translation units of libq8t.
#pragma once
#include <hip/hip_runtime.h>

#include "q8t.h"
#include "relu_sum.h"

// general kernel (igemm_generic.hip).  which: 0 fwd, 1 dgrad, 2 wgrad.  For wgrad the 16-bit
// operand is passed first (a, qa).
int q8t_generic_fc(int which, const void *a, const q8t_qparams *qa, const void *b, const q8t_qparams *qb, int M,
                   int N, int K, float *out_f, void *out_acc, void *ws, hipStream_t st);
size_t q8t_generic_fc_ws(int which, int M, int N, int K);
int q8t_generic_conv(int which, const q8t_conv_desc *d, const void *a, const q8t_qparams *qa, const void *b,
                     const q8t_qparams *qb, float *out_f, void *out_acc, void *ws, hipStream_t st);
size_t q8t_generic_conv_ws(int which, const q8t_conv_desc *d);
int q8t_conv_reduction_check(int which, const q8t_conv_desc *d);

// Per-workgroup statistics of the corrected integer outputs of one output channel, gathered in a
// convolution's epilogue for the Range BN that follows it (Sec. 3; Sec. 4: the normalizer already
// knows the range).  y = scale * acc is monotone in acc, so min / max of y are the images of these.
// Layout of a partial buffer: [channel / 64][nbx workgroups][channel % 64].
struct Q8tConvStat {
    long long sum;
    int mn, mx;
};
// stats[0][k] = mean, [1][k] = min, [2][k] = max over n values per channel, from nact (<= nbx) partials (conv_fast.hip)
int q8t_conv_stats_finalize(const Q8tConvStat *part, int K, int nbx, int nact, double n, const q8t_qparams *qa,
                            const q8t_qparams *qb, float *stats, hipStream_t st);

// specialised convolution kernels (conv_fast.hip)
bool q8t_fast_conv_supported(int which, const q8t_conv_desc *d, const void *a, const void *b, const void *out_f,
                             const void *out_acc);
size_t q8t_fast_conv_ws(int which, const q8t_conv_desc *d);
// bn_stats (nullable, forward only): [3][K] mean / min / max of the float result per output channel
// relu_sum (nullable, layer gradient with a float result): the epilogue stores act > 0 ? result + other : 0
// (relu_sum.h); act and other 16-byte aligned
int q8t_fast_conv(int which, const q8t_conv_desc *d, const void *a, const q8t_qparams *qa, const void *b,
                  const q8t_qparams *qb, float *out_f, void *out_acc, float *bn_stats, void *ws, hipStream_t st,
                  const Q8tReluSum *relu_sum = nullptr, const void *packed = nullptr);
// packed (nullable, both kernels): the filter already in the kernel's layout with its column sums (repack.h); the
// pre-pass is skipped and that part of the workspace stays unused

// 3x3 stride-1 layers with many channels on small planes: 128 x 256 tiles, activations staged once per
// 64-channel chunk, weights streamed (conv_wide.hip).  Same contract as q8t_fast_conv.
bool q8t_wide_conv_supported(int which, const q8t_conv_desc *d, const void *a, const void *out_f, const void *out_acc);
size_t q8t_wide_conv_ws(int which, const q8t_conv_desc *d);
int q8t_wide_conv(int which, const q8t_conv_desc *d, const void *a, const q8t_qparams *qa, const void *b,
                  const q8t_qparams *qb, float *out_f, void *out_acc, float *bn_stats, void *ws, hipStream_t st,
                  const void *packed = nullptr);
// Q8T_PACK_* layout the wide-tile kernel takes for this product, by shape alone (Q8T_PACK_NONE: not its shape)
int q8t_wide_conv_pack_layout(int which, const q8t_conv_desc *d);

// Range BN statistics of an NCHW tensor alone (range_bn.hip); ws as for q8t_range_bn_fwd
int q8t_range_bn_stats(const float *x, int N, int C, int H, int W, float *stats_out, void *ws, hipStream_t st);

// general MFMA path over a channel-contiguous copy of the operand (conv_nhwc.hip): forward and
// layer gradient, channel counts that are multiples of 64
bool q8t_nhwc_conv_supported(int which, const q8t_conv_desc *d);
size_t q8t_nhwc_conv_ws(int which, const q8t_conv_desc *d);
// bn_stats (nullable, forward only): [3][K] mean / min / max of the float result, gathered in the epilogue
// through stats_ws (q8t_nhwc_conv_stats_ws bytes, 16-byte aligned)
int q8t_nhwc_conv(int which, const q8t_conv_desc *d, const void *a, const q8t_qparams *qa, const void *b,
                  const q8t_qparams *qb, float *out_f, void *out_acc, float *bn_stats, void *stats_ws, void *ws,
                  hipStream_t st);
size_t q8t_nhwc_conv_stats_ws(const q8t_conv_desc *d);

// forward with fewer than 64 input channels (first layer): explicit im2col rows + the same GEMM
bool q8t_smallc_conv_supported(int which, const q8t_conv_desc *d);
size_t q8t_smallc_conv_ws(int which, const q8t_conv_desc *d);
// bn_stats as for q8t_nhwc_conv; only where q8t_smallc_conv_stats_ws(d) != 0 (one block of 64 output channels, fused kernel)
int q8t_smallc_conv(const q8t_conv_desc *d, const void *a, const q8t_qparams *qa, const void *b, const q8t_qparams *qb,
                    float *out_f, void *out_acc, float *bn_stats, void *stats_ws, void *ws, hipStream_t st);
size_t q8t_smallc_conv_stats_ws(const q8t_conv_desc *d);

// forward with very few input channels and 64 output channels, filter rows of at most 8 taps: operand fragments read
// straight from a staged band of input rows, filter in registers (conv_first.hip).  Contract of q8t_smallc_conv.
bool q8t_first_conv_supported(const q8t_conv_desc *d, const void *a, const void *out_f, const void *out_acc);
size_t q8t_first_conv_ws(const q8t_conv_desc *d);
size_t q8t_first_conv_stats_ws(const q8t_conv_desc *d);
int q8t_first_conv(const q8t_conv_desc *d, const void *a, const q8t_qparams *qa, const void *b, const q8t_qparams *qb,
                   float *out_f, void *out_acc, float *bn_stats, void *stats_ws, void *ws, hipStream_t st);

// specialised 3x3 weight-gradient kernel (wgrad_fast.hip)
bool q8t_fast_wgrad_supported(const q8t_conv_desc *d, const void *g16, const void *x, const void *dw,
                              const void *acc);
size_t q8t_fast_wgrad_ws(const q8t_conv_desc *d);
int q8t_fast_wgrad(const q8t_conv_desc *d, const int16_t *g16, const q8t_qparams *qg, const int8_t *x,
                   const q8t_qparams *qx, float *dw, int64_t *acc_out, void *ws, hipStream_t st);

// general weight-gradient path: byte planes of the gradient x im2col rows of the input as one
// int8 MFMA GEMM with the reduction split into overflow-free slices (wgrad_gemm.hip)
bool q8t_gemm_wgrad_supported(const q8t_conv_desc *d);
size_t q8t_gemm_wgrad_ws(const q8t_conv_desc *d);
int q8t_gemm_wgrad(const q8t_conv_desc *d, const int16_t *g16, const q8t_qparams *qg, const int8_t *x,
                   const q8t_qparams *qx, float *dw, int64_t *acc_out, void *ws, hipStream_t st);


// weight gradient of 3x3 convolutions with 14x14 or 7x7 result planes, stride 1 or 2: padded planes in
// LDS, no operand rewritten in HBM (wgrad_planes.hip)
bool q8t_planes_wgrad_supported(const q8t_conv_desc *d, const void *g16, const void *x, const void *dw,
                                const void *acc);
size_t q8t_planes_wgrad_ws(const q8t_conv_desc *d);
int q8t_planes_wgrad(const q8t_conv_desc *d, const int16_t *g16, const q8t_qparams *qg, const int8_t *x,
                     const q8t_qparams *qx, float *dw, int64_t *acc_out, void *ws, hipStream_t st);

// glue.hip: out [N,C,P,Q] = x[.., p*s, q*s] of 8-bit codes, P = (H-1)/s + 1, Q = (W-1)/s + 1 (the operand of a 1x1
// convolution with stride s and no padding, which is the stride-1 layer on these positions)
int q8t_subsample_codes(const int8_t *x, int N, int C, int H, int W, int s, int8_t *out, hipStream_t st);

// quantize.hip: nearest 8-bit quantization of x with the range given as npairs (<= 1024) float2 (min, max) pairs
int q8t_quantize8_from_partials(const float *x, int64_t n, const void *minmax_pairs, int npairs, int8_t *q_out,
                                q8t_qparams *qp_out, hipStream_t st);
