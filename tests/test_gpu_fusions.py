"""GPU parity of the fused calls: convolution forward that also returns the Range BN statistics
of its result, and Range BN forward from given statistics (normalization pass only)."""
import numpy as np
import pytest

import oracle
import synth
from gpu_util import close, dev, host, qp_dev_from, require_gpu, same_ints, same_qparams

pytestmark = pytest.mark.gpu

CASES = [
    (3, 64, 56, 56, 64, 3, 3, 1, 1),     # specialised kernel, statistics from its epilogue
    (2, 64, 14, 14, 64, 3, 3, 1, 1),
    (9, 64, 14, 14, 128, 3, 3, 1, 1),    # two output-channel chunks
    (2, 256, 10, 10, 64, 1, 1, 1, 0),
    (40, 64, 6, 6, 64, 3, 3, 1, 1),      # more workgroups than rows to give them: inactive ones must not count
    (3, 256, 14, 14, 256, 3, 3, 1, 1),   # wide-tile kernel: statistics per 32x32 tile column, ragged last tile
    (5, 256, 7, 7, 512, 3, 3, 1, 1),     # ... unaligned planes, two column tiles
    (2, 64, 16, 16, 128, 3, 3, 2, 1),    # strided: statistics from the epilogue of the implicit-GEMM kernel
    (5, 64, 28, 28, 128, 3, 3, 2, 1),    # ragged last row tile
    (3, 128, 14, 14, 256, 3, 3, 2, 1),   # 256-channel tiles
    (7, 64, 28, 28, 128, 1, 1, 2, 0),    # 1x1 projection at stride 2 (runs as the stride-1 layer on the gathered positions)
    (3, 128, 56, 56, 64, 1, 1, 2, 0),    # ... on large planes
    (5, 64, 14, 14, 128, 1, 1, 2, 0),    # ... 7x7 result planes: the general strided path
    (11, 256, 7, 7, 512, 3, 3, 1, 1),    # 7x7 planes
    (3, 128, 15, 13, 64, 3, 3, 1, 1),    # odd plane at stride 1
    (6, 3, 64, 64, 64, 7, 7, 2, 3),      # first layer: statistics from the fused small-channel kernel
    (3, 3, 45, 52, 64, 7, 7, 2, 3),      # ... ragged rows per workgroup
    (2, 3, 224, 224, 64, 7, 7, 2, 3),    # ... at its real plane size
    (2, 3, 7, 6, 4, 3, 3, 1, 1),         # other shapes: product, then the statistics pass
    (2, 3, 32, 32, 32, 7, 7, 2, 3),
]


def _rand_q(g, shape, bits=8):
    half = 2 ** (bits - 1)
    lv = g.integers(0, 2 ** bits, size=shape)
    qp = oracle.QParams(0.0, 0.0, float(np.float32(g.uniform(0.01, 0.1))), 1.0, int(g.integers(0, 2 ** bits)), bits)
    return (lv - half).astype(np.int8), qp


@pytest.mark.parametrize("case", CASES)
def test_conv_forward_with_range_bn_statistics(case):
    q8t = require_gpu()
    g = synth.rng(1000 + sum(case))
    N, C, H, W, K, R, S, st, pad = case
    sx, px = _rand_q(g, (N, C, H, W))
    sw, pw = _rand_q(g, (K, C, R, S))
    d, od = q8t.conv_desc(*case), oracle.conv_desc(*case)
    y, acc, stats = q8t.qconv_fwd_bn_stats(d, dev(sx), qp_dev_from(px), dev(sw), qp_dev_from(pw), want_acc=True)
    oy, oacc = oracle.qconv_fwd(od, sx, px, sw, pw)
    same_ints(host(acc), oacc)
    close(host(y), oy)
    ost = oracle.range_bn_stats(oy)
    sth = host(stats)
    assert np.array_equal(sth[1:], ost[1:])      # min / max: exact
    close(sth[0], ost[0])                        # mean: fp64 sum in another order


def test_conv_statistics_at_full_size_feed_the_normalization():
    # config-2 layer at batch 128: conv with statistics -> normalization from those statistics,
    # float and 8-bit outputs, against the oracle run on the GPU's own conv result and statistics
    q8t = require_gpu()
    case = (128, 64, 56, 56, 64, 3, 3, 1, 1)
    x, w, _ = synth.conv_layer(seed=11, N=128)
    qx, px = q8t.quantize(dev(x), 8)
    qw, pw = q8t.quantize(dev(w), 8)
    d = q8t.conv_desc(*case)
    y, _, stats = q8t.qconv_fwd_bn_stats(d, qx, px, qw, pw)
    yh, sth = host(y), host(stats)
    ost = oracle.range_bn_stats(yh)
    assert np.array_equal(sth[1:], ost[1:])
    close(sth[0], ost[0])
    bn, q, qp = q8t.range_bn_fwd_apply(y, stats, eps=1e-5, quantized=True)
    obn, _, oq, oqp = oracle.range_bn_fwd(yh, eps=1e-5, stats=sth, quantized=True)
    same_ints(host(bn), obn)
    same_qparams(q8t, qp, oqp)
    same_ints(host(q), oq)


@pytest.mark.parametrize("shape", [(6, 7, 16, 16), (3, 2, 40, 36), (4, 5, 3, 3), (64, 128, 1, 1)])
def test_range_bn_forward_from_given_statistics(shape):
    q8t = require_gpu()
    x, _ = synth.range_bn_input(sum(shape), *shape)
    g = synth.rng(7)
    gamma = g.uniform(-1.5, 1.5, size=shape[1]).astype(np.float32)
    beta = g.uniform(-0.5, 0.5, size=shape[1]).astype(np.float32)
    _, stats, _, _ = q8t.range_bn_fwd(dev(x), dev(gamma), dev(beta), 1e-5)
    sth = host(stats)
    y, q, qp = q8t.range_bn_fwd_apply(dev(x), stats, dev(gamma), dev(beta), 1e-5, quantized=True)
    oy, _, oq, oqp = oracle.range_bn_fwd(x, gamma, beta, 1e-5, stats=sth, quantized=True)
    same_ints(host(y), oy)
    same_qparams(q8t, qp, oqp)
    same_ints(host(q), oq)


RELU_SHAPES = [(6, 7, 16, 16), (3, 2, 40, 36), (4, 5, 3, 3), (64, 128, 1, 1), (5, 9, 7, 7), (8, 5, 6, 7)]


@pytest.mark.parametrize("shape", RELU_SHAPES)
@pytest.mark.parametrize("affine", [False, True])
def test_range_bn_relu_forward(shape, affine):
    # normalization + ReLU + 8-bit output in one pass: everything elementwise, so bit for bit
    q8t = require_gpu()
    x, _ = synth.range_bn_input(sum(shape), *shape)
    g = synth.rng(8)
    gamma = g.uniform(-1.5, 1.5, size=shape[1]).astype(np.float32) if affine else None
    beta = g.uniform(-0.5, 0.5, size=shape[1]).astype(np.float32) if affine else None
    stats = oracle.range_bn_stats(x)
    gd = None if gamma is None else dev(gamma)
    bd = None if beta is None else dev(beta)
    y, q, qp = q8t.range_bn_relu_fwd_apply(dev(x), dev(stats), gd, bd, 1e-5, quantized=True)
    oy, oq, oqp = oracle.range_bn_relu_fwd(x, stats, gamma, beta, 1e-5, quantized=True)
    same_ints(host(y), oy)
    same_qparams(q8t, qp, oqp)
    same_ints(host(q), oq)
    # codes alone (no fp32 output): the form the next layer consumes
    _, q2, qp2 = q8t.range_bn_relu_fwd_apply(dev(x), dev(stats), gd, bd, 1e-5, quantized=True, want_y=False)
    same_ints(host(q2), oq)
    same_qparams(q8t, qp2, oqp)


@pytest.mark.parametrize("shape", RELU_SHAPES + [(16, 64, 56, 56), (8, 12, 7, 7)])
def test_range_bn_relu_backward_with_bifurcated_quantization(shape):
    q8t = require_gpu()
    x, dy = synth.range_bn_input(3 + sum(shape), *shape)
    g = synth.rng(9)
    gamma = g.uniform(-1.5, 1.5, size=shape[1]).astype(np.float32)
    beta = g.uniform(-0.5, 0.5, size=shape[1]).astype(np.float32)
    eps = 1e-5
    stats = oracle.range_bn_stats(x)
    dx, dgamma, dbeta, q8, qp8, q16, qp16 = q8t.range_bn_relu_bwd_bifurcate(dev(x), dev(dy), dev(stats), dev(gamma),
                                                                            dev(beta), eps, seed8=51, seed16=52)
    odx, odg, odb = oracle.range_bn_relu_bwd(x, dy, stats, gamma, beta, eps)
    close(host(dgamma), odg)
    close(host(dbeta), odb)
    dxh = host(dx)
    close(dxh, odx)
    # the same as masking first and calling the plain fused backward (bit for bit)
    masked = oracle.range_bn_relu_mask(x, dy, stats, gamma, beta, eps)
    dx2, dg2, db2, r8, rp8, r16, rp16 = q8t.range_bn_bwd_bifurcate(dev(x), dev(masked), dev(stats), dev(gamma), eps,
                                                                   seed8=51, seed16=52)
    assert np.array_equal(dxh, host(dx2))
    assert np.array_equal(host(dgamma), host(dg2)) and np.array_equal(host(dbeta), host(db2))
    same_ints(host(q8), host(r8))
    same_ints(host(q16), host(r16))
    # codes against the oracle's quantizer on the GPU's own dx
    s8, _, o8 = oracle.quantize(dxh, 8, True, seed=51)
    s16, _, o16 = oracle.quantize(dxh, 16, True, seed=52)
    same_qparams(q8t, qp8, o8)
    same_qparams(q8t, qp16, o16)
    same_ints(host(q8), s8)
    same_ints(host(q16), s16)


@pytest.mark.parametrize("case", [
    (3, 64, 56, 56, 64, 3, 3, 1, 1),     # 3x3 stride 1 on 56x56 planes: the register-tile kernel's epilogue
    (3, 128, 28, 28, 128, 3, 3, 1, 1),   # ... 28x28
    (5, 256, 14, 14, 256, 3, 3, 1, 1),   # wide-tile kernel, aligned planes
    (6, 512, 7, 7, 512, 3, 3, 1, 1),     # ... 7x7 planes: the transposed write-out
    (3, 64, 28, 28, 128, 3, 3, 2, 1),    # stride 2: the two column classes of a row written as pairs
    (2, 128, 14, 14, 256, 3, 3, 2, 1),
    (2, 64, 15, 13, 64, 3, 3, 1, 1),     # odd plane: scalar stores
    (2, 64, 14, 14, 128, 1, 1, 2, 0),    # shapes without the step in an epilogue: product, then the plumbing pass
    (2, 24, 9, 9, 40, 3, 3, 1, 1),
])
@pytest.mark.parametrize("with_other", [True, False])
def test_layer_gradient_with_the_end_of_the_block_in_its_epilogue(case, with_other):
    # dx = act > 0 ? dgrad + other : 0 in one call: bit-identical to the two separate calls, and both against the oracle
    q8t = require_gpu()
    g = synth.rng(sum(case) + 3)
    N, C, H, W, K, R, S, st, pad = case
    od = oracle.conv_desc(*case)
    sg, pg = _rand_q(g, (N, K, od.P, od.Q))
    sw, pw = _rand_q(g, (K, C, R, S))
    other = synth.normal(g, (N, C, H, W), std=3.0) if with_other else None
    act = synth.normal(g, (N, C, H, W), std=1.0)
    act[act < 0.3] = 0.0                       # a rectified tensor: many exact zeros
    d = q8t.conv_desc(*case)
    dpg, dpw = qp_dev_from(pg), qp_dev_from(pw)
    od_dev = None if other is None else dev(other)
    dx = q8t.qconv_dgrad_relu_sum(d, dev(sg), dpg, dev(sw), dpw, od_dev, dev(act))
    plain, _ = q8t.qconv_dgrad(d, dev(sg), dpg, dev(sw), dpw)
    ref = q8t.relu_bwd_sum(plain, od_dev, dev(act))
    assert np.array_equal(host(dx), host(ref))
    odx, _ = oracle.qconv_dgrad(od, sg, pg, sw, pw)
    ores = oracle.relu_bwd_sum(odx, other, act)
    close(host(dx), ores)
    same_ints(host(dx) == 0, ores == 0)


PACK_CASES = [
    (3, 256, 14, 14, 256, 3, 3, 1, 1),   # wide tiles, 256 columns, both products
    (5, 256, 7, 7, 512, 3, 3, 1, 1),     # ... forward 512 -> two column tiles; layer gradient 256 columns
    (7, 128, 7, 7, 128, 3, 3, 1, 1),     # wide tiles, 128 columns
    (2, 64, 56, 56, 64, 3, 3, 1, 1),     # 64-column register tiles
    (2, 64, 28, 28, 128, 1, 1, 1, 0),    # ... 1x1
    (3, 64, 28, 28, 128, 1, 1, 2, 0),    # 1x1 at stride 2: forward on the gathered positions; layer gradient packs nothing
    (2, 64, 16, 16, 128, 3, 3, 2, 1),    # strided 3x3: nothing to pack ahead
    (2, 3, 32, 32, 64, 7, 7, 2, 3),      # first layer: nothing to pack ahead
]


def test_products_with_filters_packed_ahead():
    # every filter packed by ONE launch, then handed to the products: bit-identical to the calls that pack on their own
    q8t = require_gpu()
    g = synth.rng(77)
    layers, jobs = [], []
    for case in PACK_CASES:
        N, C, H, W, K, R, S, st, pad = case
        d = q8t.conv_desc(*case)
        sx, px = _rand_q(g, (N, C, H, W))
        sw, pw = _rand_q(g, (K, C, R, S))
        sg, pg = _rand_q(g, (N, K, d.P, d.Q))
        ops = dict(d=d, qx=dev(sx), px=qp_dev_from(px), qw=dev(sw), pw=qp_dev_from(pw), qg=dev(sg), pg=qp_dev_from(pg),
                   other=dev(synth.normal(g, (N, C, H, W), std=1.0)),
                   act=dev(np.maximum(synth.normal(g, (N, C, H, W), std=1.0), 0).astype(np.float32)))
        layers.append(ops)
        jobs.append((d, 0, ops["qw"]))
        jobs.append((d, 1, ops["qw"]))
    packed = q8t.qconv_pack_multi(jobs)
    sizes = [q8t.qconv_pack_size(j[0], j[1]) for j in jobs]
    assert [b is None for b in packed] == [s == 0 for s in sizes]
    assert sizes[0] > 0 and sizes[1] > 0 and sizes[6] > 0 and sizes[10] > 0     # wide, register tile, gathered 1x1
    assert sizes[11] == 0 and sizes[12] == 0 and sizes[13] == 0 and sizes[14] == 0 and sizes[15] == 0
    for i, o in enumerate(layers):
        pf, pd = packed[2 * i], packed[2 * i + 1]
        y0, a0, s0 = q8t.qconv_fwd_bn_stats(o["d"], o["qx"], o["px"], o["qw"], o["pw"], want_acc=True)
        y1, a1, s1 = q8t.qconv_fwd_bn_stats(o["d"], o["qx"], o["px"], o["qw"], o["pw"], want_acc=True, packed=pf)
        assert np.array_equal(host(a0), host(a1)) and np.array_equal(host(y0), host(y1)) and np.array_equal(host(s0), host(s1))
        dx0, c0 = q8t.qconv_dgrad(o["d"], o["qg"], o["pg"], o["qw"], o["pw"], want_acc=True)
        dx1, c1 = q8t.qconv_dgrad(o["d"], o["qg"], o["pg"], o["qw"], o["pw"], want_acc=True, packed=pd)
        assert np.array_equal(host(c0), host(c1)) and np.array_equal(host(dx0), host(dx1))
        r0 = q8t.qconv_dgrad_relu_sum(o["d"], o["qg"], o["pg"], o["qw"], o["pw"], o["other"], o["act"])
        r1 = q8t.qconv_dgrad_relu_sum(o["d"], o["qg"], o["pg"], o["qw"], o["pw"], o["other"], o["act"], packed=pd)
        assert np.array_equal(host(r0).view(np.int32), host(r1).view(np.int32))
