"""GPU parity: Range BN forward/backward vs the oracle.

min/max are order-independent and must be bit-equal; the mean and the backward sums are long
float sums (fp64 on both sides, different order), compared within tolerance.  Everything
elementwise is then checked bit for bit by re-running the oracle's elementwise stage on the
GPU's own statistics."""
import numpy as np
import pytest

import oracle
import synth
from gpu_util import same_ints, close, dev, host, require_gpu, same_qparams

pytestmark = pytest.mark.gpu

SHAPES = [(8, 5, 6, 7),      # ragged, scalar path
          (4, 3, 8, 8),      # small planes
          (6, 7, 16, 16),    # vector path
          (3, 2, 40, 36),    # several sweeps per plane, ragged tail inside a plane
          (64, 128, 1, 1),   # FC activations (config 0)
          (2, 1, 1, 1),      # smallest legal n
          (5, 70, 20, 20)]


def _inputs(shape, seed):
    g = synth.rng(seed)
    N, C, H, W = shape
    x = (g.standard_normal(shape) * g.uniform(0.1, 3, (1, C, 1, 1)) + g.uniform(-2, 2, (1, C, 1, 1))).astype(np.float32)
    dy = synth.normal(g, shape, std=1e-2)
    gamma = g.uniform(-2, 2, C).astype(np.float32)
    beta = g.uniform(-1, 1, C).astype(np.float32)
    return x, dy, gamma, beta


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("affine", [False, True])
@pytest.mark.parametrize("eps", [0.0, 1e-5])
def test_forward(shape, affine, eps):
    q8t = require_gpu()
    x, _, gamma, beta = _inputs(shape, 1)
    if not affine:
        gamma = beta = None
    y, stats, q, qp = q8t.range_bn_fwd(dev(x), None if gamma is None else dev(gamma),
                                       None if beta is None else dev(beta), eps, quantized=True)
    oy, ostats, _, _ = oracle.range_bn_fwd(x, gamma, beta, eps)
    st = host(stats)
    assert np.array_equal(st[1:], ostats[1:])          # min, max: exact
    close(st[0], ostats[0])                            # mean: fp64 sums in a different order
    close(host(y), oy)
    # elementwise stage, bit for bit, on the GPU's statistics
    fy, _, fq, fqp = oracle.range_bn_fwd(x, gamma, beta, eps, stats=st, quantized=True)
    same_ints(host(y), fy)
    same_qparams(q8t, qp, fqp)
    same_ints(host(q), fq)


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("affine", [False, True])
def test_backward(shape, affine):
    q8t = require_gpu()
    x, dy, gamma, _ = _inputs(shape, 2)
    if not affine:
        gamma = None
    eps = 1e-5
    ostats = oracle.range_bn_stats(x)
    dx, dgamma, dbeta = q8t.range_bn_bwd(dev(x), dev(dy), dev(ostats), None if gamma is None else dev(gamma), eps)
    odx, odg, odb = oracle.range_bn_bwd(x, dy, ostats, gamma, eps)
    close(host(dgamma), odg)
    close(host(dbeta), odb)
    close(host(dx), odx)


def test_ties_at_the_extrema():
    q8t = require_gpu()
    g = synth.rng(9)
    x = g.standard_normal((4, 2, 8, 8)).astype(np.float32)
    x[0, 0, 0, 0] = x[3, 0, 5, 5] = 9.0
    x[1, 0, 2, 2] = x[2, 0, 7, 1] = -9.0
    x[:, 1] = 1.25  # constant channel: max == min everywhere
    dy = g.standard_normal(x.shape).astype(np.float32)
    stats = oracle.range_bn_stats(x)
    dx, _, _ = q8t.range_bn_bwd(dev(x), dev(dy), dev(stats), None, 1e-3)
    odx, _, _ = oracle.range_bn_bwd(x, dy, stats, None, 1e-3)
    close(host(dx), odx)
    y, st, _, _ = q8t.range_bn_fwd(dev(x), eps=1e-3)
    oy, _, _, _ = oracle.range_bn_fwd(x, eps=1e-3, stats=host(st))
    same_ints(host(y), oy)


def test_config1_full_size():
    # 128x64x56x56, half Gaussian / half Laplace channels, 8-bit per-tensor output, eps 1e-5
    q8t = require_gpu()
    x, dy = synth.range_bn_input(seed=0)
    xd, dyd = dev(x), dev(dy)
    y, stats, q, qp = q8t.range_bn_fwd(xd, eps=1e-5, quantized=True)
    oy, ostats, _, _ = oracle.range_bn_fwd(x, eps=1e-5)
    st = host(stats)
    assert np.array_equal(st[1:], ostats[1:])
    close(st[0], ostats[0])
    close(host(y), oy)
    fy, _, fq, fqp = oracle.range_bn_fwd(x, eps=1e-5, stats=st, quantized=True)
    same_ints(host(y), fy)
    same_qparams(q8t, qp, fqp)
    same_ints(host(q), fq)
    n_unforced = int((host(q) != oracle.range_bn_fwd(x, eps=1e-5, quantized=True)[2]).sum())
    print("int8 codes differing from the un-forced oracle run:", n_unforced, "of", x.size)
    assert n_unforced <= x.size * 1e-5
    dx, dgamma, dbeta = q8t.range_bn_bwd(xd, dyd, stats, None, 1e-5)
    odx, odg, odb = oracle.range_bn_bwd(x, dy, st, None, 1e-5)
    close(host(dbeta), odb)
    close(host(dgamma), odg)
    close(host(dx), odx)
    # int8-only output (no fp32 y written) gives the same codes
    _, _, q2, _ = q8t.range_bn_fwd(xd, eps=1e-5, quantized=True, want_y=False)
    assert np.array_equal(host(q2), host(q))


def test_rejects_degenerate_batch():
    q8t = require_gpu()
    with pytest.raises(q8t.binding.Q8TError) as e:
        q8t.range_bn_fwd(dev(np.ones((1, 3, 1, 1), np.float32)))
    assert e.value.code == -2


@pytest.mark.parametrize("shape", [(6, 7, 16, 16), (3, 2, 40, 36), (128, 64, 56, 56), (5, 9, 7, 7), (64, 128, 1, 1),
                                   (8, 12, 7, 7), (4, 8, 5, 5), (32, 64, 7, 7)])   # the last three: flat groups of four
def test_backward_fused_with_bifurcated_quantization(shape):
    # same results as the two separate calls; the codes are checked against the oracle's quantizer
    # run on the GPU's own dx (bit-exact), dx itself against the oracle within tolerance
    q8t = require_gpu()
    x, dy, gamma, _ = _inputs(shape, 4) if shape[0] < 100 else (*synth.range_bn_input(seed=1), None, None)
    eps = 1e-5
    stats = oracle.range_bn_stats(x)
    xd, dyd, sd = dev(x), dev(dy), dev(stats)
    gd = None if gamma is None else dev(gamma)
    dx, dgamma, dbeta, q8, qp8, q16, qp16 = q8t.range_bn_bwd_bifurcate(xd, dyd, sd, gd, eps, seed8=41, seed16=42)
    dx2, dgamma2, dbeta2 = q8t.range_bn_bwd(xd, dyd, sd, gd, eps)
    r8, rp8, r16, rp16 = q8t.quantize_bifurcate(dx2, seed8=41, seed16=42)
    assert np.array_equal(host(dx), host(dx2))
    assert np.array_equal(host(dgamma), host(dgamma2)) and np.array_equal(host(dbeta), host(dbeta2))
    assert q8t.qparams_to_host(qp8) == q8t.qparams_to_host(rp8)
    assert q8t.qparams_to_host(qp16) == q8t.qparams_to_host(rp16)
    same_ints(host(q8), host(r8))
    same_ints(host(q16), host(r16))
    dxh = host(dx)
    odx, _, _ = oracle.range_bn_bwd(x, dy, stats, gamma, eps)
    close(dxh, odx)
    s8, _, o8 = oracle.quantize(dxh, 8, True, seed=41)
    s16, _, o16 = oracle.quantize(dxh, 16, True, seed=42)
    same_qparams(q8t, qp8, o8)
    same_qparams(q8t, qp16, o16)
    same_ints(host(q8), s8)
    same_ints(host(q16), s16)


@pytest.mark.parametrize("shape", [(6, 7, 16, 16), (5, 9, 7, 7), (16, 64, 56, 56)])
def test_fused_backward_without_the_fp32_result(shape):
    # the codes do not depend on whether dx itself is written
    q8t = require_gpu()
    x, dy, gamma, _ = _inputs(shape, 6)
    stats = oracle.range_bn_stats(x)
    xd, dyd, sd, gd = dev(x), dev(dy), dev(stats), dev(gamma)
    dx, dg, db, q8, qp8, q16, qp16 = q8t.range_bn_bwd_bifurcate(xd, dyd, sd, gd, 1e-5, seed8=7, seed16=8)
    nx, ng, nb, r8, rp8, r16, rp16 = q8t.range_bn_bwd_bifurcate(xd, dyd, sd, gd, 1e-5, seed8=7, seed16=8, want_dx=False)
    assert nx is None
    assert np.array_equal(host(dg), host(ng)) and np.array_equal(host(db), host(nb))
    assert q8t.qparams_to_host(qp8) == q8t.qparams_to_host(rp8) and q8t.qparams_to_host(qp16) == q8t.qparams_to_host(rp16)
    same_ints(host(q8), host(r8))
    same_ints(host(q16), host(r16))


@pytest.mark.parametrize("hw", [(16, 16), (7, 7)])
def test_fused_backward_range_with_ties_and_a_constant_channel(hw):
    # the quantizer's range comes from the extremes of dy per kind of coordinate (ordinary, at the
    # channel maximum, at the minimum, at both): several maxima, several minima, a constant channel
    # (every coordinate is both) and a channel whose extreme dx sits on an extremal coordinate
    q8t = require_gpu()
    g = synth.rng(21)
    N, C, (H, W) = 4, 5, hw
    x = g.standard_normal((N, C, H, W)).astype(np.float32)
    x[:, 0].flat[[3, 77, 150]] = 9.0          # three maxima
    x[:, 1].flat[[5, 6, 190]] = -9.0          # three minima
    x[:, 2] = 1.25                            # constant: max == min everywhere
    dy = (g.standard_normal((N, C, H, W)) * 1e-2).astype(np.float32)
    dy[:, 3] *= 1e-3                          # tiny gradients: the +-kb terms dominate the channel's range
    dy[0, 0].flat[3] = 5.0                    # the largest gradient sits on a maximum
    gamma = np.array([1.5, -0.7, 1.0, 2.0, -1.0], np.float32)
    eps = 1e-5
    stats = oracle.range_bn_stats(x)
    dx, dg, db, q8, qp8, q16, qp16 = q8t.range_bn_bwd_bifurcate(dev(x), dev(dy), dev(stats), dev(gamma), eps, seed8=3, seed16=4)
    dxh = host(dx)
    odx, _, _ = oracle.range_bn_bwd(x, dy, stats, gamma, eps)
    close(dxh, odx)
    s8, _, o8 = oracle.quantize(dxh, 8, True, seed=3)
    s16, _, o16 = oracle.quantize(dxh, 16, True, seed=4)
    same_qparams(q8t, qp8, o8)
    same_qparams(q8t, qp16, o16)
    same_ints(host(q8), s8)
    same_ints(host(q16), s16)
