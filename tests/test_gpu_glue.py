"""GPU parity of the network plumbing (stem pooling fused with Range BN + ReLU, residual add + ReLU with
the quantization of its result, ReLU backward) against the oracle."""
import numpy as np
import pytest

import oracle
import synth
from gpu_util import close, dev, host, require_gpu, same_ints, same_qparams

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("shape", [(2, 3, 8, 8), (1, 2, 7, 9), (3, 64, 112, 112), (2, 5, 33, 20), (1, 1, 1, 2), (2, 4, 16, 24)])
def test_stem_pooling_forward_and_backward(shape):
    q8t = require_gpu()
    g = synth.rng(sum(shape))
    x = synth.normal(g, shape, std=1.0)
    C = shape[1]
    gamma = synth.normal(g, (C,), std=1.0)
    beta = synth.normal(g, (C,), std=0.3)
    stats = oracle.range_bn_stats(x)
    out, idx = q8t.range_bn_relu_maxpool_fwd(dev(x), dev(stats), dev(gamma), dev(beta), 1e-5)
    oout, oidx = oracle.range_bn_relu_maxpool_fwd(x, stats, gamma, beta, 1e-5)
    same_ints(host(out), oout)          # a maximum of bit-identical values
    same_ints(host(idx), oidx)
    gp = synth.normal(g, oout.shape, std=1e-2)
    dy = q8t.maxpool_relu_bwd(dev(gp), idx, shape[2], shape[3])
    ody = oracle.maxpool_relu_bwd(gp, oidx, shape[2], shape[3])
    close(host(dy), ody)                # up to four float terms per position, added in the same order
    same_ints(host(dy) == 0, ody == 0)


@pytest.mark.parametrize("n", [1, 7, 4099, 1 << 20, (1 << 22) + 5])
def test_add_relu_with_quantization_matches_the_separate_steps(n):
    q8t = require_gpu()
    g = synth.rng(n)
    a, b = synth.normal(g, (n,), std=1.0), synth.normal(g, (n,), std=0.5)
    out, q, qp = q8t.add_relu_quantize(dev(a), dev(b))
    oout, omax = oracle.add_relu(a, b)
    same_ints(host(out), oout)
    sq, _, oqp = oracle.quantize(oout, 8)        # the plain two-pass quantization of the result
    same_qparams(q8t, qp, oqp)
    same_ints(host(q), sq)
    out2, q2, _ = q8t.add_relu_quantize(dev(a), dev(b), quantized=False)
    assert q2 is None and np.array_equal(host(out2), oout)
    # nothing positive: range [0, 0]
    out3, q3, qp3 = q8t.add_relu_quantize(dev(-np.abs(a)), dev(-np.abs(b)))
    sq3, _, oqp3 = oracle.quantize(np.zeros(n, np.float32), 8)
    same_qparams(q8t, qp3, oqp3)
    same_ints(host(q3), sq3)


@pytest.mark.parametrize("n", [1, 6, 4099, (1 << 21) + 3])
def test_relu_backward_with_and_without_the_other_branch(n):
    q8t = require_gpu()
    g = synth.rng(n + 1)
    gr, out, other = synth.normal(g, (n,), std=1.0), np.maximum(synth.normal(g, (n,), std=1.0), 0), synth.normal(g, (n,), std=1.0)
    same_ints(host(q8t.relu_bwd_add(dev(gr), dev(out))), oracle.relu_bwd_add(gr, out))
    same_ints(host(q8t.relu_bwd_add(dev(gr), dev(out), dev(other))), oracle.relu_bwd_add(gr, out, other))
    # the sum of two consumers' gradients, masked in the same pass
    same_ints(host(q8t.relu_bwd_sum(dev(gr), dev(other), dev(out))), oracle.relu_bwd_sum(gr, other, out))
    same_ints(host(q8t.relu_bwd_sum(dev(gr), dev(other))), oracle.relu_bwd_sum(gr, other))
    same_ints(host(q8t.relu_bwd_sum(dev(gr), None, dev(out))), oracle.relu_bwd_sum(gr, None, out))


@pytest.mark.parametrize("shape", [(2, 3, 8, 8), (3, 5, 7, 7), (4, 64, 14, 14), (2, 6, 5, 6), (16, 64, 56, 56)])
def test_block_tail_range_bn_add_relu_quantize(shape):
    # relu(bn(x) + o) and its 8-bit codes in one call, the shortcut plain or normalized by its own statistics
    q8t = require_gpu()
    g = synth.rng(sum(shape) + 3)
    x, o = synth.normal(g, shape, std=1.0), synth.normal(g, shape, std=1.0)
    C = shape[1]
    gamma, beta = g.uniform(-1.5, 1.5, C).astype(np.float32), g.uniform(-0.5, 0.5, C).astype(np.float32)
    og, ob = g.uniform(0.5, 1.5, C).astype(np.float32), g.uniform(-0.5, 0.5, C).astype(np.float32)
    eps = 1e-5
    st, so = oracle.range_bn_stats(x), oracle.range_bn_stats(o)
    out, q, qp = q8t.range_bn_add_relu_quantize(dev(x), dev(st), dev(o), dev(gamma), dev(beta), eps=eps)
    oout, _ = oracle.range_bn_add_relu(x, st, o, gamma, beta, eps=eps)
    same_ints(host(out), oout)
    sq, _, oqp = oracle.quantize(oout, 8)
    same_qparams(q8t, qp, oqp)
    same_ints(host(q), sq)
    out2, q2, qp2 = q8t.range_bn_add_relu_quantize(dev(x), dev(st), dev(o), None, None, dev(so), dev(og), dev(ob), eps)
    oout2, _ = oracle.range_bn_add_relu(x, st, o, None, None, so, og, ob, eps)
    same_ints(host(out2), oout2)
    sq2, _, oqp2 = oracle.quantize(oout2, 8)
    same_qparams(q8t, qp2, oqp2)
    same_ints(host(q2), sq2)
    out3, q3, _ = q8t.range_bn_add_relu_quantize(dev(x), dev(st), dev(o), dev(gamma), dev(beta), eps=eps, quantized=False)
    assert q3 is None and np.array_equal(host(out3), oout)


@pytest.mark.parametrize("shape", [(2, 3, 32, 32), (3, 64, 112, 112), (2, 4, 36, 32), (5, 2, 64, 48),   # gathered in both passes
                                   (2, 3, 8, 8), (1, 2, 7, 9), (2, 5, 33, 20)])                           # through the workspace
@pytest.mark.parametrize("want_q8", [True, False])
def test_stem_backward_from_the_pooled_gradient(shape, want_q8):
    # pooling backward + Range BN backward + bifurcated quantization in one call: bit-identical to the separate calls
    # (which have their own parity tests), and the decoded 16-bit copy within one level of the oracle's dx
    q8t = require_gpu()
    g = synth.rng(sum(shape) + 1)
    N, C, H, W = shape
    x = synth.normal(g, shape, std=1.0)
    x[:, 0].flat[[3, 17, (N - 1) * H * W + 5]] = 9.0        # several maxima: listed and patched after pass 2
    if C > 2:
        x[:, 2] = 0.75                            # a constant channel: every coordinate is extremal (crowded)
    gamma = synth.normal(g, (C,), std=1.0)
    beta = synth.normal(g, (C,), std=0.3)
    stats = oracle.range_bn_stats(x)
    xd, sd, gd = dev(x), dev(stats), dev(gamma)
    _, idx = q8t.range_bn_relu_maxpool_fwd(xd, sd, gd, dev(beta), 1e-5)
    gp = synth.normal(g, tuple(idx.shape), std=1e-2)
    gpd = dev(gp)
    dg, db, q8, qp8, q16, qp16 = q8t.maxpool_range_bn_bwd_bifurcate(xd, gpd, idx, sd, gd, 1e-5, seed8=5, seed16=6, want_q8=want_q8)
    dy = q8t.maxpool_relu_bwd(gpd, idx, H, W)
    _, rg, rb, r8, rp8, r16, rp16 = q8t.range_bn_bwd_bifurcate(xd, dy, sd, gd, 1e-5, seed8=5, seed16=6, want_dx=False)
    assert np.array_equal(host(dg), host(rg)) and np.array_equal(host(db), host(rb))
    assert q8t.qparams_to_host(qp16) == q8t.qparams_to_host(rp16)
    same_ints(host(q16), host(r16))
    if want_q8:
        assert q8t.qparams_to_host(qp8) == q8t.qparams_to_host(rp8)
        same_ints(host(q8), host(r8))
    else:
        assert q8 is None and qp8 is None
    ody = oracle.maxpool_relu_bwd(gp, host(idx), H, W)
    odx, odg, odb = oracle.range_bn_bwd(x, ody, stats, gamma, 1e-5)
    close(host(dg), odg)
    close(host(db), odb)
    _, _, scale, _, zero_point, bits = q8t.qparams_to_host(qp16)
    assert bits == 16
    dec = (host(q16).astype(np.float64) + 32768 - zero_point) * scale
    assert np.max(np.abs(dec - odx)) <= 1.001 * scale + 1e-5 * np.max(np.abs(odx))


@pytest.mark.parametrize("shape,stride", [((2, 3, 8, 12), 2), ((3, 64, 56, 56), 2), ((5, 16, 28, 28), 2), ((2, 4, 14, 14), 2),
                                          ((1, 2, 7, 9), 2), ((2, 2, 9, 10), 3), ((1, 1, 4, 4), 1)])
@pytest.mark.parametrize("masked", [True, False])
def test_sum_with_a_gradient_on_the_lattice_of_a_strided_1x1_layer(shape, stride, masked):
    q8t = require_gpu()
    g = synth.rng(sum(shape) + stride)
    N, C, H, W = shape
    g1 = synth.normal(g, shape, std=1.0)
    g1[0, 0, 0, :2] = -0.0                      # x + 0 is not x for x = -0: the addition happens everywhere
    g2s = synth.normal(g, (N, C, (H + stride - 1) // stride, (W + stride - 1) // stride), std=1.0)
    out = np.maximum(synth.normal(g, shape, std=1.0), 0).astype(np.float32) if masked else None
    od = None if out is None else dev(out)
    res = q8t.relu_bwd_sum_lattice(dev(g1), dev(g2s), od, stride)
    exp = oracle.relu_bwd_sum_lattice(g1, g2s, out, stride)
    same_ints(host(res).view(np.int32), exp.view(np.int32))
    full = np.zeros(shape, np.float32)
    full[:, :, ::stride, ::stride] = g2s
    plain = q8t.relu_bwd_sum(dev(g1), dev(full), od)
    assert np.array_equal(host(res).view(np.int32), host(plain).view(np.int32))
