"""GPU parity: angle diagnostic (Sec. 5.1 eq. 1) and chunk-averaged clamping range (App. B)."""
import numpy as np
import pytest

import oracle
import synth
from gpu_util import dev, host, require_gpu, same_ints, same_qparams

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n,bits,stoch", [(1, 8, False), (1000, 8, False), (70001, 8, True), (1 << 20, 4, False),
                                          (300000, 16, True), (4097, 12, True)])
def test_angle_matches_oracle(n, bits, stoch):
    q8t = require_gpu()
    x = synth.normal(synth.rng(n + bits), (n,), std=0.7)
    q, qp = q8t.quantize(dev(x), bits, stoch, 5)
    out = host(q8t.quant_angle(dev(x), q, qp))
    stored, _, oqp = oracle.quantize(x, bits, stoch, seed=5)
    same_ints(host(q), stored)
    exp = oracle.quant_angle(x, stored, oqp)
    # fp64 sums of n terms taken in another order: each side is within n * 2^-53 (relative to the sum
    # of the magnitudes) of the exact value
    tol = 4.0 * n * 2.0 ** -53
    mags = (float(np.abs(x.astype(np.float64) * oracle.dequantize(stored, oqp)).sum()), exp[1], exp[2])
    for got, want, mag in zip(out[:3], exp[:3], mags):
        assert abs(got - want) <= tol * mag + 1e-300
    assert abs(out[3] - exp[3]) <= 3 * tol + 1e-15


def test_angle_of_config1_shaped_activation_and_gradient():
    # forward tensors keep their direction better than stochastic 8-bit gradients (Sec. 3 / Sec. 4)
    q8t = require_gpu()
    x, dy = synth.range_bn_input(seed=2, N=8)
    qx, px = q8t.quantize(dev(x), 8)
    g8, pg8, g16, pg16 = q8t.quantize_bifurcate(dev(dy), 3, 4)
    cx = host(q8t.quant_angle(dev(x), qx, px))[3]
    c8 = host(q8t.quant_angle(dev(dy), g8, pg8))[3]
    c16 = host(q8t.quant_angle(dev(dy), g16, pg16))[3]
    sx, _, opx = oracle.quantize(x, 8)
    s8, _, o8 = oracle.quantize(dy, 8, True, seed=3)
    s16, _, o16 = oracle.quantize(dy, 16, True, seed=4)
    tol = 12.0 * x.size * 2.0 ** -53
    assert abs(cx - oracle.quant_angle(x, sx, opx)[3]) < tol
    assert abs(c8 - oracle.quant_angle(dy, s8, o8)[3]) < tol
    assert abs(c16 - oracle.quant_angle(dy, s16, o16)[3]) < tol
    assert c8 < c16 <= 1.0


@pytest.mark.parametrize("n,K", [(12, 4), (10, 4), (9, 4), (1000, 1), (128 * 3000, 128), (1 << 20, 3), (5000, 5000),
                                 (64 * 56 * 56 * 16, 16)])
def test_chunk_range_matches_oracle(n, K):
    q8t = require_gpu()
    g = synth.rng(n + K)
    x = np.abs(g.standard_cauchy(size=n)).astype(np.float32) if n > 100 else synth.normal(g, (n,), std=3.0)
    got = host(q8t.chunk_range(dev(x), K))
    vmin, vmax = oracle.chunk_range(x, K)
    assert got[0] == vmin and got[1] == vmax      # bit-exact: the range decides integer codes


def test_quantize_with_chunk_averaged_clamp():
    # App. B activations: per-sample chunks, averaged range, saturating quantization
    q8t = require_gpu()
    g = synth.rng(12)
    x = np.abs(g.standard_cauchy(size=(32, 16, 14, 14))).astype(np.float32)
    rng_dev = q8t.chunk_range(dev(x), 32)
    q, qp = q8t.quantize_with_range(dev(x), rng_dev, 8)
    vr = oracle.chunk_range(x, 32)
    stored, levels, oqp = oracle.quantize(x, 8, vrange=vr)
    same_qparams(q8t, qp, oqp)
    same_ints(host(q), stored)
    assert (levels == 255).sum() > 0      # the clamp is real


def test_diagnostics_reject_bad_arguments():
    q8t = require_gpu()
    x = dev(np.ones(8, np.float32))
    with pytest.raises(q8t.binding.Q8TError) as e:
        q8t.chunk_range(x, 9)             # more chunks than elements
    assert e.value.code == -2
