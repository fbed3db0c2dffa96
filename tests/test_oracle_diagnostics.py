"""Pins of the oracle's angle diagnostic (Sec. 3) and chunk-averaged clamping range (App. B)."""
import math

import numpy as np

import oracle
import synth


def test_angle_of_exactly_representable_tensor_is_zero():
    # every value sits on a level: Q(x) == x and cos(theta) == 1
    qp = oracle.QParams(0.0, 0.0, 0.5, 2.0, 10, 8)
    levels = np.arange(0, 256)
    x = (0.5 * (levels - 10)).astype(np.float32)
    stored = (levels - 128).astype(np.int8)
    dot, nx, nq, cos = oracle.quant_angle(x, stored, qp)
    assert dot == nx == nq
    assert cos == 1.0


def test_angle_small_hand_example():
    # x = (3, 4), Q(x) = (4, 3) (scale 1, zero point 0): cos = 24/25
    qp = oracle.QParams(0.0, 0.0, 1.0, 1.0, 0, 8)
    x = np.array([3.0, 4.0], np.float32)
    stored = np.array([4 - 128, 3 - 128], np.int8)
    dot, nx, nq, cos = oracle.quant_angle(x, stored, qp)
    assert (dot, nx, nq) == (24.0, 25.0, 25.0)
    assert abs(cos - 0.96) < 1e-15


def test_angle_orthogonal_and_opposite():
    qp = oracle.QParams(0.0, 0.0, 1.0, 1.0, 128, 8)     # stored code s <-> value s
    x = np.array([1.0, 0.0], np.float32)
    assert oracle.quant_angle(x, np.array([0, 5], np.int8), qp)[3] == 0.0
    assert oracle.quant_angle(x, np.array([-7, 0], np.int8), qp)[3] == -1.0
    assert oracle.quant_angle(np.zeros(2, np.float32), np.array([1, 1], np.int8), qp)[3] == 0.0   # zero norm


def test_angle_of_gaussian_weights_follows_the_additive_noise_model():
    # Sec. 3: for W ~ N(0, sigma) and a step much smaller than |W|, Q(W) = W + eps with eps uniform in
    # [-step/2, step/2] and nearly independent of W, so cos(theta) = |W| / |W + eps| with
    # |eps|^2 = N step^2 / 12, and the bound cos(theta) >= |W| / (|W| + |eps|) holds.
    g = synth.rng(3)
    w = synth.normal(g, (1 << 20,), std=1.0)
    for bits in (8, 6, 4):
        stored, _, qp = oracle.quantize(w, bits)
        dot, nx, nq, cos = oracle.quant_angle(w, stored, qp)
        step = float(qp.scale)
        predicted = 1.0 / math.sqrt(1.0 + step * step / 12.0 / (nx / w.size))
        assert abs(cos - predicted) < 0.05 * (1.0 - predicted), (bits, cos, predicted)
        eps_norm = math.sqrt(w.size / 12.0) * step
        assert cos >= math.sqrt(nx) / (math.sqrt(nx) + eps_norm)
    # fewer bits -> larger angle
    c8 = oracle.quant_angle(w, *oracle.quantize(w, 8)[::2])[3]
    c4 = oracle.quant_angle(w, *oracle.quantize(w, 4)[::2])[3]
    assert c4 < c8 < 1.0


def test_angle_uses_the_dequantized_value_of_16_bit_codes():
    g = synth.rng(4)
    x = synth.normal(g, (4096,), std=1e-3)
    stored, _, qp = oracle.quantize(x, 16, True, seed=9)
    xq = oracle.dequantize(stored, qp).astype(np.float64)
    dot, nx, nq, cos = oracle.quant_angle(x, stored, qp)
    xd = x.astype(np.float64)
    assert abs(dot - float(xd @ xq)) <= 1e-12 * abs(dot)
    assert abs(nq - float(xq @ xq)) <= 1e-12 * nq
    assert abs(cos - float(xd @ xq) / math.sqrt(float(xd @ xd) * float(xq @ xq))) < 1e-12


def test_chunk_range_with_one_chunk_is_the_global_range():
    g = synth.rng(5)
    x = synth.normal(g, (1000,), std=2.0)
    vmin, vmax = oracle.chunk_range(x, 1)
    assert vmin == x.min() and vmax == x.max()


def test_chunk_range_hand_example():
    # chunks (1,-2,3) (10,0,-4) (5,5,5) (-1,-1,8): maxima 3,10,5,8 -> 6.5 ; minima -2,-4,5,-1 -> -0.5
    x = np.array([1, -2, 3, 10, 0, -4, 5, 5, 5, -1, -1, 8], np.float32)
    assert oracle.chunk_range(x, 4) == (np.float32(-0.5), np.float32(6.5))
    # a different cut of the same data gives a different range: the chunks are contiguous
    # two chunks (1,-2,3,10,0,-4) (5,5,5,-1,-1,8): maxima 10, 8 -> 9 ; minima -4, -1 -> -2.5
    assert oracle.chunk_range(x, 2) == (np.float32(-2.5), np.float32(9.0))

def test_chunk_range_ragged_last_chunk_and_missing_chunks():
    x = np.arange(10, dtype=np.float32)           # K=4 -> chunks of 3,3,3,1
    vmin, vmax = oracle.chunk_range(x, 4)
    assert (vmin, vmax) == (np.float32((0 + 3 + 6 + 9) / 4), np.float32((2 + 5 + 8 + 9) / 4))
    x = np.arange(9, dtype=np.float32)            # K=4 -> chunk length 3: only 3 chunks exist
    assert oracle.chunk_range(x, 4) == (np.float32(3.0), np.float32(5.0))


def test_chunk_averaged_range_is_tighter_and_saturates():
    # heavy-tailed activations: the averaged range is inside the global one, and values outside it
    # quantize to the end levels (clamping is real)
    g = synth.rng(6)
    x = np.abs(g.standard_cauchy(size=(64, 512))).astype(np.float32)
    vmin, vmax = oracle.chunk_range(x, 64)
    assert x.min() <= vmin and vmax < x.max()
    stored, levels, qp = oracle.quantize(x, 8, vrange=(vmin, vmax))
    assert (levels[x > vmax] == 255).all() and (x > vmax).any()
    assert levels.max() == 255 and levels.min() == 0
    # and the step is smaller than with the global range
    _, _, qp_global = oracle.quantize(x, 8)
    assert qp.scale < qp_global.scale
