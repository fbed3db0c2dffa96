"""Pins for the oracle's quantizer (Appendix B scheme, stochastic rounding of Section 4)
and its counter-based generator.  CPU only."""
import math
import os

import numpy as np
import pytest

import oracle


# ---------------------------------------------------------------- generator
def _read_rng_golden(golden_dir):
    words, r16 = [], None
    with open(os.path.join(golden_dir, "rng_vectors.txt")) as f:
        for line in f:
            t = line.split()
            if not t or t[0].startswith("#"):
                continue
            if t[0] == "words":
                words.append((int(t[1]), int(t[2], 16), int(t[3], 16)))
            elif t[0] == "r16":
                r16 = [int(v) for v in t[1:]]
    return words, r16


def test_rng_matches_stored_vectors(golden_dir):
    words, r16 = _read_rng_golden(golden_dir)
    for g, w0, w1 in words:
        assert oracle.rng_words(g, 1) == (w0, w1)
    assert [oracle.r16(i, 1) for i in range(len(r16))] == r16


def test_rng_words_feed_four_elements():
    # elements 4g..4g+3 take the low/high halves of w0 then of w1
    for seed in (0, 7, 2 ** 32 + 5):
        for g in (0, 3, 1000):
            w0, w1 = oracle.rng_words(g, seed)
            got = [oracle.r16(4 * g + j, seed) for j in range(4)]
            assert got == [w0 & 0xFFFF, w0 >> 16, w1 & 0xFFFF, w1 >> 16]


@pytest.mark.parametrize("seed", [0, 1, 2, 3, 2 ** 32, 2 ** 32 + 1, 0xDEADBEEFCAFEF00D])
def test_rng_uniformity(seed):
    n = 1 << 18
    r = np.array([oracle.r16(i, seed) for i in range(0, n)], dtype=np.float64)
    u = (r + 0.5) / 65536.0
    assert abs(u.mean() - 0.5) < 4 * math.sqrt(1 / 12 / n)
    assert abs(u.var() - 1 / 12) < 1e-3
    # chi-square on the high and the low byte, 255 degrees of freedom
    for b in ((r.astype(np.int64) >> 8), (r.astype(np.int64) & 255)):
        cnt = np.bincount(b, minlength=256)
        chi2 = ((cnt - n / 256) ** 2 / (n / 256)).sum()
        assert 150 < chi2 < 380
    for lag in (1, 4):
        rho = np.corrcoef(u[:-lag], u[lag:])[0, 1]
        assert abs(rho) < 0.01


def test_rng_seeds_are_decorrelated():
    n = 1 << 16
    a = np.array([oracle.r16(i, 11) for i in range(n)], dtype=np.float64)
    b = np.array([oracle.r16(i, 12) for i in range(n)], dtype=np.float64)
    c = np.array([oracle.r16(i, 11 + 2 ** 32) for i in range(n)], dtype=np.float64)
    assert abs(np.corrcoef(a, b)[0, 1]) < 0.02
    assert abs(np.corrcoef(a, c)[0, 1]) < 0.02


# ---------------------------------------------------------------- levels
@pytest.mark.parametrize("bits", [2, 4, 8, 12, 16])
def test_endpoints_land_on_first_and_last_level(bits):
    g = np.random.default_rng(bits)
    x = g.standard_normal(4099).astype(np.float32) * 3
    stored, lv, qp = oracle.quantize(x, bits)
    qmax = 2 ** bits - 1
    assert lv[np.argmin(x)] == 0
    assert lv[np.argmax(x)] == qmax
    assert lv.min() == 0 and lv.max() == qmax
    assert qp.vmin == x.min() and qp.vmax == x.max()
    # stored form is level - 2^(M-1)
    assert np.array_equal(stored.astype(np.int64) + 2 ** (bits - 1), lv)
    # real zero maps to the zero point and back to exactly zero
    _, lv0, _ = oracle.quantize(np.zeros(1, np.float32), bits, vrange=(qp.vmin, qp.vmax))
    assert lv0[0] == qp.zero_point
    z = np.array([qp.zero_point - 2 ** (bits - 1)], dtype=stored.dtype)
    assert oracle.dequantize(z, qp)[0] == 0.0


def test_integer_grid_is_reproduced_exactly():
    # integers 0..255 with 8 bits: scale 1, zero point 0, code == value
    x = np.arange(256, dtype=np.float32)
    np.random.default_rng(0).shuffle(x)
    _, lv, qp = oracle.quantize(x, 8)
    assert qp.scale == 1.0 and qp.zero_point == 0
    assert np.array_equal(lv, x.astype(np.int32))
    # a hand-built range [-51, 204]: scale 1, zero point 51
    x = np.arange(-51, 205, dtype=np.float32)
    for stochastic in (False, True):
        for seed in (0, 1, 99):
            _, lv, qp = oracle.quantize(x, 8, stochastic=stochastic, seed=seed)
            assert qp.scale == 1.0 and qp.zero_point == 51
            assert np.array_equal(lv, (x + 51).astype(np.int32))  # grid values never move


def test_range_is_widened_to_contain_zero():
    x = np.linspace(2.0, 3.0, 100).astype(np.float32)  # all positive
    _, lv, qp = oracle.quantize(x, 8)
    assert qp.vmin == 0.0 and qp.zero_point == 0
    assert lv.max() == 255 and lv.min() == int(np.rint(np.float32(2.0) * qp.inv_scale))
    x = -x
    _, lv, qp = oracle.quantize(x, 8)
    assert qp.vmax == 0.0 and qp.zero_point == 255 and lv.min() == 0


def test_constant_tensor():
    _, lv, qp = oracle.quantize(np.zeros(17, np.float32), 8)
    assert qp.scale == 1.0 and qp.zero_point == 0 and not lv.any()


@pytest.mark.parametrize("bits", [4, 8, 16])
def test_nearest_rounding_error_bound_and_noise_power(bits):
    # Appendix A, eq. (Integral): uniform rounding noise has E[eps^2] = Delta^2/12,
    # and |eps| <= Delta/2 everywhere inside the range.
    g = np.random.default_rng(5)
    x = g.standard_normal(200000).astype(np.float32)
    stored, _, qp = oracle.quantize(x, bits)
    xd = oracle.dequantize(stored, qp).astype(np.float64)
    err = xd - x
    # the zero point is rounded, so the grid is shifted by at most half a step at the ends
    assert np.abs(err).max() <= qp.scale * (1.0 + 1e-3)
    inner = (x > qp.vmin + qp.scale) & (x < qp.vmax - qp.scale)
    # t = x*inv_scale + zp is an fp32 number: near 2^bits its spacing is 2^(bits-24) levels
    slack = 1e-3 + 4 * 2.0 ** (bits - 24)
    assert np.abs(err[inner]).max() <= qp.scale * (0.5 + slack)
    assert np.mean(err[inner] ** 2) == pytest.approx(qp.scale ** 2 / 12, rel=0.03)


@pytest.mark.parametrize("bits", [2, 3, 4, 6, 8])
def test_cosine_similarity_bound(bits):
    # Section 5.2, eq. (40): cos(theta) >= sigma / (sigma + Delta/sqrt(12)) for Gaussian input
    g = np.random.default_rng(bits)
    sigma = 0.7
    x = (g.standard_normal(1 << 16) * sigma).astype(np.float32)
    stored, _, qp = oracle.quantize(x, bits)
    xd = oracle.dequantize(stored, qp).astype(np.float64)
    cos = float(np.dot(x, xd) / np.linalg.norm(x) / np.linalg.norm(xd))
    assert cos >= sigma / (sigma + qp.scale / math.sqrt(12)) - 1e-4
    assert cos <= 1.0 + 1e-12


# ---------------------------------------------------------------- stochastic rounding
def test_stochastic_rounding_is_unbiased_over_seeds():
    # Section 4: gradients need an unbiased quantizer
    g = np.random.default_rng(3)
    x = (g.standard_normal(2000) * 1e-3).astype(np.float32)
    S = 400
    acc = np.zeros(x.shape, np.float64)
    for seed in range(S):
        stored, _, qp = oracle.quantize(x, 8, stochastic=True, seed=seed)
        acc += oracle.dequantize(stored, qp)
    mean = acc / S
    inner = (x > qp.vmin + qp.scale) & (x < qp.vmax - qp.scale)
    # per-element standard error <= scale/(2 sqrt S); allow 5 sigma, and check the average bias
    assert np.abs(mean - x)[inner].max() < 5 * qp.scale / (2 * math.sqrt(S))
    assert abs(np.mean(mean - x)) < 0.02 * qp.scale
    # nearest rounding is biased on the same data point by point (sanity: the test can fail)
    stored, _, qp = oracle.quantize(x, 8)
    assert np.abs(oracle.dequantize(stored, qp) - x).max() > 0.4 * qp.scale


def test_stochastic_rounding_probability_equals_fraction():
    # a ramp of values with known fractional parts on the grid scale=1, zero point 0
    n = 1 << 16
    for frac in (0.0, 0.125, 0.5, 0.8125):
        x = np.full(n, 3.0 + frac, np.float32)
        x[0], x[1] = 0.0, 255.0  # fix the range to [0,255] -> scale 1
        _, lv, qp = oracle.quantize(x, 8, stochastic=True, seed=42)
        assert qp.scale == 1.0 and qp.zero_point == 0
        up = (lv[2:] == 4).mean()
        assert set(np.unique(lv[2:])) <= {3, 4}
        assert abs(up - frac) < 4 * math.sqrt(max(frac * (1 - frac), 1e-9) / n) + 2 ** -16


def test_stochastic_rounding_uses_the_elements_own_random_bits():
    # up  <=>  frac*65536 > r16 + 0.5, element by element
    n = 4096
    x = np.full(n, 10.25, np.float32)
    x[0], x[1] = 0.0, 255.0
    seed = 2 ** 40 + 17
    _, lv, _ = oracle.quantize(x, 8, stochastic=True, seed=seed)
    for i in range(2, n):
        expect = 10 + (1 if 0.25 * 65536 > oracle.r16(i, seed) + 0.5 else 0)
        assert lv[i] == expect


def test_stochastic_levels_stay_next_to_the_real_value():
    g = np.random.default_rng(8)
    x = (g.standard_normal(50000) * 1e-3).astype(np.float32)
    for bits in (8, 16):
        stored, lv, qp = oracle.quantize(x, bits, stochastic=True, seed=5)
        t = x.astype(np.float64) / qp.scale + qp.zero_point
        assert np.all(lv >= np.floor(t - 1e-3 * 2 ** (bits - 8)).clip(0, 2 ** bits - 1))
        assert np.all(lv <= np.ceil(t + 1e-3 * 2 ** (bits - 8)).clip(0, 2 ** bits - 1))


def test_sixteen_bit_copy_is_finer_than_eight_bit_copy():
    # Gradient bifurcation (Section 1): the 16-bit copy of g carries 256x less rounding noise
    g = np.random.default_rng(9)
    x = (g.standard_normal(100000) * 1e-3).astype(np.float32)
    s8, _, q8 = oracle.quantize(x, 8, stochastic=True, seed=1)
    s16, _, q16 = oracle.quantize(x, 16, stochastic=True, seed=2)
    e8 = np.std(oracle.dequantize(s8, q8) - x)
    e16 = np.std(oracle.dequantize(s16, q16) - x)
    assert q8.vmin == q16.vmin and q8.vmax == q16.vmax
    assert e8 / e16 == pytest.approx(65535 / 255, rel=0.05)


# ---------------------------------------------------------------- independent float32 cross-check
def test_matches_numpy_float32_sequence():
    # not a pin by itself (same formula), but it catches a compiler fusing mul+add
    g = np.random.default_rng(21)
    x = (g.standard_normal(100003) * 2.5).astype(np.float32)
    _, lv, qp = oracle.quantize(x, 8)
    vmin, vmax = min(x.min(), np.float32(0)), max(x.max(), np.float32(0))
    scale = np.float32(vmax - vmin) / np.float32(255)
    inv = np.float32(1) / scale
    zp = int(np.clip(np.rint(np.float32(-vmin) * inv), 0, 255))
    t = (x * inv).astype(np.float32) + np.float32(zp)
    ref = np.clip(np.rint(t), 0, 255).astype(np.int32)
    assert (qp.scale, qp.inv_scale, qp.zero_point) == (scale, inv, zp)
    assert np.array_equal(lv, ref)


def test_values_outside_a_supplied_range_saturate():
    # range [-1, 2]: scale 3/255, zero point 85, both ends on the grid
    x = np.array([-1e30, -5.0, -1.0, 0.0, 2.0, 5.0, 1e30, 3e9], np.float32)
    for stochastic in (False, True):
        _, lv, qp = oracle.quantize(x, 8, stochastic=stochastic, seed=3, vrange=(-1.0, 2.0))
        assert qp.zero_point == 85
        assert list(lv) == [0, 0, 0, 85, 255, 255, 255, 255]
