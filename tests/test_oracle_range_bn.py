"""Pins for the oracle's Range BN (Section 3, eq. (range); backward rule of Section 7).  CPU only."""
import math
import os

import numpy as np
import pytest

import oracle


def _golden_scale(golden_dir):
    vals, printed = [], []
    with open(os.path.join(golden_dir, "range_bn_scale.txt")) as f:
        for line in f:
            t = line.split()
            if not t or t[0].startswith("#"):
                continue
            (printed if len(t[1]) <= 4 else vals).append((int(t[0]), float(t[1])))
    return vals, printed


def test_scale_adjustment_closed_form(golden_dir):
    vals, printed = _golden_scale(golden_dir)
    assert len(vals) == 3 and len(printed) == 1
    for n, c in vals:
        assert oracle.range_bn_scale(n) == pytest.approx(c, abs=5e-10)
        assert oracle.range_bn_scale(n) == pytest.approx((2 * math.log(n)) ** -0.5, rel=1e-15)
    # the worked example of Section 5: sqrt(2 ln(3*3*2048*1024)) printed as 5.7 (truncated)
    for n, v in printed:
        assert n == 3 * 3 * 2048 * 1024
        assert math.floor(10 / oracle.range_bn_scale(n)) / 10 == v


def _gauss(seed, N, C, H, W, spread=True):
    g = np.random.default_rng(seed)
    x = g.standard_normal((N, C, H, W))
    if spread:
        x = x * g.uniform(0.1, 3, size=(1, C, 1, 1)) + g.uniform(-2, 2, size=(1, C, 1, 1))
    return x.astype(np.float32)


def test_forward_matches_the_equation_in_double():
    x = _gauss(0, 8, 5, 6, 7)
    g = np.random.default_rng(1)
    gamma = g.uniform(-2, 2, 5).astype(np.float32)
    beta = g.uniform(-1, 1, 5).astype(np.float32)
    for eps in (0.0, 1e-5):
        y, stats, _, _ = oracle.range_bn_fwd(x, gamma, beta, eps)
        ref = oracle.range_bn_fwd_f64(x, gamma, beta, eps)
        assert np.allclose(y, ref, rtol=1e-5, atol=1e-6)
    # and the double routine is eq. (range) as numpy writes it
    xd = x.astype(np.float64)
    mu = xd.mean(axis=(0, 2, 3), keepdims=True)
    cen = xd - mu
    rng = cen.max(axis=(0, 2, 3), keepdims=True) - cen.min(axis=(0, 2, 3), keepdims=True)
    n = 8 * 6 * 7
    ref2 = cen / ((2 * math.log(n)) ** -0.5 * rng)
    assert np.allclose(oracle.range_bn_fwd_f64(x), ref2, rtol=1e-12, atol=1e-12)
    assert np.array_equal(stats[1], x.min(axis=(0, 2, 3)))
    assert np.array_equal(stats[2], x.max(axis=(0, 2, 3)))
    assert np.allclose(stats[0], mu.ravel(), rtol=1e-6, atol=1e-7)


def test_output_is_centred_and_spans_sqrt_2_ln_n():
    # with eps = 0: mean(xhat) = 0 and max(xhat) - min(xhat) = 1/C(n) = sqrt(2 ln n)
    x = _gauss(2, 16, 6, 5, 5)
    n = 16 * 25
    y, _, _, _ = oracle.range_bn_fwd(x, eps=0.0)
    span = y.max(axis=(0, 2, 3)) - y.min(axis=(0, 2, 3))
    assert np.allclose(span, math.sqrt(2 * math.log(n)), rtol=1e-5)
    assert np.abs(y.astype(np.float64).mean(axis=(0, 2, 3))).max() < 1e-6
    beta = np.linspace(-1, 1, 6).astype(np.float32)
    y, _, _, _ = oracle.range_bn_fwd(x, None, beta, 0.0)
    assert np.allclose(y.astype(np.float64).mean(axis=(0, 2, 3)), beta, atol=1e-6)


def test_invariance_to_shift_and_positive_scale():
    # Section 5: BN(C*W*x) = BN(W*x); powers of two keep the float arithmetic exact
    x = _gauss(3, 8, 4, 6, 6)
    y0, _, _, _ = oracle.range_bn_fwd(x, eps=0.0)
    y1, _, _, _ = oracle.range_bn_fwd(x * np.float32(8.0), eps=0.0)
    assert np.array_equal(y0, y1)
    y2, _, _, _ = oracle.range_bn_fwd(x * np.float32(3.7) + np.float32(1.3), eps=0.0)
    assert np.allclose(y0, y2, rtol=1e-4, atol=2e-5)


def test_proportional_to_standard_batch_norm_within_the_papers_bound(golden_dir):
    with open(os.path.join(golden_dir, "gaussian_range_bound.txt")) as f:
        lo, hi = [float(v) for v in [l for l in f if not l.startswith("#")][0].split()]
    cv = {}
    for n_side, N in ((4, 4), (8, 16), (16, 64)):
        x = _gauss(4, N, 64, n_side, n_side)
        n = N * n_side * n_side
        y = oracle.range_bn_fwd_f64(x, eps=0.0)
        s = oracle.standard_bn_f64(x)
        # same centring: y is an exact multiple of standard BN's output, channel by channel
        ratio = (s * y).sum(axis=(0, 2, 3)) / (y * y).sum(axis=(0, 2, 3))  # = C(n)*range/sigma
        assert np.allclose(s, y * ratio[None, :, None, None], rtol=1e-9, atol=1e-9)
        # Section 3:  0.325 sigma <= C(n) range <= 2 sigma, a statement about the expectation:
        # the mean over 64 channels obeys it, single channels only once n is large
        assert ratio.mean() > lo and ratio.mean() < hi
        if n >= 16384:
            assert ratio.min() > lo and ratio.max() < hi
        cv[n] = ratio.std() / ratio.mean()
    ns = sorted(cv)
    assert cv[ns[0]] > cv[ns[1]] > cv[ns[2]]  # the estimate of sigma tightens as n grows


def test_without_the_scale_adjustment_the_output_is_not_unit_scale():
    # C(n) is what brings the range to the scale of sigma: with it the per-channel std of the
    # output is O(1) (between 1/2 and 1/0.325), without it it would be about 1/range ~ 0.15
    x = _gauss(5, 64, 8, 8, 8)
    y = oracle.range_bn_fwd_f64(x, eps=0.0)
    sd = y.std(axis=(0, 2, 3))
    assert sd.min() > 0.5 and sd.max() < 1 / 0.325


# ---------------------------------------------------------------- fused 8-bit output
def test_analytic_output_range_equals_true_extrema():
    x = _gauss(6, 8, 6, 7, 5)
    g = np.random.default_rng(6)
    gamma = g.uniform(-2, 2, 6).astype(np.float32)
    beta = g.uniform(-1, 1, 6).astype(np.float32)
    y, stats, q, qp = oracle.range_bn_fwd(x, gamma, beta, 1e-5, quantized=True)
    # Section 4: min and max are known to the normalizer, no further pass is needed
    assert qp.vmin == min(y.min(), 0) and qp.vmax == max(y.max(), 0)
    s2, _, qp2 = oracle.quantize(y, 8)
    assert qp2.as_tuple() == qp.as_tuple()
    assert np.array_equal(s2, q)


# ---------------------------------------------------------------- backward
def _loss_f64(x, dy, gamma, beta, eps):
    return float((oracle.range_bn_fwd_f64(x, gamma, beta, eps) * dy).sum())


@pytest.mark.parametrize("eps", [0.0, 1e-3])
def test_backward_against_central_differences(eps):
    g = np.random.default_rng(7)
    N, C, H, W = 3, 2, 2, 3
    x = g.standard_normal((N, C, H, W)).astype(np.float32)
    dy = g.standard_normal((N, C, H, W)).astype(np.float32)
    gamma = g.uniform(0.5, 2, C).astype(np.float32)
    beta = g.uniform(-1, 1, C).astype(np.float32)
    stats = oracle.range_bn_stats(x)
    dx, dgamma, dbeta = oracle.range_bn_bwd(x, dy, stats, gamma, eps)
    xd, dyd = x.astype(np.float64), dy.astype(np.float64)
    h = 1e-6
    num = np.zeros_like(xd)
    for idx in np.ndindex(*x.shape):
        xp, xm = xd.copy(), xd.copy()
        xp[idx] += h
        xm[idx] -= h
        num[idx] = (_loss_f64(xp, dyd, gamma, beta, eps) - _loss_f64(xm, dyd, gamma, beta, eps)) / (2 * h)
    assert np.allclose(dx, num, rtol=2e-4, atol=2e-5)
    for c in range(C):
        gp, gm = gamma.astype(np.float64).copy(), gamma.astype(np.float64).copy()
        gp[c] += h
        gm[c] -= h
        ng = (_loss_f64(xd, dyd, gp, beta, eps) - _loss_f64(xd, dyd, gm, beta, eps)) / (2 * h)
        assert dgamma[c] == pytest.approx(ng, rel=1e-4, abs=1e-5)
        assert dbeta[c] == pytest.approx(dyd[:, c].sum(), rel=1e-5, abs=1e-6)


def test_backward_invariants():
    # shift invariance of the forward map -> sum_j dx_j = 0;
    # scale invariance (eps = 0)           -> sum_j dx_j (x_j - mu) = 0
    x = _gauss(8, 8, 5, 6, 6)
    g = np.random.default_rng(8)
    dy = (g.standard_normal(x.shape) * 1e-2).astype(np.float32)
    gamma = g.uniform(0.5, 2, 5).astype(np.float32)
    stats = oracle.range_bn_stats(x)
    dx, _, _ = oracle.range_bn_bwd(x, dy, stats, gamma, 0.0)
    dxd = dx.astype(np.float64)
    scale = np.abs(dxd).sum(axis=(0, 2, 3))
    assert np.all(np.abs(dxd.sum(axis=(0, 2, 3))) < 1e-5 * scale)
    cen = x.astype(np.float64) - stats[0].astype(np.float64)[None, :, None, None]
    assert np.all(np.abs((dxd * cen).sum(axis=(0, 2, 3))) < 1e-5 * (np.abs(dxd) * np.abs(cen)).sum(axis=(0, 2, 3)))


def test_every_coordinate_attaining_an_extremum_receives_the_term():
    # Section 7: the derivative of max/min is one at the coordinates (plural) where it is attained
    g = np.random.default_rng(9)
    x = g.standard_normal((4, 1, 3, 3)).astype(np.float32)
    x.flat[5] = x.flat[20] = 9.0    # two maxima
    x.flat[7] = x.flat[30] = -9.0   # two minima
    dy = g.standard_normal(x.shape).astype(np.float32)
    stats = oracle.range_bn_stats(x)
    sums = oracle.range_bn_bwd_sums(x, dy, stats, 0.0)
    dx, _, _ = oracle.range_bn_bwd(x, dy, stats, None, 0.0)
    n = x.size
    cn = (2 * math.log(n)) ** -0.5
    inv = 1.0 / (cn * 18.0)
    base = inv * (dy.astype(np.float64).ravel() - sums[0, 0] / n)
    term = inv * cn * sums[1, 0]
    ref = base.copy()
    ref[[5, 20]] -= term
    ref[[7, 30]] += term
    assert np.allclose(dx.ravel(), ref, rtol=1e-5, atol=1e-6)
    assert abs(term) > 1e-3  # the term is large enough for the check to bite


def test_backward_sums_feed_dgamma_and_dbeta():
    x = _gauss(10, 6, 3, 4, 4)
    dy = _gauss(11, 6, 3, 4, 4, spread=False)
    stats = oracle.range_bn_stats(x)
    y, _, _, _ = oracle.range_bn_fwd(x, eps=1e-5)
    _, dgamma, dbeta = oracle.range_bn_bwd(x, dy, stats, None, 1e-5)
    assert np.allclose(dbeta, dy.astype(np.float64).sum(axis=(0, 2, 3)), rtol=1e-6)
    assert np.allclose(dgamma, (dy.astype(np.float64) * y).sum(axis=(0, 2, 3)), rtol=1e-6, atol=1e-6)


# ---------------------------------------------------------------- Range BN followed by ReLU
def test_relu_output_range_is_known_without_a_pass_over_the_data():
    # the rectified output's extrema are the rectified images of the channel extrema: quantizing
    # with that analytic range gives the codes a min/max search over the rectified output gives
    x = _gauss(11, 8, 6, 7, 6)
    g = np.random.default_rng(12)
    gamma = g.uniform(-2, 2, 6).astype(np.float32)
    beta = g.uniform(-1, 1, 6).astype(np.float32)
    stats = oracle.range_bn_stats(x)
    y0, _, _, _ = oracle.range_bn_fwd(x, gamma, beta, 1e-5, stats=stats)
    y, q, qp = oracle.range_bn_relu_fwd(x, stats, gamma, beta, 1e-5, quantized=True)
    assert (y >= 0).all() and np.array_equal(y[y0 > 0], y0[y0 > 0]) and (y[y0 <= 0] == 0).all()
    assert qp.vmin == 0.0 and qp.vmax == y.max()
    s2, _, qp2 = oracle.quantize(y, 8)
    assert qp2.as_tuple() == qp.as_tuple()
    assert np.array_equal(s2, q)
    # zero is exactly representable: every rectified element sits on the zero point, whose
    # dequantized value is exactly 0
    assert (q[y == 0].astype(np.int32) + 128 == qp.zero_point).all()
    assert (oracle.dequantize(q, qp)[y == 0] == 0).all()


def test_relu_with_an_all_negative_output_degenerates_cleanly():
    x = _gauss(13, 4, 2, 3, 3)
    stats = oracle.range_bn_stats(x)
    beta = np.full(2, -100.0, np.float32)
    y, q, qp = oracle.range_bn_relu_fwd(x, stats, None, beta, 1e-5, quantized=True)
    assert (y == 0).all() and qp.vmin == 0.0 and qp.vmax == 0.0
    assert (oracle.dequantize(q, qp) == 0).all()


def test_relu_backward_against_central_differences():
    g = np.random.default_rng(14)
    N, C, H, W = 3, 2, 2, 3
    x = g.standard_normal((N, C, H, W)).astype(np.float32)
    dy = g.standard_normal((N, C, H, W)).astype(np.float32)
    gamma = g.uniform(0.5, 2, C).astype(np.float32)
    beta = g.uniform(-0.5, 0.5, C).astype(np.float32)
    eps = 1e-3
    stats = oracle.range_bn_stats(x)
    dx, dgamma, dbeta = oracle.range_bn_relu_bwd(x, dy, stats, gamma, beta, eps)
    xd, dyd = x.astype(np.float64), dy.astype(np.float64)

    def loss(xx, gg, bb):
        return float((np.maximum(oracle.range_bn_fwd_f64(xx, gg, bb, eps), 0.0) * dyd).sum())

    y64 = oracle.range_bn_fwd_f64(xd, gamma, beta, eps)
    assert np.abs(y64).min() > 1e-3          # no element sits on the kink
    assert (y64 > 0).any() and (y64 < 0).any()
    h = 1e-6
    num = np.zeros_like(xd)
    for idx in np.ndindex(*x.shape):
        xp, xm = xd.copy(), xd.copy()
        xp[idx] += h
        xm[idx] -= h
        num[idx] = (loss(xp, gamma, beta) - loss(xm, gamma, beta)) / (2 * h)
    assert np.allclose(dx, num, rtol=2e-4, atol=2e-5)
    for c in range(C):
        gp, gm = gamma.astype(np.float64).copy(), gamma.astype(np.float64).copy()
        gp[c] += h
        gm[c] -= h
        assert dgamma[c] == pytest.approx((loss(xd, gp, beta) - loss(xd, gm, beta)) / (2 * h), rel=1e-4, abs=1e-5)
        bp, bm = beta.astype(np.float64).copy(), beta.astype(np.float64).copy()
        bp[c] += h
        bm[c] -= h
        assert dbeta[c] == pytest.approx((loss(xd, gamma, bp) - loss(xd, gamma, bm)) / (2 * h), rel=1e-4, abs=1e-5)


def test_relu_mask_is_the_sign_of_the_forward_output():
    x = _gauss(15, 4, 3, 5, 5)
    g = np.random.default_rng(16)
    dy = g.standard_normal(x.shape).astype(np.float32)
    gamma = g.uniform(-2, 2, 3).astype(np.float32)
    beta = g.uniform(-1, 1, 3).astype(np.float32)
    stats = oracle.range_bn_stats(x)
    y, _, _, _ = oracle.range_bn_fwd(x, gamma, beta, 1e-5, stats=stats)
    m = oracle.range_bn_relu_mask(x, dy, stats, gamma, beta, 1e-5)
    assert np.array_equal(m, np.where(y > 0, dy, np.float32(0)))
