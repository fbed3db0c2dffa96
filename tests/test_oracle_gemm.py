"""Pins for the oracle's integer products: forward, layer gradient (eq. grad_layer) and
weight gradient (eq. grad_weight) of Section 4, FC and convolution.  CPU only."""
import numpy as np
import pytest
from scipy.signal import correlate2d

import oracle


def _qp(scale, zp, bits, vmin=0.0, vmax=0.0):
    return oracle.QParams(vmin, vmax, scale, 1.0 / scale, zp, bits)


def _rand_q(g, shape, bits=8):
    """random stored codes + params with a non-trivial zero point"""
    half = 2 ** (bits - 1)
    lv = g.integers(0, 2 ** bits, size=shape)
    zp = int(g.integers(0, 2 ** bits))
    dt = np.int8 if bits <= 8 else np.int16
    return (lv - half).astype(dt), lv.astype(np.int64) - zp, _qp(float(g.uniform(0.01, 0.1)), zp, bits)


# ---------------------------------------------------------------- FC
def test_fc_products_against_pure_python_loops():
    g = np.random.default_rng(0)
    M, K, N = 5, 7, 3
    sx, ax, px = _rand_q(g, (M, K))
    sw, aw, pw = _rand_q(g, (K, N))
    sg, ag, pg = _rand_q(g, (M, N))
    sg16, ag16, pg16 = _rand_q(g, (M, N), bits=16)
    _, acc = oracle.qgemm_fwd(sx, px, sw, pw)
    for m in range(M):
        for n in range(N):
            assert acc[m, n] == sum(int(ax[m, k]) * int(aw[k, n]) for k in range(K))
    _, acc = oracle.qgemm_dgrad(sg, pg, sw, pw)
    for m in range(M):
        for k in range(K):
            assert acc[m, k] == sum(int(ag[m, n]) * int(aw[k, n]) for n in range(N))
    _, acc = oracle.qgemm_wgrad(sx, px, sg16, pg16)
    for k in range(K):
        for n in range(N):
            assert acc[k, n] == sum(int(ax[m, k]) * int(ag16[m, n]) for m in range(M))


def test_fc_reduces_to_integer_matmul_when_scale_is_one():
    # data on the integer grid 0..255: scale 1, zero point 0 -> textbook integer matmul
    g = np.random.default_rng(1)
    x = g.integers(0, 256, size=(33, 70)).astype(np.float32)
    w = g.integers(0, 256, size=(70, 19)).astype(np.float32)
    x[0, 0], x[0, 1], w[0, 0], w[0, 1] = 0, 255, 0, 255
    sx, _, px = oracle.quantize(x, 8)
    sw, _, pw = oracle.quantize(w, 8)
    y, acc = oracle.qgemm_fwd(sx, px, sw, pw)
    ref = x.astype(np.int64) @ w.astype(np.int64)
    assert np.array_equal(acc, ref)
    assert np.array_equal(y, ref.astype(np.float32))


def test_fc_float_outputs_and_library_matmul():
    g = np.random.default_rng(2)
    M, K, N = 64, 256, 128
    sx, ax, px = _rand_q(g, (M, K))
    sw, aw, pw = _rand_q(g, (K, N))
    sg, ag, pg = _rand_q(g, (M, N))
    sg16, ag16, pg16 = _rand_q(g, (M, N), bits=16)
    y, acc = oracle.qgemm_fwd(sx, px, sw, pw)
    assert np.array_equal(acc, ax @ aw)
    assert np.array_equal(y, np.float32(px.scale * pw.scale) * acc.astype(np.float32))
    dx, acc = oracle.qgemm_dgrad(sg, pg, sw, pw)
    assert np.array_equal(acc, ag @ aw.T)
    assert np.array_equal(dx, np.float32(pg.scale * pw.scale) * acc.astype(np.float32))
    dw, acc = oracle.qgemm_wgrad(sx, px, sg16, pg16)
    assert np.array_equal(acc, ax.T @ ag16)
    ref = (acc.astype(np.float64) * float(np.float32(pg16.scale * px.scale))).astype(np.float32)
    assert np.array_equal(dw, ref)
    assert np.abs(acc).max() < 2 ** 31  # fits the 32-bit accumulator contract at these sizes


def test_quantized_fc_approaches_the_float_product():
    # 8-bit forward stays close to the float product; the 16-bit weight gradient is far closer
    # than an 8-bit one would be (Section 7: g_W uses the 16-bit copy of g_l)
    g = np.random.default_rng(3)
    x = g.standard_normal((64, 256)).astype(np.float32)
    w = (g.standard_normal((256, 128)) / 16).astype(np.float32)
    dy = (g.standard_normal((64, 128)) * 1e-3).astype(np.float32)
    sx, _, px = oracle.quantize(x, 8)
    sw, _, pw = oracle.quantize(w, 8)
    y, _ = oracle.qgemm_fwd(sx, px, sw, pw)
    ref = x.astype(np.float64) @ w.astype(np.float64)
    assert np.linalg.norm(y - ref) / np.linalg.norm(ref) < 0.02
    xq = oracle.dequantize(sx, px).astype(np.float64)
    ref_w = xq.T @ dy.astype(np.float64)
    s8, _, p8 = oracle.quantize(dy, 8, stochastic=True, seed=1)
    s16, _, p16 = oracle.quantize(dy, 16, stochastic=True, seed=2)
    dw16, _ = oracle.qgemm_wgrad(sx, px, s16, p16)
    dw8 = xq.T @ oracle.dequantize(s8, p8).astype(np.float64)
    e16 = np.linalg.norm(dw16 - ref_w) / np.linalg.norm(ref_w)
    e8 = np.linalg.norm(dw8 - ref_w) / np.linalg.norm(ref_w)
    assert e16 < 1e-4 and e8 > 50 * e16


# ---------------------------------------------------------------- convolution
CONV_CASES = [
    # N, C, H, W, K, R, S, stride, pad
    (2, 3, 7, 6, 4, 3, 3, 1, 1),
    (1, 2, 9, 9, 3, 3, 3, 2, 1),
    (2, 4, 5, 5, 3, 1, 1, 1, 0),
    (1, 3, 8, 8, 2, 1, 1, 2, 0),
    (1, 2, 11, 10, 2, 7, 7, 2, 3),
    (1, 1, 6, 7, 1, 3, 3, 1, 0),
]


def _conv_case(g, case):
    N, C, H, W, K, R, S, st, pad = case
    d = oracle.conv_desc(N, C, H, W, K, R, S, st, pad)
    sx, ax, px = _rand_q(g, (N, C, H, W))
    sw, aw, pw = _rand_q(g, (K, C, R, S))
    sg, ag, pg = _rand_q(g, (N, K, d.P, d.Q))
    sg16, ag16, pg16 = _rand_q(g, (N, K, d.P, d.Q), bits=16)
    return d, (sx, ax, px), (sw, aw, pw), (sg, ag, pg), (sg16, ag16, pg16)


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_forward_against_library_correlation(case):
    g = np.random.default_rng(10)
    d, (sx, ax, px), (sw, aw, pw), _, _ = _conv_case(g, case)
    y, acc = oracle.qconv_fwd(d, sx, px, sw, pw)
    pad, st = d.pad, d.stride
    axp = np.pad(ax, ((0, 0), (0, 0), (pad, pad), (pad, pad)))  # padded taps contribute zero
    for n in range(d.N):
        for k in range(d.K):
            full = sum(correlate2d(axp[n, c].astype(np.float64), aw[k, c].astype(np.float64),
                                   mode="valid") for c in range(d.C))
            ref = np.rint(full[::st, ::st]).astype(np.int64)
            assert np.array_equal(acc[n, k], ref[:d.P, :d.Q])
    assert np.array_equal(y, np.float32(px.scale * pw.scale) * acc.astype(np.float32))


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_forward_equals_gemm_on_im2col(case):
    g = np.random.default_rng(11)
    d, (sx, ax, px), (sw, aw, pw), _, _ = _conv_case(g, case)
    _, acc = oracle.qconv_fwd(d, sx, px, sw, pw)
    pad, st = d.pad, d.stride
    axp = np.pad(ax, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    cols = np.empty((d.N * d.P * d.Q, d.C * d.R * d.S), np.int64)
    row = 0
    for n in range(d.N):
        for p in range(d.P):
            for q in range(d.Q):
                cols[row] = axp[n, :, p * st:p * st + d.R, q * st:q * st + d.S].ravel()
                row += 1
    ref = (cols @ aw.reshape(d.K, -1).T).reshape(d.N, d.P, d.Q, d.K).transpose(0, 3, 1, 2)
    assert np.array_equal(acc, ref)


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_gradients_are_adjoints_of_the_forward_map(case):
    # <g, fwd(x, w)> = <dgrad(g, w), x> = <wgrad(x, g), w>, exactly, in integers.  A wrong index,
    # a flipped filter or a transposed operand in either gradient breaks the identity.
    g = np.random.default_rng(12)
    d, (sx, ax, px), (sw, aw, pw), (sg, ag, pg), (sg16, ag16, pg16) = _conv_case(g, case)
    _, fwd = oracle.qconv_fwd(d, sx, px, sw, pw)
    _, dg = oracle.qconv_dgrad(d, sg, pg, sw, pw)
    assert int((ag * fwd).sum()) == int((dg * ax).sum())
    _, wg = oracle.qconv_wgrad(d, sx, px, sg16, pg16)
    assert int((ag16 * fwd).sum()) == int((wg * aw).sum())


@pytest.mark.parametrize("case", CONV_CASES[:3])
def test_conv_gradients_against_pure_python_loops(case):
    g = np.random.default_rng(13)
    d, (sx, ax, px), (sw, aw, pw), (sg, ag, pg), (sg16, ag16, pg16) = _conv_case(g, case)
    _, dg = oracle.qconv_dgrad(d, sg, pg, sw, pw)
    _, wg = oracle.qconv_wgrad(d, sx, px, sg16, pg16)
    ref_dx = np.zeros((d.N, d.C, d.H, d.W), np.int64)
    ref_dw = np.zeros((d.K, d.C, d.R, d.S), np.int64)
    # scatter form: walk the forward taps and push contributions back
    for n in range(d.N):
        for k in range(d.K):
            for p in range(d.P):
                for q in range(d.Q):
                    for c in range(d.C):
                        for r in range(d.R):
                            for s in range(d.S):
                                h, w = p * d.stride + r - d.pad, q * d.stride + s - d.pad
                                if 0 <= h < d.H and 0 <= w < d.W:
                                    ref_dx[n, c, h, w] += ag[n, k, p, q] * aw[k, c, r, s]
                                    ref_dw[k, c, r, s] += ag16[n, k, p, q] * ax[n, c, h, w]
    assert np.array_equal(dg, ref_dx)
    assert np.array_equal(wg, ref_dw)


def _f32_product(sa, sb, acc):
    """fl32(s_a*s_b) * (float)acc: the product of two fp32 scales is exact in double, so one cast
    rounds it once; numpy's float32 multiply rounds the second product once."""
    return np.float32(sa * sb) * acc.astype(np.float32)


def _f64_product(sa, sb, acc):
    """(float)((double)acc * (double)fl32(s_a*s_b))"""
    return (acc.astype(np.float64) * float(np.float32(sa * sb))).astype(np.float32)


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_float_outputs_use_the_scales_of_their_own_operands(case):
    # every operand gets its own scale, so a swapped or missing scale changes the result
    g = np.random.default_rng(15)
    d, (sx, ax, px), (sw, aw, pw), (sg, ag, pg), (sg16, ag16, pg16) = _conv_case(g, case)
    assert len({px.scale, pw.scale, pg.scale, pg16.scale}) == 4
    y, acc = oracle.qconv_fwd(d, sx, px, sw, pw)
    assert np.array_equal(y, _f32_product(px.scale, pw.scale, acc))
    dx, acc = oracle.qconv_dgrad(d, sg, pg, sw, pw)
    assert np.array_equal(dx, _f32_product(pg.scale, pw.scale, acc))
    dw, acc = oracle.qconv_wgrad(d, sx, px, sg16, pg16)
    assert np.array_equal(dw, _f64_product(pg16.scale, px.scale, acc))


def test_float_outputs_with_power_of_two_scales_are_exact_multiples():
    # scales 1/2, 1/4, 1/8, 1/16: every float result is the accumulator times a power of two,
    # i.e. the exact real value rounded to fp32 once (closed form)
    g = np.random.default_rng(16)
    case = (2, 3, 6, 5, 4, 3, 3, 1, 1)
    d, (sx, ax, _), (sw, aw, _), (sg, ag, _), (sg16, ag16, _) = _conv_case(g, case)
    px, pw, pg, pg16 = _qp(0.5, 7, 8), _qp(0.25, 130, 8), _qp(0.125, 99, 8), _qp(0.0625, 30000, 16)
    y, acc = oracle.qconv_fwd(d, sx, px, sw, pw)
    assert np.array_equal(y, (acc / 8.0).astype(np.float32))
    dx, acc = oracle.qconv_dgrad(d, sg, pg, sw, pw)
    assert np.array_equal(dx, (acc / 32.0).astype(np.float32))
    dw, acc = oracle.qconv_wgrad(d, sx, px, sg16, pg16)
    assert np.array_equal(dw, (acc / 32.0).astype(np.float32))
    M, K, N = 6, 9, 5
    fx, fw = sx.reshape(-1)[:M * K].reshape(M, K), sw.reshape(-1)[:K * N].reshape(K, N)
    fg, fg16 = sg.reshape(-1)[:M * N].reshape(M, N), sg16.reshape(-1)[:M * N].reshape(M, N)
    y, acc = oracle.qgemm_fwd(fx, px, fw, pw)
    assert np.array_equal(y, (acc / 8.0).astype(np.float32))
    dx, acc = oracle.qgemm_dgrad(fg, pg, fw, pw)
    assert np.array_equal(dx, (acc / 32.0).astype(np.float32))
    dw, acc = oracle.qgemm_wgrad(fx, px, fg16, pg16)
    assert np.array_equal(dw, (acc / 32.0).astype(np.float32))


def test_conv_1x1_is_a_plain_matrix_product():
    g = np.random.default_rng(14)
    d, (sx, ax, px), (sw, aw, pw), (sg, ag, pg), (sg16, ag16, pg16) = _conv_case(
        g, (3, 8, 4, 5, 6, 1, 1, 1, 0))
    _, fwd = oracle.qconv_fwd(d, sx, px, sw, pw)
    assert np.array_equal(fwd, np.einsum("nchw,kc->nkhw", ax, aw[:, :, 0, 0]))
    _, dg = oracle.qconv_dgrad(d, sg, pg, sw, pw)
    assert np.array_equal(dg, np.einsum("nkhw,kc->nchw", ag, aw[:, :, 0, 0]))
    _, wg = oracle.qconv_wgrad(d, sx, px, sg16, pg16)
    assert np.array_equal(wg[:, :, 0, 0], np.einsum("nkhw,nchw->kc", ag16, ax))


def test_byte_split_of_a_16_bit_code_is_exact():
    # identity used to run a 16x8-bit product on 8-bit multipliers: with s the stored int16,
    # hi = s >> 8 (signed) and lo = (s & 255) - 128, s == 256*hi + lo + 128 for every code
    s = np.arange(-32768, 32768, dtype=np.int64)
    hi = s >> 8
    lo = (s & 255) - 128
    assert hi.min() == -128 and hi.max() == 127 and lo.min() == -128 and lo.max() == 127
    assert np.array_equal(256 * hi + lo + 128, s)
