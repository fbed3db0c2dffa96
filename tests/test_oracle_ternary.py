"""Pins for the oracle's ternarized back-propagation pieces (appendix "Additional Experiments",
Algorithm 1): stochastic ternarization, binarization, the XNOR + population count product and the
multi-sample weight gradient.  CPU only."""
import numpy as np

import oracle


def test_ternary_codes_are_signs_or_zero_and_the_largest_element_is_always_kept():
    g = np.random.default_rng(0)
    x = (g.standard_normal(20000) * 1e-3).astype(np.float32)
    for seed in (0, 1, 2 ** 40 + 7):
        t, s = oracle.ternarize(x, seed)
        assert s == np.abs(x).max()
        assert set(np.unique(t)) <= {-1, 0, 1}
        nz = t != 0
        assert np.array_equal(t[nz], np.sign(x[nz]).astype(np.int8))      # a kept element carries its sign
        assert t[np.argmax(np.abs(x))] != 0                                # probability 1
    t, s = oracle.ternarize(np.zeros(7, np.float32), 3)
    assert s == 0 and not t.any()
    t, _ = oracle.ternarize(np.array([0.0, -2.0, 2.0, 0.0], np.float32), 5)
    assert t.tolist() == [0, -1, 1, 0]                                     # zeros never move, extremes always do


def test_ternarization_is_unbiased_and_keeps_with_probability_proportional_to_magnitude():
    # ramp of magnitudes k/16 of the maximum: P(kept) = k/16, so E[scale * t] = x
    x = np.concatenate([np.arange(17) / 16.0, -np.arange(17) / 16.0]).astype(np.float32) * 3.0
    S = 6000
    kept = np.zeros(x.size)
    mean = np.zeros(x.size)
    for seed in range(S):
        t, s = oracle.ternarize(x, seed)
        kept += t != 0
        mean += s * t.astype(np.float64)
    p = np.abs(x) / 3.0
    assert np.abs(kept / S - p).max() < 4 * 0.5 / np.sqrt(S)
    assert np.abs(mean / S - x).max() < 4 * 3.0 * 0.5 / np.sqrt(S)
    # the decision itself, element by element: |x|/max * 65536 > r16 + 0.5 in fp32
    t, s = oracle.ternarize(x, 11)
    r = np.array([oracle.r16(i, 11) for i in range(x.size)], np.float32)
    lhs = (np.abs(x) * (np.float32(1.0) / s)).astype(np.float32) * np.float32(65536.0)
    assert np.array_equal(t != 0, lhs > r + np.float32(0.5))


def test_binarize_and_bit_rows():
    x = np.array([[0.5, -0.0, -1.0, 0.0, 3.0], [-2.0, 2.0, -1e-30, 1e-30, -5.0]], np.float32)
    b = oracle.binarize(x)
    assert b.tolist() == [[1, 1, -1, 1, 1], [-1, 1, -1, 1, -1]]            # x >= 0 -> +1 (zero of either sign too)
    bits = oracle.pack_bits(b)
    assert bits.shape == (2, 1) and bits[0, 0] == 0b11011 and bits[1, 0] == 0b01010
    bt = oracle.pack_bits(b, transpose=True)                               # one bit row per column, bits along the rows
    assert bt.shape == (5, 1) and bt[:, 0].tolist() == [0b01, 0b11, 0b00, 0b11, 0b01]
    g = np.random.default_rng(1)
    c = np.where(g.random((7, 70)) < 0.5, -1, 1).astype(np.int8)
    bits = oracle.pack_bits(c)
    assert bits.shape == (7, 3)
    un = ((bits[:, :, None] >> np.arange(32, dtype=np.uint32)) & 1).reshape(7, 96).astype(np.int64)
    assert np.array_equal(un[:, :70] * 2 - 1, c) and not un[:, 70:].any()  # bits past the end are 0


def test_xnor_product_is_the_matrix_product_of_the_signs():
    g = np.random.default_rng(2)
    for M, N, K in ((5, 4, 7), (9, 13, 64), (3, 2, 100), (16, 16, 257)):
        a = np.where(g.random((M, K)) < 0.5, -1, 1).astype(np.int8)
        w = np.where(g.random((K, N)) < 0.3, -1, 1).astype(np.int8)
        y = oracle.xnor_gemm(oracle.pack_bits(a), oracle.pack_bits(w, transpose=True), K)
        assert np.array_equal(y, a.astype(np.int64) @ w.astype(np.int64))
        # matches minus mismatches = 2 * popcount(xnor) - K, the identity a population count uses
        ab, wb = oracle.pack_bits(a), oracle.pack_bits(w, transpose=True)
        pad = 32 * ab.shape[1] - K
        xnor = ~(ab[:, None, :] ^ wb[None, :, :])
        pop = np.array([[sum(bin(int(v)).count("1") for v in xnor[m, n]) for n in range(N)] for m in range(M)])
        assert np.array_equal(y, 2 * (pop - pad) - K)


def test_multi_sample_weight_gradient_follows_algorithm_1():
    g = np.random.default_rng(3)
    M, N, K = 24, 6, 10
    grad = (g.standard_normal((M, N)) * 1e-2).astype(np.float32)
    a = oracle.binarize(g.standard_normal((M, K)).astype(np.float32))
    for S in (1, 3):
        dw, acc = oracle.tern_wgrad_multi(grad, a, S, seed=50)
        ref = np.zeros((K, N), np.int64)
        for s in range(S):                                                  # the algorithm's loop, sample by sample
            t, scale = oracle.ternarize(grad, 50 + s)
            ref += a.astype(np.int64).T @ t.astype(np.int64)
        assert np.array_equal(acc, ref)
        assert np.array_equal(dw, (ref.astype(np.float64) * float(scale) / S).astype(np.float32))


def test_multi_sample_mean_converges_to_the_float_product_like_one_over_root_s():
    g = np.random.default_rng(4)
    M, N, K = 64, 8, 8
    grad = (g.standard_normal((M, N)) * 1e-2).astype(np.float32)
    a = oracle.binarize(g.standard_normal((M, K)).astype(np.float32))
    exact = a.astype(np.float64).T @ grad.astype(np.float64)

    def err(S):
        return np.mean([np.linalg.norm(oracle.tern_wgrad_multi(grad, a, S, seed=1000 * r)[0] - exact)
                        for r in range(8)])

    e1, e16, e256 = err(1), err(16), err(256)
    assert 2.5 < e1 / e16 < 6.5 and 2.5 < e16 / e256 < 6.5               # a factor of 4 per 16x samples
    assert e256 < 0.12 * e1
