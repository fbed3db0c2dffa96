"""GPU parity: stochastic ternarization, binarization, bit rows, the XNOR + population count product
and the multi-sample weight gradient of Algorithm 1 (appendix "Additional Experiments")."""
import numpy as np
import pytest

import oracle
import synth
from gpu_util import close, dev, host, require_gpu, same_ints

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n", [0, 1, 5, 4099, 1 << 20, (1 << 22) + 3])
def test_ternarize_matches_oracle(n):
    q8t = require_gpu()
    g = synth.normal(synth.rng(n), (n,), std=1e-3)
    for seed in (0, 0xDEADBEEFCAFEF00D):
        t, s = q8t.ternarize(dev(g), seed)
        ot, os_ = oracle.ternarize(g, seed)
        assert np.float32(host(s)[0]) == os_
        same_ints(host(t), ot)


def test_ternarize_all_zero_and_single_spike():
    q8t = require_gpu()
    z = np.zeros(1000, np.float32)
    t, s = q8t.ternarize(dev(z), 1)
    assert float(host(s)[0]) == 0.0 and not host(t).any()
    z[333] = -7.0
    t, s = q8t.ternarize(dev(z), 1)
    ot, os_ = oracle.ternarize(z, 1)
    assert float(host(s)[0]) == 7.0 and host(t)[333] == -1
    same_ints(host(t), ot)


@pytest.mark.parametrize("shape", [(1, 1), (7, 70), (64, 256), (33, 1000), (256, 512)])
def test_binarize_and_bit_rows_match_oracle(shape):
    q8t = require_gpu()
    x = synth.normal(synth.rng(sum(shape)), shape, std=1.0)
    x.flat[::7] = 0.0
    x.flat[3::11] = -0.0
    b = q8t.binarize(dev(x))
    ob = oracle.binarize(x)
    same_ints(host(b), ob)
    for tr in (False, True):
        bits = q8t.pack_bits(b, transpose=tr)
        same_ints(host(bits).view(np.uint32), oracle.pack_bits(ob, transpose=tr))


@pytest.mark.parametrize("mnk", [(1, 1, 1), (5, 4, 7), (64, 128, 256), (70, 65, 100), (256, 1000, 512), (130, 3, 2049)])
def test_xnor_product_matches_oracle(mnk):
    q8t = require_gpu()
    M, N, K = mnk
    g = synth.rng(M + N + K)
    a = oracle.binarize(synth.normal(g, (M, K), std=1.0))
    w = oracle.binarize(synth.normal(g, (K, N), std=1.0))
    ab = q8t.pack_bits(dev(a))
    wb = q8t.pack_bits(dev(w), transpose=True)
    y = q8t.xnor_gemm(ab, wb, K)
    oy = oracle.xnor_gemm(oracle.pack_bits(a), oracle.pack_bits(w, transpose=True), K)
    same_ints(host(y), oy)


@pytest.mark.parametrize("case", [(1, 1, 1, 1), (24, 6, 10, 3), (64, 128, 256, 1), (100, 70, 130, 5), (256, 1000, 512, 2),
                                  (200, 64, 64, 12)])
def test_multi_sample_weight_gradient_matches_oracle(case):
    q8t = require_gpu()
    M, N, K, S = case
    g = synth.rng(sum(case))
    grad = synth.normal(g, (M, N), std=1e-2)
    a = oracle.binarize(synth.normal(g, (M, K), std=1.0))
    seed = (1 << 32) - 2                       # the per-sample seeds cross a 32-bit boundary
    dw, acc = q8t.tern_wgrad_multi(dev(grad), dev(a), S, seed=seed, want_acc=True)
    odw, oacc = oracle.tern_wgrad_multi(grad, a, S, seed=seed)
    same_ints(host(acc), oacc)
    close(host(dw), odw)
    dw2, _ = q8t.tern_wgrad_multi(dev(grad), dev(a), S, seed=seed, want_acc=False)
    assert np.array_equal(host(dw), host(dw2))
