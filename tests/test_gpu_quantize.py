"""GPU parity: quantization calls vs the oracle, bit-exact codes and parameters."""
import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_util import same_ints, close, dev, host, require_gpu, same_qparams

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n", [0, 1, 3, 5, 1023, 4099, (1 << 20) + 7])
@pytest.mark.parametrize("bits", [2, 8, 16])
@pytest.mark.parametrize("stochastic", [False, True])
def test_quantize_matches_oracle(n, bits, stochastic):
    q8t = require_gpu()
    x = synth.normal(synth.rng(n + bits), (n,), std=1e-3 if stochastic else 2.0)
    q, qp = q8t.quantize(dev(x), bits, stochastic, seed=77 + n)
    s, _, oqp = oracle.quantize(x, bits, stochastic, seed=77 + n)
    same_qparams(q8t, qp, oqp)
    same_ints(host(q), s)


@pytest.mark.parametrize("bits", [4, 8, 12, 16])
def test_quantize_unaligned_pointer_and_seeds(bits):
    q8t = require_gpu()
    full = dev(synth.normal(synth.rng(3), (70001,), std=0.5))
    for off in (1, 2, 3):
        xs = full[off:]
        xh = host(xs)
        for seed in (0, 1, 2 ** 32 + 9, 0xDEADBEEFCAFEF00D):
            q, qp = q8t.quantize(xs, bits, True, seed=seed)
            s, _, oqp = oracle.quantize(xh, bits, True, seed=seed)
            same_qparams(q8t, qp, oqp)
            same_ints(host(q), s)


def test_quantize_special_ranges():
    q8t = require_gpu()
    cases = [np.zeros(100, np.float32), np.full(100, 3.5, np.float32), -np.arange(1, 300, dtype=np.float32),
             np.arange(-51, 205, dtype=np.float32), np.array([1e-30, 2e-30], np.float32),
             np.array([-3e38, 3e38], np.float32) * np.float32(0.5)]
    for x in cases:
        for stochastic in (False, True):
            q, qp = q8t.quantize(dev(x), 8, stochastic, seed=5)
            s, _, oqp = oracle.quantize(x, 8, stochastic, seed=5)
            same_qparams(q8t, qp, oqp)
            same_ints(host(q), s)


@pytest.mark.parametrize("bits", [8, 16])
def test_quantize_with_supplied_range_saturates(bits):
    q8t = require_gpu()
    x = synth.normal(synth.rng(1), (50003,), std=2.0)
    x[:4] = [-1e30, 1e30, 3e9, -3e9]
    rng = np.array([-1.0, 2.0], np.float32)
    for stochastic in (False, True):
        q, qp = q8t.quantize_with_range(dev(x), dev(rng), bits, stochastic, seed=8)
        s, _, oqp = oracle.quantize(x, bits, stochastic, seed=8, vrange=(-1.0, 2.0))
        same_qparams(q8t, qp, oqp)
        same_ints(host(q), s)


@pytest.mark.parametrize("n", [6, 4096 + 3, 1 << 21])
def test_bifurcated_gradient_copies(n):
    q8t = require_gpu()
    g = synth.normal(synth.rng(n), (n,), std=1e-3)
    q8, qp8, q16, qp16 = q8t.quantize_bifurcate(dev(g), seed8=123, seed16=2 ** 33 + 456)
    s8, _, o8 = oracle.quantize(g, 8, True, seed=123)
    s16, _, o16 = oracle.quantize(g, 16, True, seed=2 ** 33 + 456)
    same_qparams(q8t, qp8, o8)
    same_qparams(q8t, qp16, o16)
    same_ints(host(q8), s8)
    same_ints(host(q16), s16)
    # both copies dequantize back to g within one step of their own grid
    close(host(q8t.dequantize(q16, qp16)), oracle.dequantize(s16, o16))
    close(host(q8t.dequantize(q8, qp8)), oracle.dequantize(s8, o8))


def test_full_size_activation_tensor():
    # the 128x64x56x56 tensor of configs 1-3, in the launch configuration the benchmark times
    q8t = require_gpu()
    x, _, dy = synth.conv_layer(seed=0)
    q, qp = q8t.quantize(dev(x), 8)
    s, _, oqp = oracle.quantize(x, 8)
    same_qparams(q8t, qp, oqp)
    same_ints(host(q), s)
    q8, qp8, q16, qp16 = q8t.quantize_bifurcate(dev(dy), seed8=1, seed16=2)
    s8, _, o8 = oracle.quantize(dy, 8, True, seed=1)
    s16, _, o16 = oracle.quantize(dy, 16, True, seed=2)
    same_qparams(q8t, qp8, o8)
    same_qparams(q8t, qp16, o16)
    same_ints(host(q8), s8)
    same_ints(host(q16), s16)


def test_error_codes_on_device_arguments():
    q8t = require_gpu()
    x = dev(np.ones(8, np.float32))
    with pytest.raises(q8t.binding.Q8TError) as e:
        q8t.quantize(x, 17)
    assert e.value.code == -3
    with pytest.raises(ValueError):
        q8t.quantize(torch.ones(8), 8)


def test_several_tensors_in_one_call_each_with_its_own_range():
    # weights of a network: sizes from a few elements to several workgroups, a count above one launch's table,
    # a tensor whose storage is not 16-byte aligned; every result equals the single-tensor call and the oracle
    q8t = require_gpu()
    import torch
    g = synth.rng(77)
    sizes = [1, 3, 7, 16384, 16385, 36864, 70001, 147456, 5, 64 * 3 * 49] + [257 + 13 * i for i in range(30)]
    host_t = [(g.standard_normal(n) * g.uniform(0.01, 3.0) + g.uniform(-1, 1)).astype(np.float32) for n in sizes]
    dev_t = [dev(t) for t in host_t]
    odd = dev(np.concatenate([np.zeros(1, np.float32), host_t[6]]))[1:]     # same values, storage shifted by 4 bytes
    assert odd.data_ptr() % 16 != 0
    dev_t.append(odd)
    host_t.append(host_t[6])
    res = q8t.quantize_multi(dev_t, 8)
    for t, (q, qp), d in zip(host_t, res, dev_t):
        oq, _, oqp = oracle.quantize(t, 8)
        same_qparams(q8t, qp, oqp)
        same_ints(host(q), oq)
        q1, qp1 = q8t.quantize(d.contiguous(), 8)
        assert torch.equal(q1, q)
    res5 = q8t.quantize_multi(dev_t[:4], 5)
    for t, (q, qp) in zip(host_t, res5):
        oq, _, oqp = oracle.quantize(t, 5)
        same_qparams(q8t, qp, oqp)
        same_ints(host(q), oq)
