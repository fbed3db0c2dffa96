"""Pins for the oracle's network plumbing (pooling behind the first Range BN + ReLU, residual add +
ReLU): against torch's CPU routines.  CPU only."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle


def _data(seed, shape):
    g = np.random.default_rng(seed)
    return g.standard_normal(shape).astype(np.float32)


def test_stem_pooling_forward_is_max_pool_of_the_rectified_normalization():
    for shape in ((2, 3, 8, 8), (1, 2, 7, 9), (2, 4, 12, 10)):
        x = _data(sum(shape), shape)
        stats = oracle.range_bn_stats(x)
        gamma, beta = _data(1, shape[1]), _data(2, shape[1])
        v, _, _ = oracle.range_bn_relu_fwd(x, stats, gamma, beta, 1e-5)
        out, idx = oracle.range_bn_relu_maxpool_fwd(x, stats, gamma, beta, 1e-5)
        ref = F.max_pool2d(torch.from_numpy(v), 3, 2, 1).numpy()
        assert np.array_equal(out, ref)
        # idx names a position that holds the maximum, or 255 where the maximum is not positive
        N, C, H, W = shape
        for n, c, p, q in np.ndindex(out.shape):
            k = int(idx[n, c, p, q])
            if out[n, c, p, q] <= 0:
                assert k == 255
            else:
                h, w = 2 * p - 1 + k // 3, 2 * q - 1 + k % 3
                assert 0 <= h < H and 0 <= w < W and v[n, c, h, w] == out[n, c, p, q]


def test_stem_pooling_backward_against_autograd():
    shape = (2, 3, 9, 10)
    x = _data(5, shape)
    stats = oracle.range_bn_stats(x)
    out, idx = oracle.range_bn_relu_maxpool_fwd(x, stats, None, None, 1e-5)
    g = _data(6, out.shape)
    dy = oracle.maxpool_relu_bwd(g, idx, shape[2], shape[3])
    y, _, _, _ = oracle.range_bn_fwd(x, eps=1e-5, stats=stats)        # before the rectifier
    t = torch.from_numpy(y).requires_grad_(True)
    F.max_pool2d(torch.relu(t), 3, 2, 1).backward(torch.from_numpy(g))
    assert np.allclose(dy, t.grad.numpy(), rtol=1e-6, atol=1e-7)     # continuous data: no ties among positive values


def test_add_relu_and_its_backward():
    a, b = _data(7, (3, 4, 5, 6)), _data(8, (3, 4, 5, 6))
    out, mx = oracle.add_relu(a, b)
    assert np.array_equal(out, np.maximum(a + b, 0)) and mx == out.max()
    g, o = _data(9, a.shape), _data(10, a.shape)
    assert np.array_equal(oracle.relu_bwd_add(g, out), np.where(out > 0, g, 0))
    assert np.array_equal(oracle.relu_bwd_add(g, out, o), np.where(out > 0, g, np.float32(0)) + o)
    # two consumers of a rectified tensor: the sum of their gradients, masked once (torch's own backward of
    # relu(t) feeding two branches)
    assert np.array_equal(oracle.relu_bwd_sum(g, o, out), np.where(out > 0, g + o, np.float32(0)))
    assert np.array_equal(oracle.relu_bwd_sum(g, o), g + o)
    assert np.array_equal(oracle.relu_bwd_sum(g, None, out), oracle.relu_bwd_add(g, out))
    t = torch.from_numpy(a + b).requires_grad_(True)
    r = torch.relu(t)
    (r * torch.from_numpy(g) + r * torch.from_numpy(o)).sum().backward()
    assert np.allclose(oracle.relu_bwd_sum(g, o, out), t.grad.numpy(), rtol=1e-6, atol=1e-7)
    z, mz = oracle.add_relu(-np.abs(a), -np.abs(b))
    assert not z.any() and mz == 0


@pytest.mark.parametrize("shape,stride", [((2, 3, 8, 12), 2), ((1, 2, 7, 9), 2), ((2, 2, 9, 10), 3), ((1, 1, 4, 4), 1)])
def test_sum_with_a_gradient_that_lives_on_a_lattice(shape, stride):
    # the gradient of a tensor that a 1x1 / stride-s convolution read: zero off the lattice.  Pinned against the
    # plain sum with the zero-filled tensor written out, and against torch's backward of x[..., ::s, ::s]
    N, Cc, H, W = shape
    g1, out = _data(31, shape), np.maximum(_data(32, shape), 0)
    sub = (N, Cc, (H + stride - 1) // stride, (W + stride - 1) // stride)
    g2s = _data(33, sub)
    full = np.zeros(shape, np.float32)
    full[:, :, ::stride, ::stride] = g2s
    got = oracle.relu_bwd_sum_lattice(g1, g2s, out, stride)
    assert np.array_equal(got, oracle.relu_bwd_sum(g1, full, out))
    assert np.array_equal(oracle.relu_bwd_sum_lattice(g1, g2s, None, stride), g1 + full)
    t = torch.from_numpy(_data(34, shape)).requires_grad_(True)
    r = torch.relu(t)
    ((r * torch.from_numpy(g1)).sum() + (r[:, :, ::stride, ::stride] * torch.from_numpy(g2s)).sum()).backward()
    mine = oracle.relu_bwd_sum_lattice(g1, g2s, r.detach().numpy(), stride)
    assert np.allclose(mine, t.grad.numpy(), rtol=1e-6, atol=1e-7)


def test_block_tail_in_one_pass_equals_its_pieces_and_torch():
    # relu(bn(x) + o): bit-identical to the separately pinned pieces (Range BN elementwise stage from given
    # statistics, then add + ReLU), and equal to the formula evaluated by torch in fp64 within fp32 rounding
    x, o = _data(31, (3, 4, 5, 6)), _data(32, (3, 4, 5, 6))
    g = np.random.default_rng(5)
    gamma, beta = g.uniform(-1.5, 1.5, 4).astype(np.float32), g.uniform(-0.5, 0.5, 4).astype(np.float32)
    og, ob = g.uniform(0.5, 1.5, 4).astype(np.float32), g.uniform(-0.5, 0.5, 4).astype(np.float32)
    eps = 1e-5
    st, so = oracle.range_bn_stats(x), oracle.range_bn_stats(o)
    bn, _, _, _ = oracle.range_bn_fwd(x, gamma, beta, eps, stats=st)
    out, mx = oracle.range_bn_add_relu(x, st, o, gamma, beta, eps=eps)
    ref, rmx = oracle.add_relu(bn, o)
    assert np.array_equal(out, ref) and mx == rmx == out.max()
    bno, _, _, _ = oracle.range_bn_fwd(o, og, ob, eps, stats=so)
    out2, mx2 = oracle.range_bn_add_relu(x, st, o, gamma, beta, so, og, ob, eps)
    ref2, _ = oracle.add_relu(bn, bno)
    assert np.array_equal(out2, ref2) and mx2 == out2.max()
    n = x.shape[0] * x.shape[2] * x.shape[3]
    cn = (2.0 * np.log(n)) ** -0.5

    def bn64(t, s, ga, be):
        t = torch.from_numpy(t).double()
        mu, mn, mxx = (torch.from_numpy(s[i]).double().view(1, -1, 1, 1) for i in range(3))
        return (t - mu) / (cn * (mxx - mn) + eps) * torch.from_numpy(ga).double().view(1, -1, 1, 1) + \
            torch.from_numpy(be).double().view(1, -1, 1, 1)
    t2 = torch.relu(bn64(x, st, gamma, beta) + bn64(o, so, og, ob)).numpy()
    assert np.allclose(out2, t2, rtol=1e-5, atol=1e-5)
    t1 = torch.relu(bn64(x, st, gamma, beta) + torch.from_numpy(o).double()).numpy()
    assert np.allclose(out, t1, rtol=1e-5, atol=1e-5)
