"""Helpers shared by the GPU parity tests."""
import numpy as np
import pytest
import torch

RTOL, ATOL = 1e-5, 1e-6   # float tolerance stated by the target: 1e-5 relative / 1e-6 absolute


def require_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_1805_11046_amd as q8t
    return q8t


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def host(t):
    return None if t is None else t.cpu().numpy()


def same_qparams(q8t, qp_dev, oqp):
    got = q8t.qparams_to_host(qp_dev)
    exp = oqp.as_tuple()
    assert got == tuple(float(np.float32(v)) if i < 4 else v for i, v in enumerate(exp)), (got, exp)


def qp_dev_from(oqp):
    """device q8t_qparams holding an oracle QParams (for feeding the product calls)"""
    f = np.array([oqp.vmin, oqp.vmax, oqp.scale, oqp.inv_scale], np.float32).view(np.int32)
    i = np.array([oqp.zero_point, oqp.bits], np.int32)
    return dev(np.concatenate([f, i]))


def close(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    bad = np.abs(a - b) > ATOL + RTOL * np.abs(b)
    assert not bad.any(), "%d of %d outside tolerance, max abs diff %g" % (bad.sum(), bad.size, np.abs(a - b).max())


def same_ints(got, exp):
    """bit-exact comparison with a short failure message"""
    got = np.asarray(got)
    exp = np.asarray(exp)
    assert got.shape == exp.shape, (got.shape, exp.shape)
    bad = got != exp   # exact comparison (integers; floats value by value)
    if bad.any():
        idx = tuple(int(v) for v in np.argwhere(bad)[0])
        raise AssertionError("%d of %d values differ; first at %s: got %r, expected %r"
                             % (bad.sum(), bad.size, idx, got[idx], exp[idx]))
