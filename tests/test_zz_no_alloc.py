"""GPU: the allocation-free entry point q8t_quantize_noalloc against q8t_quantize (same kernels, the
partial results in the library's static device array instead of a caller workspace)."""
import pytest
import torch

from gpu_util import require_gpu

pytestmark = pytest.mark.gpu


def _pair(q8t, x, bits, stochastic, seed):
    dt = torch.int8 if bits <= 8 else torch.int16
    ref_q, ref_p = q8t.quantize(x, bits, stochastic=stochastic, seed=seed)
    # every buffer of the new call exists before it is made; the fill shows stale output as a mismatch
    q = torch.full(x.shape, 77, dtype=dt, device=x.device)
    p = torch.full((6,), -1, dtype=torch.int32, device=x.device)
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    q8t.quantize_noalloc(x, q, p, bits, stochastic=stochastic, seed=seed)
    after = torch.cuda.memory_stats()["allocation.all.allocated"]
    torch.cuda.synchronize()
    assert before == after                      # the binding allocated nothing through torch either
    assert torch.equal(p, ref_p), (p, ref_p)    # range, scale, zero point: bit for bit
    assert torch.equal(q, ref_q)


def test_two_calls_in_a_row_the_second_smaller():
    q8t = require_gpu()
    q8t.init()
    g = torch.Generator(device="cuda:0").manual_seed(5)
    # 3 000 007 elements: ragged tail, several hundred partial results in the scratch array
    big = torch.randn(3000007, generator=g, device="cuda:0") * 3.0 + 1.0
    # 200 003 elements with a narrower range: fewer partial results, so the scratch still holds pairs of
    # the first call beyond the ones this call writes; none of them may leak into its range
    small = torch.randn(200003, generator=g, device="cuda:0") * 0.01
    _pair(q8t, big, 8, False, 0)
    _pair(q8t, small, 8, False, 0)
    _pair(q8t, big, 16, True, 0x1234567890ABCDEF)
    _pair(q8t, small, 5, True, 3)


def test_sizes_that_bypass_or_empty_the_scratch():
    q8t = require_gpu()
    g = torch.Generator(device="cuda:0").manual_seed(6)
    for n in (0, 1, 65536, 65537):
        x = torch.randn(n, generator=g, device="cuda:0")
        _pair(q8t, x, 8, False, 0)
        _pair(q8t, x, 8, True, 9)


def test_size_beyond_the_maximum_is_rejected():
    q8t = require_gpu()
    x = torch.zeros(16, device="cuda:0")
    q = torch.zeros(16, dtype=torch.int8, device="cuda:0")
    p = torch.zeros(6, dtype=torch.int32, device="cuda:0")
    rc = q8t.binding._lib.q8t_quantize_noalloc(x.data_ptr(), (1 << 34) + 1, 8, 0, 0, q.data_ptr(), p.data_ptr(), None)
    assert rc == -2
