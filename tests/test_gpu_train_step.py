"""The chained training step (paper_1805_11046_amd.train_step): the fused node structure (stem pooling inside the
Range BN pass, whole residual blocks as one node with the masked gradient sum, codes handed from layer to layer)
must give what the plain structure gives (every Range BN, ReLU, pooling, sum and quantization its own pass, torch's
autograd for the glue): same loss, same weight gradients.  Both run the same library products; a layer's stochastic
roundings are seeded by its position in the network, so the two structures draw the same random numbers."""
import pytest

from gpu_util import require_gpu

pytestmark = pytest.mark.gpu


def test_fused_and_plain_resnet18_steps_agree():
    require_gpu()
    import torch
    from paper_1805_11046_amd import train_step as ts
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(5)
    ws = ts.make_weights(dev, gen)
    x = torch.randn((4, 3, 224, 224), device=dev, generator=gen)
    labels = torch.randint(0, 1000, (4,), device=dev, generator=gen)
    params = [ws["conv1"], ws["fc"]] + [w for b in ws["blocks"] for w in b.values()]
    results = []
    for fuse in (True, False):
        ts._fuse = fuse
        for p in params:
            p.grad = None
        loss = ts.step(x, labels, ws)
        torch.cuda.synchronize()
        results.append((float(loss.detach()), [p.grad.clone() for p in params]))
    ts._fuse = True
    (lf, gf), (lp, gp) = results
    assert lf == lp
    for i, (a, b) in enumerate(zip(gf, gp)):
        assert torch.equal(a, b), "gradient of parameter %d differs: max |diff| %g" % (i, float((a - b).abs().max()))


def test_steps_leave_no_memory_behind():
    # the nodes of a step must not keep each other alive (a node that saves its own output would, until the cycle
    # collector happens to run): allocated device memory is the same after every step
    require_gpu()
    import gc
    import torch
    from paper_1805_11046_amd import train_step as ts
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(6)
    ws = ts.make_weights(dev, gen)
    x = torch.randn((2, 3, 224, 224), device=dev, generator=gen)
    labels = torch.randint(0, 1000, (2,), device=dev, generator=gen)
    params = [ws["conv1"], ws["fc"]] + [w for b in ws["blocks"] for w in b.values()]
    gc.collect()
    gc.disable()
    try:
        seen = []
        for _ in range(4):
            for p in params:
                p.grad = None
            ts.step(x, labels, ws)
            torch.cuda.synchronize()
            seen.append(torch.cuda.memory_allocated())
    finally:
        gc.enable()
    assert seen[1] == seen[2] == seen[3], seen


def test_weight_gradients_on_a_second_stream_change_nothing():
    require_gpu()
    import torch
    from paper_1805_11046_amd import train_step as ts
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    ws = ts.make_weights(dev, gen)
    x = torch.randn((4, 3, 224, 224), device=dev, generator=gen)
    labels = torch.randint(0, 1000, (4,), device=dev, generator=gen)
    params = [ws["conv1"], ws["fc"]] + [w for b in ws["blocks"] for w in b.values()]
    results = []
    try:
        for overlap in (False, True, True):
            ts._overlap = overlap
            for p in params:
                p.grad = None
            loss = ts.step(x, labels, ws)
            torch.cuda.synchronize()
            results.append((float(loss.detach()), [p.grad.clone() for p in params]))
    finally:
        ts._overlap = False
    for lo, go in results[1:]:
        assert lo == results[0][0]
        for i, (a, b) in enumerate(zip(results[0][1], go)):
            assert torch.equal(a, b), "gradient of parameter %d differs" % i


def test_filters_packed_in_one_launch_change_nothing():
    # the step with every filter packed ahead by one launch against the step whose products pack their own
    require_gpu()
    import torch
    from paper_1805_11046_amd import train_step as ts
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(11)
    ws = ts.make_weights(dev, gen)
    x = torch.randn((4, 3, 224, 224), device=dev, generator=gen)
    labels = torch.randint(0, 1000, (4,), device=dev, generator=gen)
    params = [ws["conv1"], ws["fc"]] + [w for b in ws["blocks"] for w in b.values()]
    results = []
    try:
        for pack in (False, True, True):
            ts._pack = pack
            for p in params:
                p.grad = None
            loss = ts.step(x, labels, ws)
            torch.cuda.synchronize()
            results.append((float(loss.detach()), [p.grad.clone() for p in params]))
            if pack:
                assert len(ts._pcache) >= 30      # most layers have a packed form in both directions
            else:
                assert len(ts._pcache) == 0
    finally:
        ts._pack = False
    for lo, go in results[1:]:
        assert lo == results[0][0]
        for i, (a, b) in enumerate(zip(results[0][1], go)):
            assert torch.equal(a, b), "gradient of parameter %d differs" % i
