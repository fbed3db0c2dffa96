"""GPU parity at the full sizes of the workloads, in the launch configuration the benchmark times.

Forward and layer-gradient outputs of image n depend on image n only, so the oracle computes a
sample of images one by one; the weight gradient reduces over the whole batch and is compared in
full.  A second test chains the calls of one layer step and checks every stage against the oracle
run on the GPU's own intermediates (bit-exact integers stage by stage)."""
import numpy as np
import pytest

import oracle
import synth
from gpu_util import close, dev, host, require_gpu, same_ints, same_qparams

pytestmark = pytest.mark.gpu


def _sub_desc(case, n):
    c = list(case)
    c[0] = n
    return oracle.conv_desc(*c)


def _check_conv_layer(q8t, case, seed, sample, check_dgrad=True):
    N, C, H, W, K, R, S, st, pad = case
    # the network's input is N(0,1); every other layer sees rectified activations
    x, w, dy = synth.conv_layer(seed=seed, N=N, C=C, H=H, W=W, K=K, R=R, S=S, stride=st, pad=pad, relu_input=C != 3)
    d = q8t.conv_desc(*case)
    qx, px = q8t.quantize(dev(x), 8)
    qw, pw = q8t.quantize(dev(w), 8)
    g8, pg8, g16, pg16 = q8t.quantize_bifurcate(dev(dy), seed8=21, seed16=22)
    sx, _, opx = oracle.quantize(x, 8)
    sw, _, opw = oracle.quantize(w, 8)
    s8, _, o8 = oracle.quantize(dy, 8, True, seed=21)
    s16, _, o16 = oracle.quantize(dy, 16, True, seed=22)
    del x, dy
    same_qparams(q8t, px, opx)
    same_qparams(q8t, pw, opw)
    same_qparams(q8t, pg8, o8)
    same_qparams(q8t, pg16, o16)
    same_ints(host(qx), sx)
    same_ints(host(g8), s8)
    same_ints(host(g16), s16)
    d1 = _sub_desc(case, 1)
    y, acc = q8t.qconv_fwd(d, qx, px, qw, pw, want_acc=True)
    for n in sample:
        oy, oacc = oracle.qconv_fwd(d1, sx[n:n + 1], opx, sw, opw)
        same_ints(host(acc[n:n + 1]), oacc)
        close(host(y[n:n + 1]), oy)
    del y, acc
    if check_dgrad:
        dx, accd = q8t.qconv_dgrad(d, g8, pg8, qw, pw, want_acc=True)
        for n in sample:
            odx, oaccd = oracle.qconv_dgrad(d1, s8[n:n + 1], o8, sw, opw)
            same_ints(host(accd[n:n + 1]), oaccd)
            close(host(dx[n:n + 1]), odx)
        del dx, accd
    # the weight gradient reduces over the whole batch: compared in full, always
    dw, accw = q8t.qconv_wgrad(d, qx, px, g16, pg16, want_acc=True)
    odw, oaccw = oracle.qconv_wgrad(oracle.conv_desc(*case), sx, opx, s16, o16)
    same_ints(host(accw), oaccw)
    close(host(dw), odw)


def test_config2_conv3x3_full_size():
    q8t = require_gpu()
    _check_conv_layer(q8t, (128, 64, 56, 56, 64, 3, 3, 1, 1), seed=0, sample=(0, 77, 127))


def test_config3_bottleneck_convs_full_size():
    q8t = require_gpu()
    _check_conv_layer(q8t, (128, 256, 56, 56, 64, 1, 1, 1, 0), seed=1, sample=(0, 127))
    _check_conv_layer(q8t, (128, 64, 56, 56, 256, 1, 1, 1, 0), seed=2, sample=(5, 126))


# every distinct convolution of ResNet-18 at batch 256 (the persistent row schedules, image splits and
# reduction slices of the kernels depend on the batch, so the batch is the real one)
RESNET18_B256 = [
    (256, 64, 56, 56, 64, 3, 3, 1, 1),
    (256, 128, 28, 28, 128, 3, 3, 1, 1),
    (256, 256, 14, 14, 256, 3, 3, 1, 1),
    (256, 512, 7, 7, 512, 3, 3, 1, 1),
    (256, 64, 56, 56, 128, 3, 3, 2, 1),
    (256, 128, 28, 28, 256, 3, 3, 2, 1),
    (256, 256, 14, 14, 512, 3, 3, 2, 1),
    (256, 64, 56, 56, 128, 1, 1, 2, 0),
    (256, 128, 28, 28, 256, 1, 1, 2, 0),
    (256, 256, 14, 14, 512, 1, 1, 2, 0),
]


@pytest.mark.parametrize("case", RESNET18_B256)
def test_config4_layer_shapes(case):
    q8t = require_gpu()
    _check_conv_layer(q8t, case, seed=3, sample=(0, 131, case[0] - 1))


def test_config4_first_layer_full_batch():
    # 7x7 stride 2, 3 -> 64 channels on 224x224 at batch 256: forward on sampled images, the weight
    # gradient (reduction over 256*112*112 positions) in full.  The input of the network has no
    # gradient, so the layer gradient of this layer is not part of a training step; it is checked at
    # batch 16 below.
    q8t = require_gpu()
    _check_conv_layer(q8t, (256, 3, 224, 224, 64, 7, 7, 2, 3), seed=3, sample=(0, 255), check_dgrad=False)


def test_config4_first_layer_gradient_to_the_input():
    q8t = require_gpu()
    _check_conv_layer(q8t, (16, 3, 224, 224, 64, 7, 7, 2, 3), seed=3, sample=(0, 15))


def test_config4_fc_layer_full_batch():
    # the classifier: 256 x 512 -> 1000, all three products in full
    q8t = require_gpu()
    g = synth.rng(9)
    x = np.abs(synth.normal(g, (256, 512), std=1.0))
    w = synth.normal(g, (512, 1000), std=(2.0 / 512) ** 0.5)
    dy = synth.normal(g, (256, 1000), std=1e-3)
    qx, px = q8t.quantize(dev(x), 8)
    qw, pw = q8t.quantize(dev(w), 8)
    g8, pg8, g16, pg16 = q8t.quantize_bifurcate(dev(dy), seed8=5, seed16=6)
    sx, _, opx = oracle.quantize(x, 8)
    sw, _, opw = oracle.quantize(w, 8)
    s8, _, o8 = oracle.quantize(dy, 8, True, seed=5)
    s16, _, o16 = oracle.quantize(dy, 16, True, seed=6)
    same_ints(host(qx), sx)
    same_ints(host(qw), sw)
    same_ints(host(g8), s8)
    same_ints(host(g16), s16)
    y, acc = q8t.qgemm_fwd(qx, px, qw, pw, want_acc=True)
    oy, oacc = oracle.qgemm_fwd(sx, opx, sw, opw)
    same_ints(host(acc), oacc)
    close(host(y), oy)
    dx, accd = q8t.qgemm_dgrad(g8, pg8, qw, pw, want_acc=True)
    odx, oaccd = oracle.qgemm_dgrad(s8, o8, sw, opw)
    same_ints(host(accd), oaccd)
    close(host(dx), odx)
    dw, accw = q8t.qgemm_wgrad(qx, px, g16, pg16, want_acc=True)
    odw, oaccw = oracle.qgemm_wgrad(sx, opx, s16, o16)
    same_ints(host(accw), oaccw)
    close(host(dw), odw)


def test_layer_step_chain_stage_by_stage():
    # quantize -> conv fwd -> Range BN fwd -> Range BN bwd -> bifurcated quantization -> dgrad, wgrad.
    # Every stage is checked against the oracle fed with the GPU's output of the stage before.
    q8t = require_gpu()
    case = (4, 64, 56, 56, 64, 3, 3, 1, 1)
    x, w, _ = synth.conv_layer(seed=5, N=4)
    dout = synth.normal(synth.rng(6), (4, 64, 56, 56), std=1e-2)
    d, od = q8t.conv_desc(*case), oracle.conv_desc(*case)
    qx, px = q8t.quantize(dev(x), 8)
    qw, pw = q8t.quantize(dev(w), 8)
    y, acc = q8t.qconv_fwd(d, qx, px, qw, pw, want_acc=True)
    bn, stats, _, _ = q8t.range_bn_fwd(y, eps=1e-5)
    g, dgam, dbet = q8t.range_bn_bwd(y, dev(dout), stats, None, 1e-5)
    g8, pg8, g16, pg16 = q8t.quantize_bifurcate(g, seed8=31, seed16=32)
    dx, accd = q8t.qconv_dgrad(d, g8, pg8, qw, pw, want_acc=True)
    dw, accw = q8t.qconv_wgrad(d, qx, px, g16, pg16, want_acc=True)

    sx, _, opx = oracle.quantize(x, 8)
    sw, _, opw = oracle.quantize(w, 8)
    same_ints(host(qx), sx)
    same_ints(host(qw), sw)
    oy, oacc = oracle.qconv_fwd(od, sx, opx, sw, opw)
    same_ints(host(acc), oacc)
    close(host(y), oy)
    yh, sth = host(y), host(stats)
    obn, ost, _, _ = oracle.range_bn_fwd(yh, eps=1e-5)
    assert np.array_equal(sth[1:], ost[1:])
    close(sth[0], ost[0])
    fbn, _, _, _ = oracle.range_bn_fwd(yh, eps=1e-5, stats=sth)
    same_ints(host(bn), fbn)
    og, odg, odb = oracle.range_bn_bwd(yh, dout, sth, None, 1e-5)
    close(host(g), og)
    close(host(dgam), odg)
    close(host(dbet), odb)
    gh = host(g)
    s8, _, o8 = oracle.quantize(gh, 8, True, seed=31)
    s16, _, o16 = oracle.quantize(gh, 16, True, seed=32)
    same_qparams(q8t, pg8, o8)
    same_qparams(q8t, pg16, o16)
    same_ints(host(g8), s8)
    same_ints(host(g16), s16)
    odx, oaccd = oracle.qconv_dgrad(od, s8, o8, sw, opw)
    same_ints(host(accd), oaccd)
    close(host(dx), odx)
    odw, oaccw = oracle.qconv_wgrad(od, sx, opx, s16, o16)
    same_ints(host(accw), oaccw)
    close(host(dw), odw)
    # un-forced end-to-end run of the oracle from the same inputs: the 8-bit gradient codes may
    # differ in a handful of places (the fp64 sums of the BN backward are taken in another order)
    g_or, _, _ = oracle.range_bn_bwd(oy, dout, oracle.range_bn_stats(oy), None, 1e-5)
    s8_free, _, _ = oracle.quantize(g_or, 8, True, seed=31)
    diff = int((s8_free != host(g8)).sum())
    print("8-bit gradient codes differing from the un-forced oracle chain:", diff, "of", s8_free.size)
    assert diff <= 1e-4 * s8_free.size


def _layer_forward(q8t, od, d, a_dev, w, tag):
    """quantize -> conv (+ Range BN statistics from its epilogue) -> Range BN; every stage against
    the oracle fed with the GPU's output of the stage before.  Returns what the backward needs."""
    ah = host(a_dev)
    qa, pa = q8t.quantize(a_dev, 8)
    qw, pw = q8t.quantize(dev(w), 8)
    sa, _, opa = oracle.quantize(ah, 8)
    sw, _, opw = oracle.quantize(w, 8)
    same_qparams(q8t, pa, opa)
    same_ints(host(qa), sa)
    same_ints(host(qw), sw)
    y, acc, stats = q8t.qconv_fwd_bn_stats(d, qa, pa, qw, pw, want_acc=True)
    oy, oacc = oracle.qconv_fwd(od, sa, opa, sw, opw)
    same_ints(host(acc), oacc)
    close(host(y), oy)
    yh, sth = host(y), host(stats)
    ost = oracle.range_bn_stats(yh)
    assert np.array_equal(sth[1:], ost[1:]), tag
    close(sth[0], ost[0])
    bn, _, _ = q8t.range_bn_fwd_apply(y, stats, eps=1e-5)
    obn, _, _, _ = oracle.range_bn_fwd(yh, eps=1e-5, stats=sth)
    same_ints(host(bn), obn)
    return dict(qa=qa, pa=pa, qw=qw, pw=pw, sa=sa, opa=opa, sw=sw, opw=opw, y=y, yh=yh, stats=stats, sth=sth, bn=bn)


def _layer_backward(q8t, od, d, L, dbn_dev, seed):
    """Range BN backward fused with the bifurcated quantization -> layer and weight gradients."""
    dbn = host(dbn_dev)
    g, dgam, dbet, g8, pg8, g16, pg16 = q8t.range_bn_bwd_bifurcate(L["y"], dbn_dev, L["stats"], None, 1e-5, seed, seed + 1)
    og, odg, odb = oracle.range_bn_bwd(L["yh"], dbn, L["sth"], None, 1e-5)
    close(host(g), og)
    close(host(dgam), odg)
    close(host(dbet), odb)
    gh = host(g)
    s8, _, o8 = oracle.quantize(gh, 8, True, seed=seed)
    s16, _, o16 = oracle.quantize(gh, 16, True, seed=seed + 1)
    same_qparams(q8t, pg8, o8)
    same_qparams(q8t, pg16, o16)
    same_ints(host(g8), s8)
    same_ints(host(g16), s16)
    dx, accd = q8t.qconv_dgrad(d, g8, pg8, L["qw"], L["pw"], want_acc=True)
    odx, oaccd = oracle.qconv_dgrad(od, s8, o8, L["sw"], L["opw"])
    same_ints(host(accd), oaccd)
    close(host(dx), odx)
    dw, accw = q8t.qconv_wgrad(d, L["qa"], L["pa"], g16, pg16, want_acc=True)
    odw, oaccw = oracle.qconv_wgrad(od, L["sa"], L["opa"], s16, o16)
    same_ints(host(accw), oaccw)
    close(host(dw), odw)
    return dx


def test_config3_bottleneck_block_forward_and_backward_chain():
    # 1x1 256->64, 3x3 64->64, 1x1 64->256 at 56x56, Range BN + ReLU after each (ReLU and its mask are
    # plain elementwise glue outside the method, done with torch on the device), batch 4.
    import torch
    q8t = require_gpu()
    N = 4
    x, (w1, w2, w3), dout = synth.bottleneck_block(seed=4, N=N)
    cases = [(N, 256, 56, 56, 64, 1, 1, 1, 0), (N, 64, 56, 56, 64, 3, 3, 1, 1), (N, 64, 56, 56, 256, 1, 1, 1, 0)]
    ds = [q8t.conv_desc(*c) for c in cases]
    ods = [oracle.conv_desc(*c) for c in cases]
    a = dev(x)
    layers = []
    for i, w in enumerate((w1, w2, w3)):
        L = _layer_forward(q8t, ods[i], ds[i], a, w, "layer %d" % i)
        layers.append(L)
        a = torch.relu(L["bn"])
    grad = dev(dout)
    for i in (2, 1, 0):
        L = layers[i]
        dbn = grad * (L["bn"] > 0).to(grad.dtype)       # ReLU backward
        grad = _layer_backward(q8t, ods[i], ds[i], L, dbn.contiguous(), seed=100 + 10 * i)
    assert tuple(grad.shape) == x.shape and bool(torch.isfinite(grad).all())


def test_config4_resnet18_training_step_chain():
    # Full ResNet-18 forward + backward at batch 2 (the oracle re-runs every call of the method on the
    # GPU's own inputs to that call: stage-by-stage bit-exact integers, floats within tolerance).
    # Every conv / FC product and every BN is the library's; ReLU, pooling, the residual adds and the
    # softmax cross-entropy are elementwise glue outside the method and are left to torch autograd.
    import torch
    import torch.nn.functional as F
    q8t = require_gpu()
    N = 2
    g = synth.rng(44)
    x = synth.normal(g, (N, 3, 224, 224), std=1.0)
    labels = torch.as_tensor(g.integers(0, 1000, size=N), device="cuda:0")
    state = {"seed": 1000, "n": 0}

    def he(cout, cin, r):
        return synth.normal(g, (cout, cin, r, r), std=(2.0 / (cin * r * r)) ** 0.5)

    class ConvBN(torch.autograd.Function):
        @staticmethod
        def forward(ctx, a, w_np, stride, pad):
            a = a.contiguous()
            n, c, h, wd = a.shape
            k, _, r, s = w_np.shape
            case = (n, c, h, wd, k, r, s, stride, pad)
            ctx.d, ctx.od = q8t.conv_desc(*case), oracle.conv_desc(*case)
            ctx.L = _layer_forward(q8t, ctx.od, ctx.d, a, w_np, str(case))
            state["n"] += 1
            return ctx.L["bn"]

        @staticmethod
        def backward(ctx, dbn):
            state["seed"] += 2
            dx = _layer_backward(q8t, ctx.od, ctx.d, ctx.L, dbn.contiguous(), seed=state["seed"])
            return dx, None, None, None

    class Linear(torch.autograd.Function):
        @staticmethod
        def forward(ctx, a, w_np):
            a = a.contiguous()
            ah = host(a)
            qa, pa = q8t.quantize(a, 8)
            qw, pw = q8t.quantize(dev(w_np), 8)
            sa, _, opa = oracle.quantize(ah, 8)
            sw, _, opw = oracle.quantize(w_np, 8)
            same_ints(host(qa), sa)
            same_ints(host(qw), sw)
            y, acc = q8t.qgemm_fwd(qa, pa, qw, pw, want_acc=True)
            oy, oacc = oracle.qgemm_fwd(sa, opa, sw, opw)
            same_ints(host(acc), oacc)
            close(host(y), oy)
            ctx.saved = (qa, pa, qw, pw, sa, opa, sw, opw)
            return y

        @staticmethod
        def backward(ctx, dy):
            qa, pa, qw, pw, sa, opa, sw, opw = ctx.saved
            dy = dy.contiguous()
            dyh = host(dy)
            g8, pg8, g16, pg16 = q8t.quantize_bifurcate(dy, 7, 8)
            s8, _, o8 = oracle.quantize(dyh, 8, True, seed=7)
            s16, _, o16 = oracle.quantize(dyh, 16, True, seed=8)
            same_ints(host(g8), s8)
            same_ints(host(g16), s16)
            dx, accd = q8t.qgemm_dgrad(g8, pg8, qw, pw, want_acc=True)
            odx, oaccd = oracle.qgemm_dgrad(s8, o8, sw, opw)
            same_ints(host(accd), oaccd)
            close(host(dx), odx)
            dw, accw = q8t.qgemm_wgrad(qa, pa, g16, pg16, want_acc=True)
            odw, oaccw = oracle.qgemm_wgrad(sa, opa, s16, o16)
            same_ints(host(accw), oaccw)
            close(host(dw), odw)
            return dx, None

    def block(a, cin, cout, stride):
        h = F.relu(ConvBN.apply(a, he(cout, cin, 3), stride, 1))
        h = ConvBN.apply(h, he(cout, cout, 3), 1, 1)
        sc = a if (stride == 1 and cin == cout) else ConvBN.apply(a, he(cout, cin, 1), stride, 0)
        return F.relu(h + sc)

    inp = dev(x).requires_grad_(True)
    a = F.relu(ConvBN.apply(inp, he(64, 3, 7), 2, 3))
    a = F.max_pool2d(a, 3, 2, 1)
    for cin, cout, stride in [(64, 64, 1), (64, 64, 1), (64, 128, 2), (128, 128, 1), (128, 256, 2), (256, 256, 1),
                              (256, 512, 2), (512, 512, 1)]:
        a = block(a, cin, cout, stride)
    a = F.adaptive_avg_pool2d(a, 1).flatten(1)
    logits = Linear.apply(a, synth.normal(g, (512, 1000), std=(2.0 / 512) ** 0.5))
    loss = F.cross_entropy(logits, labels)
    loss.backward()
    assert state["n"] == 20                    # 17 3x3 / 7x7 convs + 3 downsample 1x1
    assert bool(torch.isfinite(inp.grad).all()) and float(inp.grad.abs().max()) > 0.0
