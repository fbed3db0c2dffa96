"""One synthetic ResNet-18 training step (forward + backward) with every conv / FC product and
every batch-norm running through the library: 8-bit forward and layer-gradient products, 16x8-bit
weight gradients from the bifurcated gradient copies, Range BN with its statistics gathered in
the conv epilogue (Sections 3, 4 and 7 of the paper).

    python -m paper_1805_11046_amd.resnet18_step [--batch 256] [--steps 5] [--breakdown]

ReLU, max/avg pooling, the residual additions and the softmax cross-entropy are elementwise glue
outside the method; they are left to torch (autograd supplies their gradients).  The optimizer
update is not part of the measured step.  Inputs N(0,1), He-normal weights, random labels.
Prints the step time, the share of the library calls in it and, with --breakdown, the time per
entry point.  Needs a GPU.
"""
import argparse
import collections
import time

import torch
import torch.nn.functional as F

from . import binding as q8t

_times = collections.defaultdict(float)
_breakdown = False


def _call(name, fn, *a, **k):
    if not _breakdown:
        return fn(*a, **k)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    r = fn(*a, **k)
    e1.record()
    _pending.append((name, e0, e1))
    return r


_pending = []
_seed = [1]


class ConvBN(torch.autograd.Function):
    """quantize -> conv forward (+ Range BN statistics) -> Range BN;  backward: Range BN backward +
    bifurcated gradient quantization -> layer gradient, weight gradient."""

    @staticmethod
    def forward(ctx, a, w, stride, pad, need_dx):
        a = a.contiguous()
        n, c, h, wd = a.shape
        k, _, r, s = w.shape
        d = q8t.conv_desc(n, c, h, wd, k, r, s, stride, pad)
        qa, pa = _call("quantize (activations)", q8t.quantize, a, 8)
        qw, pw = _call("quantize (weights)", q8t.quantize, w, 8)
        y, _, stats = _call("qconv_fwd_bn_stats", q8t.qconv_fwd_bn_stats, d, qa, pa, qw, pw)
        bn, _, _ = _call("range_bn_fwd_apply", q8t.range_bn_fwd_apply, y, stats, None, None, 1e-5)
        ctx.saved = (d, qa, pa, qw, pw, y, stats, need_dx)
        return bn

    @staticmethod
    def backward(ctx, dbn):
        d, qa, pa, qw, pw, y, stats, need_dx = ctx.saved
        _seed[0] += 2
        _, _, _, g8, pg8, g16, pg16 = _call("range_bn_bwd_bifurcate", q8t.range_bn_bwd_bifurcate, y, dbn.contiguous(),
                                            stats, None, 1e-5, _seed[0], _seed[0] + 1)
        dx = None
        if need_dx:
            dx, _ = _call("qconv_dgrad", q8t.qconv_dgrad, d, g8, pg8, qw, pw)
        dw, _ = _call("qconv_wgrad", q8t.qconv_wgrad, d, qa, pa, g16, pg16)
        return dx, dw, None, None, None


class Linear(torch.autograd.Function):
    @staticmethod
    def forward(ctx, a, w):
        a = a.contiguous()
        qa, pa = _call("quantize (activations)", q8t.quantize, a, 8)
        qw, pw = _call("quantize (weights)", q8t.quantize, w, 8)
        y, _ = _call("qgemm_fwd", q8t.qgemm_fwd, qa, pa, qw, pw)
        ctx.saved = (qa, pa, qw, pw)
        return y

    @staticmethod
    def backward(ctx, dy):
        qa, pa, qw, pw = ctx.saved
        _seed[0] += 2
        g8, pg8, g16, pg16 = _call("quantize_bifurcate", q8t.quantize_bifurcate, dy.contiguous(), _seed[0], _seed[0] + 1)
        dx, _ = _call("qgemm_dgrad", q8t.qgemm_dgrad, g8, pg8, qw, pw)
        dw, _ = _call("qgemm_wgrad", q8t.qgemm_wgrad, qa, pa, g16, pg16)
        return dx, dw


STAGES = [(64, 64, 1), (64, 64, 1), (64, 128, 2), (128, 128, 1), (128, 256, 2), (256, 256, 1), (256, 512, 2), (512, 512, 1)]


def make_weights(dev, gen):
    def he(cout, cin, r):
        w = torch.randn((cout, cin, r, r), device=dev, generator=gen) * (2.0 / (cin * r * r)) ** 0.5
        return w.requires_grad_(True)

    ws = {"conv1": he(64, 3, 7), "blocks": []}
    for cin, cout, stride in STAGES:
        b = {"c1": he(cout, cin, 3), "c2": he(cout, cout, 3)}
        if stride != 1 or cin != cout:
            b["sc"] = he(cout, cin, 1)
        ws["blocks"].append(b)
    ws["fc"] = (torch.randn((512, 1000), device=dev, generator=gen) * (2.0 / 512) ** 0.5).requires_grad_(True)
    return ws


def step(x, labels, ws):
    a = F.relu(ConvBN.apply(x, ws["conv1"], 2, 3, False))     # the network input needs no gradient
    a = F.max_pool2d(a, 3, 2, 1)
    for (cin, cout, stride), b in zip(STAGES, ws["blocks"]):
        h = F.relu(ConvBN.apply(a, b["c1"], stride, 1, True))
        h = ConvBN.apply(h, b["c2"], 1, 1, True)
        sc = ConvBN.apply(a, b["sc"], stride, 0, True) if "sc" in b else a
        a = F.relu(h + sc)
    a = F.adaptive_avg_pool2d(a, 1).flatten(1)
    loss = F.cross_entropy(Linear.apply(a, ws["fc"]), labels)
    loss.backward()
    return loss


def main():
    global _breakdown
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--breakdown", action="store_true")
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(0)
    ws = make_weights(dev, gen)
    x = torch.randn((args.batch, 3, 224, 224), device=dev, generator=gen)
    labels = torch.randint(0, 1000, (args.batch,), device=dev, generator=gen)
    params = [ws["conv1"], ws["fc"]] + [w for b in ws["blocks"] for w in b.values()]

    def one():
        for p in params:
            p.grad = None
        return step(x, labels, ws)

    for _ in range(args.warmup):
        loss = one()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        loss = one()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    assert bool(torch.isfinite(loss)) and all(p.grad is not None and bool(torch.isfinite(p.grad).all()) for p in params)
    print("resnet18 training step, batch %d: %.2f ms / step (%.0f images/s), loss %.4f" % (args.batch, ms, args.batch / ms * 1e3, float(loss.detach())))
    if args.breakdown:
        _breakdown = True
        one()
        torch.cuda.synchronize()
        for name, e0, e1 in _pending:
            _times[name] += e0.elapsed_time(e1)
        lib = sum(_times.values())
        print("library calls: %.2f ms of the step" % lib)
        for name, t in sorted(_times.items(), key=lambda kv: -kv[1]):
            print("  %-28s %8.3f ms" % (name, t))


if __name__ == "__main__":
    main()
