"""Synthetic training steps (forward + backward) with every conv / FC product and every batch-norm
running through the library: 8-bit forward and layer-gradient products, 16x8-bit weight gradients
from the bifurcated gradient copies, Range BN with its statistics gathered in the conv epilogue
(Sections 3, 4 and 7 of the paper).

    python -m paper_1805_11046_amd.train_step --net resnet18   [--batch 256] [--steps 5] [--breakdown]
    python -m paper_1805_11046_amd.train_step --net bottleneck [--batch 128] [--steps 20] [--breakdown]

resnet18: the full network on 3x224x224 inputs ~N(0,1), 1000 classes, random labels.
bottleneck: one ResNet-50 block, 1x1 256->64, 3x3 64->64, 1x1 64->256 at 56x56, each followed by
Range BN (+ReLU), identity shortcut; inputs |N(0,1)|, output gradient ~N(0, sigma 1e-3).
He-normal weights everywhere.

ReLU, max/avg pooling, the residual additions and the softmax cross-entropy are elementwise glue
outside the method; they are left to torch (autograd supplies their gradients).  The optimizer
update is not part of the measured step.  Where a Range BN feeds a ReLU and then only the next
convolution, the three passes (normalize, rectify, quantize) run as one that emits the 8-bit
codes (--no-fuse keeps them apart).  Prints the step time and, with --breakdown, per entry
point: time, share, integer throughput of the products (2 x multiply-accumulates of the layer, the
weight gradient counted once although it executes two byte-plane products) and algorithmic bytes
per second of the streaming calls.  Needs a GPU.
"""
import argparse
import collections
import time

import torch
import torch.nn.functional as F

from . import binding as q8t

_breakdown = False   # time every library call with events
_bracket = None      # or only the calls of this entry point
_fuse = True
_angles = None   # with --angles: {kind: [cosines]} of tensors against their quantized copies


def _call(name, ops, nbytes, fn, *a, tag="", **k):
    """Run one library call; with --breakdown (or for the one entry point being bracketed) also time
    it with events on the launch stream and book its integer operations and algorithmic bytes under
    `name` (and `tag`, the layer it belongs to)."""
    if not (_breakdown or _bracket == name):
        return fn(*a, **k)
    e0 = _evpool.pop() if _evpool else torch.cuda.Event(enable_timing=True)
    e1 = _evpool.pop() if _evpool else torch.cuda.Event(enable_timing=True)
    e0.record()
    r = fn(*a, **k)
    e1.record()
    _pending.append((name, tag, ops, nbytes, e0, e1))
    return r


def record(breakdown=False, bracket=None):
    """Switch the event timing of library calls on or off (see _call)."""
    global _breakdown, _bracket
    _breakdown, _bracket = breakdown, bracket


def drain():
    """The (name, tag, ops, bytes, microseconds) records collected since the last drain (synchronizes)."""
    torch.cuda.synchronize()
    out = [(n, t, o, b, e0.elapsed_time(e1) * 1e3) for n, t, o, b, e0, e1 in _pending]
    for rec in _pending:   # the events go back to the pool: creating a pair per call costs the host more than recording it
        _evpool.extend(rec[4:6])
    del _pending[:]
    return out


def _tag(d):
    return "%dx%d%s %d->%d @%d" % (d.R, d.S, "/%d" % d.stride if d.stride > 1 else "", d.C, d.K, d.H)


def _angle(kind, t, q, qp):
    if _angles is not None:
        _angles.setdefault(kind, []).append(q8t.quant_angle(t, q, qp)[3])


_qcache = {}   # data_ptr of an activation -> (codes, parameters) left behind by the kernel that wrote it
_pcache = {}   # (data_ptr of a layer's weight codes, 0 forward / 1 layer gradient) -> its packed filter for this step
_pbufs = {}    # the same keys by weight tensor: buffers kept from step to step
# Pack all filters in one launch after the weights are quantized (off: every product packs its own, a small launch in
# front of each).  Off: the best runs gain 0.06 ms of 8.5 with it, but the timed single-stream loop came out 0.3 - 1.5
# ms slower in most trials (first processes on a fresh machine above all), with unchanged per-call times; until that is
# understood the step keeps the per-call pre-pass.  tests/test_gpu_train_step.py runs both ways.
_pack = False


def _packed(qw, which):
    return _pcache.get((qw.data_ptr(), which))


def _quantize(name, t):
    hit = _qcache.get(t.data_ptr())
    if hit is not None and hit[0].shape == t.shape:
        return hit
    n = t.numel()
    # two passes over the fp32 tensor and one byte written; small tensors stay in registers (one pass)
    q, qp = _call(name, 0, (9 if n > 65536 else 5) * n, q8t.quantize, t, 8)
    _angle("weights, 8 bit" if "weights" in name else "activations, 8 bit", t, q, qp)
    return q, qp


def _bn_bwd(fn, name, ny, *args):
    """Range BN backward + the two gradient copies; with --angles the fp32 gradient is kept for the
    cosine against its copies."""
    want = _angles is not None
    # algorithmic bytes per element: pass 1 reads x and dy (8), pass 2 reads dy (4; and x again under the rectifier,
    # whose mask it recomputes) and writes the two copies (3), plus dx (4) when it is wanted
    per = (19 if "relu" in name else 15) + (4 if want else 0)
    r = _call(name, 0, per * ny, fn, *args, want_dx=want)
    if want:
        _angle("layer gradients, 8 bit", r[0], r[3], r[4])
        _angle("layer gradients, 16 bit", r[0], r[5], r[6])
    return r


_overlap = False     # weight gradients on a second stream (see _wgrad)
_side = {}           # device index -> [stream, workspace]


def _wgrad(d, qa, pa, g16, pg16, ops, nx, ny):
    """The weight gradient of a layer.  Nothing downstream of it is needed before the optimizer, so with
    `_overlap` it is issued on a second stream (default priority) with a workspace of its own and runs beside the
    Range BN passes and layer gradients of the layers below it, which are bound by memory and vector arithmetic where
    this product is bound by the matrix units and LDS; step() joins the stream at its end."""
    if not _overlap or _breakdown or _bracket:    # calls that are being timed one by one stay on one stream
        return _call("qconv_wgrad", ops, nx + 2 * ny, q8t.qconv_wgrad, d, qa, pa, g16, pg16, tag=_tag(d))[0]
    dev = g16.device
    main = torch.cuda.current_stream(dev)
    ent = _side.get(dev.index)
    if ent is None:
        ent = _side[dev.index] = [torch.cuda.Stream(dev), None]
    side = ent[0]
    side.wait_stream(main)          # the codes were written on the main stream
    need = q8t.qconv_workspace_size(d, 2)
    with torch.cuda.stream(side):
        if ent[1] is None or ent[1].numel() < need:
            ent[1] = torch.empty(max(int(need), 256), dtype=torch.uint8, device=dev)
        dw, _ = _call("qconv_wgrad", ops, nx + 2 * ny, q8t.qconv_wgrad, d, qa, pa, g16, pg16, ws=ent[1], tag=_tag(d))
    _keep.append((qa, pa, g16, pg16))   # their memory must not be handed out again before the side stream is done with it
    return dw


_keep = []


def _join_side():
    for idx, (side, _) in _side.items():
        torch.cuda.current_stream(idx).wait_stream(side)
    del _keep[:]   # freed on the main stream, which is now behind the side stream


_pending = []
_evpool = []
_layer = [0]   # layers are numbered in forward order; a layer's backward draws its two roundings with seeds 2 id + 1, + 2


def _next_layer():
    _layer[0] += 1
    return _layer[0]


def _convbn_fwd(a, w, stride, pad, apply=True):
    """quantize -> conv forward (+ Range BN statistics) -> Range BN; returns the normalized tensor (apply=False: the
    conv result and its statistics, for a consumer that normalizes on the fly) and what the backward pass needs"""
    a = a.contiguous()
    n, c, h, wd = a.shape
    k, _, r, s = w.shape
    d = q8t.conv_desc(n, c, h, wd, k, r, s, stride, pad)
    qa, pa = _quantize("quantize (activations)", a)
    qw, pw = _quantize("quantize (weights)", w)
    ops = 2.0 * n * d.P * d.Q * k * c * r * s
    nx, ny = a.numel(), n * k * d.P * d.Q
    y, _, stats = _call("qconv_fwd_bn_stats", ops, nx + 4 * ny, q8t.qconv_fwd_bn_stats, d, qa, pa, qw, pw, tag=_tag(d),
                        packed=_packed(qw, 0))
    saved = (d, qa, pa, qw, pw, y, stats, ops, nx, ny, _next_layer())
    if not apply:
        return (y, stats), saved
    bn, _, _ = _call("range_bn_fwd_apply", 0, 8 * ny, q8t.range_bn_fwd_apply, y, stats, None, None, 1e-5)
    return bn, saved


def _convbn_bwd(saved, dbn, need_dx, lattice=False):
    """Range BN backward + bifurcated gradient quantization -> layer gradient, weight gradient.  lattice: for a 1x1
    layer with a stride and no padding the layer gradient is returned on the positions the layer read (the stride-1
    product at the reduced resolution; it is zero everywhere else), for q8t.relu_bwd_sum_lattice"""
    d, qa, pa, qw, pw, y, stats, ops, nx, ny, lid = saved
    _, _, _, g8, pg8, g16, pg16 = _bn_bwd(q8t.range_bn_bwd_bifurcate, "range_bn_bwd_bifurcate", ny, y, dbn.contiguous(),
                                          stats, None, 1e-5, 2 * lid + 1, 2 * lid + 2)
    dx = None
    if need_dx and lattice:
        ds = q8t.conv_desc(d.N, d.C, d.P, d.Q, d.K, 1, 1, 1, 0)
        dx, _ = _call("qconv_dgrad", ops, ny + 4 * (nx // (d.stride * d.stride)), q8t.qconv_dgrad, ds, g8, pg8, qw, pw, tag=_tag(d),
                      packed=_packed(qw, 1))
    elif need_dx:
        dx, _ = _call("qconv_dgrad", ops, ny + 4 * nx, q8t.qconv_dgrad, d, g8, pg8, qw, pw, tag=_tag(d), packed=_packed(qw, 1))
    dw = _wgrad(d, qa, pa, g16, pg16, ops, nx, ny)
    return dx, dw


class ConvBN(torch.autograd.Function):
    """conv + Range BN as one autograd node (see _convbn_fwd / _convbn_bwd)."""

    @staticmethod
    def forward(ctx, a, w, stride, pad, need_dx):
        bn, ctx.saved = _convbn_fwd(a, w, stride, pad)
        ctx.need_dx = need_dx
        return bn

    @staticmethod
    def backward(ctx, dbn):
        dx, dw = _convbn_bwd(ctx.saved, dbn, ctx.need_dx)
        return dx, dw, None, None, None


class StemConvBNPool(torch.autograd.Function):
    """First layer: quantize -> conv forward (+ Range BN statistics) -> Range BN + ReLU + 3x3/2 max pooling in one
    pass (the normalized 112x112 tensor is never written); backward: pooled gradient -> Range BN backward + 16-bit
    copy of its result, the upstream gradient of the Range BN gathered from the pooled one on the fly -> weight
    gradient.  The network input needs no gradient."""

    @staticmethod
    def forward(ctx, a, w, stride, pad):
        a = a.contiguous()
        n, c, h, wd = a.shape
        k, _, r, s = w.shape
        d = q8t.conv_desc(n, c, h, wd, k, r, s, stride, pad)
        qa, pa = _quantize("quantize (activations)", a)
        qw, pw = _quantize("quantize (weights)", w)
        ops = 2.0 * n * d.P * d.Q * k * c * r * s
        nx, ny = a.numel(), n * k * d.P * d.Q
        y, _, stats = _call("qconv_fwd_bn_stats", ops, nx + 4 * ny, q8t.qconv_fwd_bn_stats, d, qa, pa, qw, pw, tag=_tag(d))
        pooled, idx = _call("range_bn_relu_maxpool_fwd", 0, 4 * ny + 5 * (ny // 4), q8t.range_bn_relu_maxpool_fwd, y, stats,
                            None, None, 1e-5)
        ctx.saved = (d, qa, pa, y, stats, idx, ops, nx, ny, _next_layer())
        return pooled

    @staticmethod
    def backward(ctx, gp):
        d, qa, pa, y, stats, idx, ops, nx, ny, lid = ctx.saved
        if _angles is None:
            # the unpooled gradient is never written: both passes gather it from the pooled one; no 8-bit copy (the
            # network input needs no gradient).  Bytes: x once (4), the pooled gradient and its indices twice
            # (2 * 5 / 4), the 16-bit copy (2)
            _, _, _, _, g16, pg16 = _call("maxpool_range_bn_bwd_bifurcate", 0, 6 * ny + 10 * (ny // 4),
                                          q8t.maxpool_range_bn_bwd_bifurcate, y, gp.contiguous(), idx, stats, None, 1e-5,
                                          2 * lid + 1, 2 * lid + 2, False)
        else:
            dy = _call("maxpool_relu_bwd", 0, 5 * (ny // 4) + 4 * ny, q8t.maxpool_relu_bwd, gp.contiguous(), idx, d.P, d.Q)
            _, _, _, g8, pg8, g16, pg16 = _bn_bwd(q8t.range_bn_bwd_bifurcate, "range_bn_bwd_bifurcate", ny, y, dy, stats, None,
                                                  1e-5, 2 * lid + 1, 2 * lid + 2)
        dw = _wgrad(d, qa, pa, g16, pg16, ops, nx, ny)
        return None, dw, None, None


def _chain_fwd(a, specs, ws, apply_last=True):
    """conv -> Range BN -> ReLU -> conv -> Range BN [-> ReLU -> conv -> Range BN]: between two
    convolutions the normalization, the ReLU and the 8-bit quantization of the next operand are one
    pass that writes codes only (no fp32 activation, no separate quantization)"""
    a = a.contiguous()
    qa, pa = _quantize("quantize (activations)", a)
    saved = []
    shape = a.shape
    for i, (w, (stride, pad)) in enumerate(zip(ws, specs)):
        n, c, h, wd = shape
        k, _, r, s = w.shape
        d = q8t.conv_desc(n, c, h, wd, k, r, s, stride, pad)
        qw, pw = _quantize("quantize (weights)", w)
        ops = 2.0 * n * d.P * d.Q * k * c * r * s
        nx, ny = n * c * h * wd, n * k * d.P * d.Q
        y, _, stats = _call("qconv_fwd_bn_stats", ops, nx + 4 * ny, q8t.qconv_fwd_bn_stats, d, qa, pa, qw, pw, tag=_tag(d),
                            packed=_packed(qw, 0))
        saved.append((d, qa, pa, qw, pw, y, stats, ops, nx, ny, _next_layer()))
        if i + 1 < len(ws):
            _, qa, pa = _call("range_bn_relu_fwd_apply (int8 out)", 0, 5 * ny, q8t.range_bn_relu_fwd_apply, y, stats,
                              None, None, 1e-5, True, False)
        elif apply_last:
            out, _, _ = _call("range_bn_fwd_apply", 0, 8 * ny, q8t.range_bn_fwd_apply, y, stats, None, None, 1e-5)
        else:
            out = (y, stats)     # the consumer normalizes on the fly
        shape = (n, k, d.P, d.Q)
    return out, saved


def _chain_bwd(saved, g, need_dx, block_end=None):
    """backward of _chain_fwd: the ReLU mask is recomputed inside the Range BN backward.  block_end = (other, act):
    the chain is the main branch of a residual block; the layer gradient of its first convolution then also adds
    the other branch's gradient and applies the mask of the block's input (act > 0) in its epilogue."""
    g = g.contiguous()
    dws = [None] * len(saved)
    for i in range(len(saved) - 1, -1, -1):
        d, qa, pa, qw, pw, y, stats, ops, nx, ny, lid = saved[i]
        if i + 1 == len(saved):
            r = _bn_bwd(q8t.range_bn_bwd_bifurcate, "range_bn_bwd_bifurcate", ny, y, g, stats, None, 1e-5, 2 * lid + 1,
                        2 * lid + 2)
        else:
            r = _bn_bwd(q8t.range_bn_relu_bwd_bifurcate, "range_bn_relu_bwd_bifurcate", ny, y, g, stats, None, None,
                        1e-5, 2 * lid + 1, 2 * lid + 2)
        g8, pg8, g16, pg16 = r[3:]
        g = None
        if i == 0 and block_end is not None:
            other, act = block_end
            g = _call("qconv_dgrad", ops, ny + (12 if other is not None else 8) * nx, q8t.qconv_dgrad_relu_sum, d, g8, pg8,
                      qw, pw, other, act, tag=_tag(d), packed=_packed(qw, 1))
        elif i > 0 or need_dx:
            g, _ = _call("qconv_dgrad", ops, ny + 4 * nx, q8t.qconv_dgrad, d, g8, pg8, qw, pw, tag=_tag(d), packed=_packed(qw, 1))
        dws[i] = _wgrad(d, qa, pa, g16, pg16, ops, nx, ny)
    return g, dws


class ConvChain(torch.autograd.Function):
    """a chain of convolutions with fused Range BN / ReLU / quantization between them as one autograd node"""

    @staticmethod
    def forward(ctx, a, need_dx, specs, *ws):
        out, saved = _chain_fwd(a, specs, ws)
        ctx.saved = (saved, need_dx)
        return out

    @staticmethod
    def backward(ctx, g):
        saved, need_dx = ctx.saved
        g, dws = _chain_bwd(saved, g, need_dx)
        return (g, None, None, *dws)


class ResBlock(torch.autograd.Function):
    """A whole basic block as one node: conv chain + shortcut (identity or 1x1 conv + Range BN) + add + ReLU with the
    8-bit codes of the result left behind.  Its input gets gradients from both branches; they are summed -- and, when
    the input is itself the rectified output of the previous block, masked by that rectifier -- in one pass
    (`mask_input`), so the previous block receives an already masked gradient (`grad_is_masked`) and no separate
    sum and masking passes run between blocks."""

    @staticmethod
    def forward(ctx, a, stride, quantized, mask_input, grad_is_masked, w1, w2, wsc):
        # the last Range BN of the chain, the shortcut's Range BN (if it has one), the sum, the rectifier and the
        # 8-bit codes of the result are one pass over the conv results
        (y2, st2), chain = _chain_fwd(a, ((stride, 1), (1, 1)), (w1, w2), apply_last=False)
        n = y2.numel()
        if wsc is None:
            scs = None
            out, q, qp = _call("range_bn_add_relu_quantize", 0, (17 if quantized else 12) * n, q8t.range_bn_add_relu_quantize,
                               y2, st2, a.contiguous(), eps=1e-5, quantized=quantized)
        else:
            (ysc, stsc), scs = _convbn_fwd(a, wsc, stride, 0, apply=False)
            out, q, qp = _call("range_bn_add_relu_quantize", 0, (17 if quantized else 12) * n, q8t.range_bn_add_relu_quantize,
                               y2, st2, ysc, other_stats=stsc, eps=1e-5, quantized=quantized)
        if quantized:
            _qcache[out.data_ptr()] = (q, qp)
        # (a detached alias of the output: the output itself would point back at this node and keep the whole step's
        # saved tensors alive until the cycle collector runs)
        ctx.saved = (chain, scs, a if mask_input else None, out.detach(), grad_is_masked)
        return out

    @staticmethod
    def backward(ctx, g):
        chain, scs, a, out, grad_is_masked = ctx.saved
        g = g.contiguous()
        gm = g if grad_is_masked else _call("relu_bwd_add", 0, 12 * g.numel(), q8t.relu_bwd_add, g, out)
        stride = chain[0][0].stride
        if scs is not None and a is not None and stride > 1:
            # the shortcut's gradient stays on the lattice its 1x1 layer read: no zero-filled tensor is written or read
            gs, dwsc = _convbn_bwd(scs, gm, True, lattice=True)
            gc, (dw1, dw2) = _chain_bwd(chain, gm, True)
            ga = _call("relu_bwd_sum", 0, 12 * gc.numel() + 4 * gs.numel(), q8t.relu_bwd_sum_lattice, gc, gs, a, stride)
            return ga, None, None, None, None, dw1, dw2, dwsc
        gs, dwsc = (gm, None) if scs is None else _convbn_bwd(scs, gm, True)
        if a is not None:
            ga, (dw1, dw2) = _chain_bwd(chain, gm, True, (gs, a))
        else:
            gc, (dw1, dw2) = _chain_bwd(chain, gm, True)
            ga = _call("relu_bwd_sum", 0, 12 * gc.numel(), q8t.relu_bwd_sum, gc, gs, None)
        return ga, None, None, None, None, dw1, dw2, dwsc


class Linear(torch.autograd.Function):
    @staticmethod
    def forward(ctx, a, w):
        a = a.contiguous()
        qa, pa = _quantize("quantize (activations)", a)
        qw, pw = _quantize("quantize (weights)", w)
        ops = 2.0 * a.shape[0] * a.shape[1] * w.shape[1]
        y, _ = _call("qgemm_fwd", ops, a.numel() + w.numel() + 4 * a.shape[0] * w.shape[1], q8t.qgemm_fwd, qa, pa, qw, pw)
        ctx.saved = (qa, pa, qw, pw, ops, _next_layer())
        return y

    @staticmethod
    def backward(ctx, dy):
        qa, pa, qw, pw, ops, lid = ctx.saved
        g8, pg8, g16, pg16 = _call("quantize_bifurcate", 0, 11 * dy.numel(), q8t.quantize_bifurcate, dy.contiguous(),
                                   2 * lid + 1, 2 * lid + 2)
        dx, _ = _call("qgemm_dgrad", ops, dy.numel() + qw.numel() + 4 * qa.numel(), q8t.qgemm_dgrad, g8, pg8, qw, pw)
        dw, _ = _call("qgemm_wgrad", ops, qa.numel() + 2 * dy.numel() + 4 * qw.numel(), q8t.qgemm_wgrad, qa, pa, g16, pg16)
        return dx, dw


STAGES = [(64, 64, 1), (64, 64, 1), (64, 128, 2), (128, 128, 1), (128, 256, 2), (256, 256, 1), (256, 512, 2), (512, 512, 1)]


def _he(dev, gen, cout, cin, r):
    w = torch.randn((cout, cin, r, r), device=dev, generator=gen) * (2.0 / (cin * r * r)) ** 0.5
    return w.requires_grad_(True)


def make_weights(dev, gen):
    def he(cout, cin, r):
        return _he(dev, gen, cout, cin, r)

    ws = {"conv1": he(64, 3, 7), "blocks": []}
    for cin, cout, stride in STAGES:
        b = {"c1": he(cout, cin, 3), "c2": he(cout, cout, 3)}
        if stride != 1 or cin != cout:
            b["sc"] = he(cout, cin, 1)
        ws["blocks"].append(b)
    ws["fc"] = (torch.randn((512, 1000), device=dev, generator=gen) * (2.0 / 512) ** 0.5).requires_grad_(True)
    return ws


def _quantize_weights(tensors):
    """all weight tensors of the network in one call (two launches instead of one or two per tensor); the layers
    find the codes in the cache when they ask for them"""
    tensors = [t if t.is_contiguous() else t.contiguous() for t in tensors]
    n = sum(t.numel() for t in tensors)
    res = _call("quantize (weights)", 0, 9 * n, q8t.quantize_multi, [t.detach() for t in tensors], 8)
    for t, (q, qp) in zip(tensors, res):
        _angle("weights, 8 bit", t, q, qp)
        _qcache[t.data_ptr()] = (q, qp)


def _pack_filters(x, ws):
    """The filters of every convolution of the network, in the layouts its forward and layer-gradient kernels read,
    by one launch (the products then skip their own small pre-pass)."""
    n = x.shape[0]
    h = (x.shape[2] + 2 * 3 - 7) // 2 + 1      # first layer 7x7 / 2, pad 3
    h = (h + 2 * 1 - 3) // 2 + 1               # pooling 3x3 / 2, pad 1
    jobs, keys = [], []

    def add(w, d, which):
        qw, _ = _quantize("quantize (weights)", w)
        jobs.append((d, which, qw))
        keys.append(((w.data_ptr(), which), (qw.data_ptr(), which)))

    for (cin, cout, stride), b in zip(STAGES, ws["blocks"]):
        h2 = (h + 2 - 3) // stride + 1
        d1 = q8t.conv_desc(n, cin, h, h, cout, 3, 3, stride, 1)
        d2 = q8t.conv_desc(n, cout, h2, h2, cout, 3, 3, 1, 1)
        for w, d in ((b["c1"], d1), (b["c2"], d2)):
            add(w, d, 0)
            add(w, d, 1)
        if "sc" in b:
            add(b["sc"], q8t.conv_desc(n, cin, h, h, cout, 1, 1, stride, 0), 0)
            # its layer gradient runs as the stride-1 product on the positions the layer read (_convbn_bwd)
            add(b["sc"], q8t.conv_desc(n, cin, h2, h2, cout, 1, 1, 1, 0), 1)
        h = h2
    nbytes = 2 * sum(j[2].numel() for j in jobs)
    bufs = _call("qconv_pack_multi", 0, nbytes, q8t.qconv_pack_multi, jobs, [_pbufs.get(k[0]) for k in keys])
    for (kw, kq), b in zip(keys, bufs):
        if b is not None:
            _pbufs[kw] = b
            _pcache[kq] = b


def step(x, labels, ws):
    _qcache.clear()
    _pcache.clear()
    _layer[0] = 0
    if _fuse:
        _quantize_weights([ws["conv1"], ws["fc"]] + [w for b in ws["blocks"] for w in b.values()])
        if _pack:
            _pack_filters(x, ws)
    if _fuse:
        a = StemConvBNPool.apply(x, ws["conv1"], 2, 3)
    else:
        a = F.relu(ConvBN.apply(x, ws["conv1"], 2, 3, False))     # the network input needs no gradient
        a = F.max_pool2d(a, 3, 2, 1)
    last = len(ws["blocks"]) - 1
    for i, ((cin, cout, stride), b) in enumerate(zip(STAGES, ws["blocks"])):
        if _fuse:
            # the first block's input is the pooled tensor (its rectifier is inside the pooling indices); the last
            # block's output goes to torch's pooling, which hands back an unmasked gradient
            a = ResBlock.apply(a, stride, i != last, i != 0, i != last, b["c1"], b["c2"], b.get("sc"))
        else:
            h = F.relu(ConvBN.apply(a, b["c1"], stride, 1, True))
            h = ConvBN.apply(h, b["c2"], 1, 1, True)
            sc = ConvBN.apply(a, b["sc"], stride, 0, True) if "sc" in b else a
            a = F.relu(h + sc)
    a = F.adaptive_avg_pool2d(a, 1).flatten(1)
    loss = F.cross_entropy(Linear.apply(a, ws["fc"]), labels)
    loss.backward()
    _join_side()
    return loss


def bottleneck_step(x, gy, ws):
    _layer[0] = 0
    if _fuse:
        h = ConvChain.apply(x, True, ((1, 0), (1, 1), (1, 0)), *ws)
    else:
        h = F.relu(ConvBN.apply(x, ws[0], 1, 0, True))
        h = F.relu(ConvBN.apply(h, ws[1], 1, 1, True))
        h = ConvBN.apply(h, ws[2], 1, 0, True)
    out = F.relu(h + x)
    out.backward(gy)
    return out


def main():
    global _breakdown, _fuse, _angles
    ap = argparse.ArgumentParser()
    ap.add_argument("--net", choices=["resnet18", "bottleneck"], default="resnet18")
    ap.add_argument("--batch", type=int, default=0, help="default 256 (resnet18) / 128 (bottleneck)")
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--breakdown", action="store_true")
    ap.add_argument("--angles", action="store_true",
                    help="after the timing, one more step that reports the cosine between tensors and their "
                         "quantized copies (Sec. 5.1 (Problem Statement), eq. (1)) per kind of tensor")
    ap.add_argument("--no-fuse", action="store_true",
                    help="Range BN, ReLU and the next layer's quantization as separate passes")
    args = ap.parse_args()
    _fuse = not args.no_fuse
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(0)
    if args.net == "resnet18":
        args.batch = args.batch or 256
        ws = make_weights(dev, gen)
        x = torch.randn((args.batch, 3, 224, 224), device=dev, generator=gen)
        labels = torch.randint(0, 1000, (args.batch,), device=dev, generator=gen)
        params = [ws["conv1"], ws["fc"]] + [w for b in ws["blocks"] for w in b.values()]

        def one():
            for p in params:
                p.grad = None
            return step(x, labels, ws)
    else:
        args.batch = args.batch or 128
        params = [_he(dev, gen, 64, 256, 1), _he(dev, gen, 64, 64, 3), _he(dev, gen, 256, 64, 1)]
        x = torch.randn((args.batch, 256, 56, 56), device=dev, generator=gen).abs_().requires_grad_(True)
        gy = torch.randn((args.batch, 256, 56, 56), device=dev, generator=gen) * 1e-3

        def one():
            for p in params:
                p.grad = None
            x.grad = None
            return bottleneck_step(x, gy, params).sum()

    for _ in range(args.warmup):
        loss = one()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        loss = one()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    assert bool(torch.isfinite(loss)) and all(p.grad is not None and bool(torch.isfinite(p.grad).all()) for p in params)
    print("%s training step, batch %d%s: %.2f ms / step (%.0f images/s)" % (
        args.net, args.batch, "" if _fuse else " (unfused)", ms, args.batch / ms * 1e3))
    if args.angles:
        import math
        _angles = {}
        one()
        torch.cuda.synchronize()
        print("cosine between a tensor and its quantized copy, mean / min over the layers (angle of the mean):")
        for kind, vals in sorted(_angles.items()):
            c = torch.stack(vals).double().cpu()
            print("  %-26s %3d tensors  mean %.8f  min %.8f  (%.3f deg)" % (
                kind, len(vals), float(c.mean()), float(c.min()), math.degrees(math.acos(min(1.0, float(c.mean()))))))
        _angles = None
    if args.breakdown:
        _breakdown = True
        one()
        torch.cuda.synchronize()
        acc = collections.defaultdict(lambda: [0.0, 0.0, 0.0, 0])
        for name, _, ops, nbytes, e0, e1 in _pending:
            a = acc[name]
            a[0] += e0.elapsed_time(e1)
            a[1] += ops
            a[2] += nbytes
            a[3] += 1
        lib = sum(a[0] for a in acc.values())
        print("library calls: %.2f ms of the step (each call timed with events, launch gaps included)" % lib)
        print("  %-34s %6s %9s %9s %10s" % ("entry point", "calls", "ms", "TOP/s", "GB/s (alg.)"))
        for name, (t, ops, nbytes, cnt) in sorted(acc.items(), key=lambda kv: -kv[1][0]):
            print("  %-34s %6d %9.3f %9s %10.0f" % (name, cnt, t, "%.0f" % (ops / t / 1e9) if ops else "-", nbytes / t / 1e6))


if __name__ == "__main__":
    main()
