"""Benchmark of the 8-bit training hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input, for the
ResNet-18 3x3 conv layer 64->64 @56x56, batch 128 (the conv of config 2 followed by the Range BN
of config 1's shape, 128x64x56x56):

  forward : quantize X and W (min/max, nearest) -> int8 conv forward, whose epilogue also gathers the
            Range BN statistics -> Range BN normalization to an 8-bit per-tensor output (config 1)
  backward: Range BN backward fused with the bifurcated stochastic quantization of the gradient
            (8-bit and 16-bit copies) -> int8 layer-gradient conv -> 16x8-bit weight-gradient conv

All inputs (X, W, upstream gradient, fp32) are resident in HBM before the timed region.  The
reported value is the useful int8 throughput of the three products over the WHOLE step
(3 * 2*M*N*K operations / step time); per-call times, TOPS and GB/s are listed next to it.
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0   # dense int8 MFMA, MI355X (5.0 POP/s)
PEAK_HBM_GBS = 8000.0     # HBM3E, MI355X


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batch", type=int, default=128)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-batch", type=int, default=128)
    return ap.parse_args()


class LayerStep:
    """Buffers and the call sequence of one layer step.  Every call goes through the C ABI."""

    def __init__(self, q8t, torch, batch, seed):
        self.q8t, self.torch = q8t, torch
        dev = torch.device("cuda:0")
        N, C, H, W, K = batch, 64, 56, 56, 64
        self.dims = (N, C, H, W, K)
        g = torch.Generator(device=dev)
        g.manual_seed(seed)
        # synthetic inputs with the workload's distributions: |N(0,1)| activations (post-ReLU),
        # He-normal weights (var 2/576), N(0, std 1e-3)-scale upstream gradient
        self.x = torch.randn((N, C, H, W), device=dev, generator=g).abs_()
        self.w = torch.randn((K, C, 3, 3), device=dev, generator=g) * (2.0 / (C * 9)) ** 0.5
        self.dout = torch.randn((N, K, H, W), device=dev, generator=g) * 1e-2
        self.desc = q8t.conv_desc(N, C, H, W, K, 3, 3, 1, 1)
        e = lambda shape, dt: torch.empty(shape, dtype=dt, device=dev)
        self.qx, self.px = e((N, C, H, W), torch.int8), q8t.new_qparams(dev)
        self.qw, self.pw = e((K, C, 3, 3), torch.int8), q8t.new_qparams(dev)
        self.y = e((N, K, H, W), torch.float32)
        self.bnq = e((N, K, H, W), torch.int8)   # Range BN output, 8-bit per tensor (what the next layer's product reads)
        self.pbn = q8t.new_qparams(dev)
        self.stats = e((3, K), torch.float32)
        self.g = e((N, K, H, W), torch.float32)
        self.g8, self.pg8 = e((N, K, H, W), torch.int8), q8t.new_qparams(dev)
        self.g16, self.pg16 = e((N, K, H, W), torch.int16), q8t.new_qparams(dev)
        self.dx = e((N, C, H, W), torch.float32)
        self.dw = e((K, C, 3, 3), torch.float32)
        n = N * C * H * W
        ops = 2.0 * N * H * W * K * C * 9
        # (name, callable, algorithmic bytes per call, useful int8 ops per call)
        self.calls = [
            ("quantize_x", lambda s: q8t.quantize(self.x, 8, False, 0, q_out=self.qx, qp_out=self.px), 9.0 * n, 0),
            ("quantize_w", lambda s: q8t.quantize(self.w, 8, False, 0, q_out=self.qw, qp_out=self.pw),
             9.0 * self.w.numel(), 0),
            # the conv epilogue also gathers the Range BN statistics of its result (mean, min, max per
            # channel), so the normalization needs no pass of its own over y for them
            ("qconv_fwd_bn_stats", lambda s: q8t.qconv_fwd_bn_stats(self.desc, self.qx, self.px, self.qw, self.pw,
                                                                    out=self.y, stats_out=self.stats),
             1.0 * n + 4.0 * n, ops),
            # config 1: the normalized output leaves as 8-bit codes with the analytic range
            # (4 read + 1 written per element)
            ("range_bn_fwd_apply", lambda s: q8t.range_bn_fwd_apply(self.y, self.stats, None, None, 1e-5,
                                                                    quantized=True, want_y=False, q_out=self.bnq,
                                                                    qp_out=self.pbn), 5.0 * n, 0),
            # Range BN backward with the bifurcated quantization of its result: 8 B/element for the
            # sums (x, dy), which also yield the range of dx, then 8 read + 4 (dx) + 1 + 2 written
            # in the second pass: the gradient is quantized where it is computed
            ("range_bn_bwd_bifurcate", lambda s: q8t.range_bn_bwd_bifurcate(
                self.y, self.dout, self.stats, None, 1e-5, 2 * s + 1, 2 * s + 2, dx_out=self.g, q8_out=self.g8,
                qp8_out=self.pg8, q16_out=self.g16, qp16_out=self.pg16), 23.0 * n, 0),
            ("qconv_dgrad", lambda s: q8t.qconv_dgrad(self.desc, self.g8, self.pg8, self.qw, self.pw, out=self.dx),
             1.0 * n + 4.0 * n, ops),
            ("qconv_wgrad", lambda s: q8t.qconv_wgrad(self.desc, self.qx, self.px, self.g16, self.pg16,
                                                      out=self.dw), 2.0 * n + 1.0 * n, ops),
        ]
        self.useful_ops = 3.0 * ops

    def step(self, s, bracket=None, ev=None):
        for name, fn, _, _ in self.calls:
            if name == bracket:
                ev[0].record()
                fn(s)
                ev[1].record()
            else:
                fn(s)


def time_calls(step, torch, iters=10):
    """average duration of every call, each timed alone with events on the launch stream"""
    out = {}
    for name, fn, _, _ in step.calls:
        fn(0)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(iters):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        out[name] = e0.elapsed_time(e1) / iters * 1e3  # microseconds
    return out


def cpu_baseline(batch, seed):
    """the oracle as it stands, on the host cores, on the same layer step at a smaller batch"""
    import numpy as np
    import oracle
    import synth
    x, w, dout = synth.conv_layer(seed=seed, N=batch)
    dout = dout * np.float32(10.0)
    d = oracle.conv_desc(batch, 64, 56, 56, 64, 3, 3, 1, 1)
    t0 = time.perf_counter()
    sx, _, px = oracle.quantize(x, 8)
    sw, _, pw = oracle.quantize(w, 8)
    y, _ = oracle.qconv_fwd(d, sx, px, sw, pw)
    _, stats, _, _ = oracle.range_bn_fwd(y, eps=1e-5, quantized=True)
    g, _, _ = oracle.range_bn_bwd(y, dout, stats, None, 1e-5)
    s8, _, p8 = oracle.quantize(g, 8, True, 1)
    s16, _, p16 = oracle.quantize(g, 16, True, 2)
    oracle.qconv_dgrad(d, s8, p8, sw, pw)
    oracle.qconv_wgrad(d, sx, px, s16, p16)
    dt = time.perf_counter() - t0
    ops = 3 * 2.0 * batch * 56 * 56 * 64 * 64 * 9
    return {"value": ops / dt / 1e12, "unit": "TOPS", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "same layer step at batch %d (%.1f s of CPU work)" % (batch, dt)}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives are part of it); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    if not os.path.exists(os.path.join(ROOT, "paper_1805_11046_amd", "libq8t.so")):
        import __graft_entry__
        __graft_entry__.build()
    import paper_1805_11046_amd as q8t

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    step = LayerStep(q8t, torch, args.batch, args.seed)
    for s in range(max(args.warmup, 1)):
        step.step(s)
    torch.cuda.synchronize()
    per_call = time_calls(step, torch)
    dominant = max(per_call, key=per_call.get)

    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        step.step(1000 + s, dominant, ev[s])
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    dom_us = sum(a.elapsed_time(b) for a, b in ev) / args.steps * 1e3

    calls = {}
    for name, _, nbytes, ops in step.calls:
        us = per_call[name]
        c = {"us": round(us, 2), "GB/s": round(nbytes / us / 1e3, 1), "hbm_frac": round(nbytes / us / 1e3 / PEAK_HBM_GBS, 3)}
        if ops:
            c["TOPS"] = round(ops / us / 1e6, 1)
            c["mfma_frac"] = round(ops / us / 1e6 / PEAK_INT8_TOPS, 4)
        calls[name] = c
    _, _, dom_bytes, dom_ops = next(c for c in step.calls if c[0] == dominant)
    # the 16x8-bit weight gradient executes two int8 products per useful one
    dom_hbm_floor = dom_bytes / PEAK_HBM_GBS / 1e3
    dom_mfma_floor = dom_ops * (2 if dominant == "qconv_wgrad" else 1) / PEAK_INT8_TOPS / 1e6
    if dom_ops and dom_mfma_floor > dom_hbm_floor:
        ach = dom_ops / dom_us / 1e6
        roofline = {"bound": "mfma", "achieved": round(ach, 2), "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                    "frac": round(ach / PEAK_INT8_TOPS, 4), "traffic": None}
    else:
        ach = dom_bytes / dom_us / 1e3
        roofline = {"bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(ach / PEAK_HBM_GBS, 4), "traffic": None}
    try:   # HBM bytes per call measured with rocprofv3 --pmc (profiles/), if recorded for this call
        with open(os.path.join(ROOT, "profiles", "hbm_traffic_layer_step.json")) as f:
            roofline["traffic"] = json.load(f).get(dominant) if args.batch == 128 else None
    except OSError:
        pass
    roofline["kernel"] = dominant
    roofline["us_per_launch"] = round(dom_us, 2)

    N, C, H, W, K = step.dims
    res = {
        "metric": "int8 qgemm TOPS (fwd/dgrad/wgrad, % MFMA peak); Range BN + quantize GB/s",
        "value": round(step.useful_ops / (ms_per_step * 1e-3) / 1e12, 3),
        "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": "resnet18 conv3x3 64->64 @56x56 batch %d: quantize + qconv fwd/dgrad/wgrad(16x8) "
                               "+ Range BN fwd/bwd on 128x64x56x56 (configs 1+2)" % N,
                   "global_batch": N, "value_is": "useful int8 ops of the three products / whole step time"},
        "roofline": roofline,
        "calls": calls,
    }
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(args.cpu_batch, args.seed)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
