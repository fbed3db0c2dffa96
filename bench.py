"""Benchmark of the 8-bit training hot path on one MI355X.

Headline workload: one synthetic ResNet-18 training step at batch 256 (3x224x224 inputs ~N(0,1),
He-normal weights, 1000 classes, random labels; forward + backward, no optimizer update).  Every
conv / FC product runs through the library as an 8-bit forward, an 8-bit layer gradient and a
16x8-bit weight gradient, every batch-norm is Range BN (statistics from the conv epilogue, fused
with ReLU / the next operand's quantization / the bifurcated gradient quantization where the graph
allows); ReLU, pooling, residual additions and the loss are elementwise glue outside the method
and run in torch.  One "step" = that whole pass.  All inputs are resident in HBM before the timed
region.

`value` = useful int8 operations of all products of the step (2 x multiply-accumulates; the weight
gradient counted once although it executes two byte-plane products) / whole step time.
`calls` lists every library entry point as timed IN SEQUENCE inside the step (events on the launch
stream around each call, every call starting on cold caches), per layer for the products.
`roofline` is the entry point with the largest share of the step, timed the same way inside the
timed region.  `stream_ceiling` is what a plain copy / read kernel reaches on this machine on tensors of
the step's size, rotating over buffers so that nothing is found in the Infinity Cache.
`layer_step` is the single-layer step of the smaller workloads (3x3 conv 64->64 @56x56, batch 128,
with the Range BN of that shape), timed the same way.
Prints ONE JSON line.
"""
import argparse
import collections
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
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-batches", type=int, nargs=2, default=(16, 32),
                    help="the two batch sizes at which the oracle is timed")
    ap.add_argument("--no-layer-step", action="store_true")
    ap.add_argument("--no-second-stream", action="store_true",
                    help="skip the extra run with the weight gradients on a second stream (profiles trace the headline only)")
    return ap.parse_args()


# --------------------------------------------------------------------------- ResNet-18 step
def executed_factor(name):
    """int8 MFMA operations executed per useful operation: the 16-bit operand of the weight gradient
    is two byte planes"""
    return 2.0 if "wgrad" in name else 1.0


def summarize_calls(records, steps):
    """records: (name, tag, ops, bytes, us) of `steps` whole steps -> per entry point and per layer"""
    by = collections.OrderedDict()
    for name, tag, ops, nbytes, us in records:
        e = by.setdefault(name, {"launches": 0, "us": 0.0, "ops": 0.0, "bytes": 0.0, "floor_us": 0.0, "layers": {}})
        e["launches"] += 1
        e["us"] += us
        e["ops"] += ops
        e["bytes"] += nbytes
        floor = max(nbytes / PEAK_HBM_GBS / 1e3, ops * executed_factor(name) / PEAK_INT8_TOPS / 1e6)
        e["floor_us"] += floor
        if ops and tag:
            l = e["layers"].setdefault(tag, {"launches": 0, "us": 0.0, "ops": 0.0, "bytes": 0.0, "floor_us": 0.0})
            l["launches"] += 1
            l["us"] += us
            l["ops"] += ops
            l["bytes"] += nbytes
            l["floor_us"] += floor

    def fmt(e):
        us = e["us"] / steps
        out = {"launches": e["launches"] // steps, "us": round(us, 1),
               "GB/s": round(e["bytes"] / steps / us / 1e3, 1),
               "hbm_frac": round(e["bytes"] / steps / us / 1e3 / PEAK_HBM_GBS, 3)}
        if e["ops"]:
            out["TOPS"] = round(e["ops"] / steps / us / 1e6, 1)
            out["mfma_frac"] = round(e["ops"] / steps / us / 1e6 / PEAK_INT8_TOPS, 4)
            # share of the time that the binding roof (HBM or int8 MFMA, per launch) accounts for
            out["binding_roof_frac"] = round(e["floor_us"] / e["us"], 3)
        return out

    calls = {}
    for name, e in by.items():
        c = fmt(e)
        if e["layers"]:
            c["layers"] = {tag: fmt(l) for tag, l in e["layers"].items()}
        calls[name] = c
    return calls, by


def roofline_of(name, records, steps):
    """algorithmic bytes or operations per launch / average launch duration of one entry point"""
    recs = [r for r in records if r[0] == name]
    us = sum(r[4] for r in recs)
    ops = sum(r[2] for r in recs) * executed_factor(name)
    nbytes = sum(r[3] for r in recs)
    launches = len(recs)
    if ops / PEAK_INT8_TOPS / 1e6 > nbytes / PEAK_HBM_GBS / 1e3:
        ach = ops / us / 1e6
        roof = {"bound": "mfma", "achieved": round(ach, 1), "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                "frac": round(ach / PEAK_INT8_TOPS, 4), "traffic": None,
                "per_launch": {"ops_executed": round(ops / launches), "us": round(us / launches, 2)}}
    else:
        ach = nbytes / us / 1e3
        roof = {"bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(ach / PEAK_HBM_GBS, 4), "traffic": None,
                "per_launch": {"bytes": round(nbytes / launches), "us": round(us / launches, 2)}}
    roof["kernel"] = name
    roof["launches_per_step"] = launches // steps
    roof["us_per_step"] = round(us / steps, 1)
    roof["per_launch"]["algorithmic_bytes"] = round(nbytes / launches)
    roof["traffic"], src = measured_traffic(name, launches // steps)
    if src:
        roof["traffic_source"] = src
    return roof


def measured_traffic(name, launches_per_step):
    """HBM bytes per launch from the committed counter summary of this same workload (two rocprofv3 --pmc runs,
    calibrated on the copy kernel); None where the summary has no entry for the call or the batch is another one"""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic_resnet18_b256.json")
    try:
        with open(path) as f:
            table = json.load(f)
    except (OSError, ValueError):
        return None, None
    src = "profiles/hbm_traffic_resnet18_b256.json, measured at commit %s" % table.get("_measured_at_commit", "?")
    for key, per_step in table.items():
        if key.startswith("_") or key.endswith("_factor"):
            continue
        names = [k.strip() for k in key.replace("(+relu)", "").split("+")]
        if name in names and len(names) == 1:
            return round(per_step / launches_per_step), src
    return None, None


def resnet18(torch, batch, seed):
    from paper_1805_11046_amd import train_step as ts
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    ws = ts.make_weights(dev, gen)
    x = torch.randn((batch, 3, 224, 224), device=dev, generator=gen)
    labels = torch.randint(0, 1000, (batch,), device=dev, generator=gen)
    params = [ws["conv1"], ws["fc"]] + [w for b in ws["blocks"] for w in b.values()]

    def one():
        for p in params:
            p.grad = None
        return ts.step(x, labels, ws)

    return ts, one, params


# --------------------------------------------------------------------------- measured streaming ceiling
def stream_ceiling(q8t, torch, nbytes=102760448, sets=6, rounds=3):
    """plain copy / read kernels on buffers of one activation tensor's size (128x64x56x56 fp32),
    rotating over `sets` buffer pairs (1.2 GB) so that every launch starts cold"""
    dev = torch.device("cuda:0")
    src = [torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(sets)]
    dst = [torch.empty(nbytes, dtype=torch.uint8, device=dev) for _ in range(sets)]
    out = {}
    for mode, key, moved in ((0, "copy", 2.0 * nbytes), (1, "read", 1.0 * nbytes)):
        for i in range(sets):
            q8t.probe_stream(mode, src[i], dst[i], nbytes)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for r in range(rounds):
            for i in range(sets):
                q8t.probe_stream(mode, src[i], dst[i], nbytes)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / (rounds * sets)
        out[key] = {"GB/s": round(moved / us / 1e3, 1), "frac_of_peak": round(moved / us / 1e3 / PEAK_HBM_GBS, 3),
                    "us": round(us, 2)}
    out["what"] = "%d MB per buffer, %d buffer pairs in rotation, %d launches each" % (nbytes // 1000000, sets, rounds * sets)
    return out


# --------------------------------------------------------------------------- single-layer step
class LayerStep:
    """Buffers and the call sequence of one layer step (3x3 conv 64->64 @56x56 with its Range BN).
    Every call goes through the C ABI."""

    def __init__(self, q8t, torch, batch, seed):
        dev = torch.device("cuda:0")
        N, C, H, W, K = batch, 64, 56, 56, 64
        self.dims = (N, C, H, W, K)
        g = torch.Generator(device=dev)
        g.manual_seed(seed)
        # |N(0,1)| activations (post-ReLU), He-normal weights (var 2/576), N(0, sigma 1e-2) upstream gradient
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
            # the normalized output leaves as 8-bit codes with the analytic range (4 read + 1 written)
            ("range_bn_fwd_apply", lambda s: q8t.range_bn_fwd_apply(self.y, self.stats, None, None, 1e-5,
                                                                    quantized=True, want_y=False, q_out=self.bnq,
                                                                    qp_out=self.pbn), 5.0 * n, 0),
            # Range BN backward with the bifurcated quantization of its result: 8 B/element for the
            # sums (x, dy), which also yield the range of dx, then 8 read + 4 (dx) + 1 + 2 written
            ("range_bn_bwd_bifurcate", lambda s: q8t.range_bn_bwd_bifurcate(
                self.y, self.dout, self.stats, None, 1e-5, 2 * s + 1, 2 * s + 2, dx_out=self.g, q8_out=self.g8,
                qp8_out=self.pg8, q16_out=self.g16, qp16_out=self.pg16), 23.0 * n, 0),
            ("qconv_dgrad", lambda s: q8t.qconv_dgrad(self.desc, self.g8, self.pg8, self.qw, self.pw, out=self.dx),
             1.0 * n + 4.0 * n, ops),
            ("qconv_wgrad", lambda s: q8t.qconv_wgrad(self.desc, self.qx, self.px, self.g16, self.pg16,
                                                      out=self.dw), 2.0 * n + 1.0 * n, ops),
        ]
        self.useful_ops = 3.0 * ops

    def step(self, s, events=None):
        for i, (name, fn, _, _) in enumerate(self.calls):
            if events is not None:
                events[i][0].record()
                fn(s)
                events[i][1].record()
            else:
                fn(s)


def layer_step_record(q8t, torch, seed, steps=20, warmup=3):
    step = LayerStep(q8t, torch, 128, seed)
    for s in range(warmup):
        step.step(s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        step.step(100 + s)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    # per call, in sequence: events around every call of every step
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in step.calls]
          for _ in range(steps)]
    for s in range(steps):
        step.step(200 + s, ev[s])
    torch.cuda.synchronize()
    calls = {}
    for i, (name, _, nbytes, ops) in enumerate(step.calls):
        us = sum(ev[s][i][0].elapsed_time(ev[s][i][1]) for s in range(steps)) / steps * 1e3
        c = {"us": round(us, 2), "GB/s": round(nbytes / us / 1e3, 1), "hbm_frac": round(nbytes / us / 1e3 / PEAK_HBM_GBS, 3)}
        if ops:
            c["TOPS"] = round(ops / us / 1e6, 1)
            c["mfma_frac"] = round(ops / us / 1e6 / PEAK_INT8_TOPS, 4)
        calls[name] = c
    return {"workload": "3x3 conv 64->64 @56x56 batch 128: quantize + qconv fwd/dgrad/wgrad(16x8) + Range BN fwd/bwd "
                        "on 128x64x56x56",
            "ms_per_step": round(ms, 4), "TOPS": round(step.useful_ops / (ms * 1e-3) / 1e12, 1),
            "calls_in_sequence": calls}


# --------------------------------------------------------------------------- CPU baseline (oracle)
RESNET18_CONVS = [(3, 224, 64, 7, 2, 3, 1)] + [
    # (Cin, H, Cout, R, stride, pad, how many such layers)
    (64, 56, 64, 3, 1, 1, 4),
    (64, 56, 128, 3, 2, 1, 1), (128, 28, 128, 3, 1, 1, 3), (64, 56, 128, 1, 2, 0, 1),
    (128, 28, 256, 3, 2, 1, 1), (256, 14, 256, 3, 1, 1, 3), (128, 28, 256, 1, 2, 0, 1),
    (256, 14, 512, 3, 2, 1, 1), (512, 7, 512, 3, 1, 1, 3), (256, 14, 512, 1, 2, 0, 1),
]


def cpu_baseline(batches, seed):
    """The oracle as it stands on the host cores: every conv layer and the FC layer of ResNet-18, each as
    one layer step of the method (quantize X and W, forward product, Range BN forward and backward,
    the two stochastic copies of the gradient, layer gradient, weight gradient) on synthetic inputs
    of its shape, at two small batch sizes.  The glue between layers is not part of the method and
    is left out.  Throughput in useful int8 operations does not depend on the batch, so the value
    at the larger batch stands for the full batch; both are reported."""
    import numpy as np
    import oracle
    import synth

    def run(batch):
        total_ops, total_t = 0.0, 0.0
        for (cin, h, cout, r, st, pad, count) in RESNET18_CONVS:
            x, w, dy = synth.conv_layer(seed=seed, N=batch, C=cin, H=h, W=h, K=cout, R=r, S=r, stride=st, pad=pad,
                                        relu_input=cin != 3)
            dy = dy * np.float32(10.0)
            d = oracle.conv_desc(batch, cin, h, h, cout, r, r, st, pad)
            t0 = time.perf_counter()
            sx, _, px = oracle.quantize(x, 8)
            sw, _, pw = oracle.quantize(w, 8)
            y, _ = oracle.qconv_fwd(d, sx, px, sw, pw)
            _, stats, _, _ = oracle.range_bn_fwd(y, eps=1e-5)
            g, _, _ = oracle.range_bn_bwd(y, dy, stats, None, 1e-5)
            s8, _, p8 = oracle.quantize(g, 8, True, 1)
            s16, _, p16 = oracle.quantize(g, 16, True, 2)
            n_products = 2
            if cin != 3:   # the network input has no gradient
                oracle.qconv_dgrad(d, s8, p8, sw, pw)
                n_products = 3
            oracle.qconv_wgrad(d, sx, px, s16, p16)
            total_t += (time.perf_counter() - t0) * count
            total_ops += n_products * 2.0 * batch * d.P * d.Q * cout * cin * r * r * count
        g = synth.rng(seed + 1)
        x = np.abs(synth.normal(g, (batch, 512), std=1.0))
        w = synth.normal(g, (512, 1000), std=(2.0 / 512) ** 0.5)
        dy = synth.normal(g, (batch, 1000), std=1e-3)
        t0 = time.perf_counter()
        sx, _, px = oracle.quantize(x, 8)
        sw, _, pw = oracle.quantize(w, 8)
        oracle.qgemm_fwd(sx, px, sw, pw)
        s8, _, p8 = oracle.quantize(dy, 8, True, 1)
        s16, _, p16 = oracle.quantize(dy, 16, True, 2)
        oracle.qgemm_dgrad(s8, p8, sw, pw)
        oracle.qgemm_wgrad(sx, px, s16, p16)
        total_t += time.perf_counter() - t0
        total_ops += 3 * 2.0 * batch * 512 * 1000
        return total_ops, total_t

    res = [run(b) for b in batches]
    (o0, t0), (o1, t1) = res
    return {"value": round(o1 / t1 / 1e12, 5), "unit": "TOPS", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "all 20 conv layers + FC of ResNet-18, each as one layer step of the method on synthetic inputs "
                      "of its shape (no glue; a shape that occurs k times is timed once and counted k times), at batch %d (%.1f s, %.4f TOPS) and batch %d (%.1f s, %.4f TOPS); "
                      "time is linear in the batch, so batch 256 extrapolates to %.0f s at the same TOPS"
                      % (batches[0], t0, o0 / t0 / 1e12, batches[1], t1, o1 / t1 / 1e12, t1 * 256.0 / batches[1])}


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
    ts, one, params = resnet18(torch, args.batch, args.seed)
    for _ in range(max(args.warmup, 1)):
        loss = one()
    torch.cuda.synchronize()

    # every library call timed in sequence, to find the entry point with the largest share.  Three
    # steps are recorded and the one with the smallest total is reported: a step now and then carries
    # a stall of several ms in one call (the allocator behind the glue returning memory to the driver)
    ts.record(breakdown=True)
    one()            # one untimed step in this mode: its events and buffers exist afterwards
    ts.drain()
    per_step = []
    for _ in range(3):
        one()
        per_step.append(ts.drain())
    ts.record()
    records = min(per_step, key=lambda r: sum(x[4] for x in r))
    calls, by = summarize_calls(records, 1)
    dominant = max(by, key=lambda k: by[k]["us"])
    useful_ops = sum(r[2] for r in records)
    library_ms = sum(r[4] for r in records) / 1e3

    # the timed region: K whole steps; only the dominant entry point carries events
    ts.record(bracket=dominant)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        loss = one()
    issue = time.perf_counter() - t0   # the host has queued every launch; the GPU is still working
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    dom_records = ts.drain()
    ts.record()
    assert bool(torch.isfinite(loss)) and all(p.grad is not None for p in params)
    ms_per_step = dt / args.steps * 1e3
    roofline = roofline_of(dominant, dom_records, args.steps)

    # the same K steps with the weight gradients on a second stream (nothing downstream needs them before the optimizer):
    # reported beside the headline, which keeps one stream so that the events around the dominant entry point time that
    # entry point alone
    ms_overlap = None
    if not args.no_second_stream:
        ts._overlap = True
        for _ in range(2):
            one()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            loss2 = one()
        torch.cuda.synchronize()
        ms_overlap = (time.perf_counter() - t0) / args.steps * 1e3
        ts._overlap = False
        assert bool(torch.isfinite(loss2))
    if args.batch != 256:
        roofline["traffic"] = None   # the counter summary is of the batch-256 step
        roofline.pop("traffic_source", None)

    res = {
        "metric": "int8 qgemm TOPS (fwd/dgrad/wgrad, % MFMA peak); Range BN + quantize GB/s",
        "value": round(useful_ops / (ms_per_step * 1e-3) / 1e12, 3),
        "unit": "TOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": "ResNet-18 training step (forward + backward), batch %d, 3x224x224 inputs, every conv/FC as "
                               "8-bit fwd / 8-bit dgrad / 16x8-bit wgrad and every BN as Range BN (config 4)" % args.batch,
                   "global_batch": args.batch,
                   "value_is": "useful int8 ops of all products of the step / whole step time (glue in torch included)",
                   "images_per_s": round(args.batch / ms_per_step * 1e3, 1),
                   "library_calls_ms_per_step": round(library_ms, 3),
                   "host_issue_ms_per_step": round(issue / args.steps * 1e3, 3),
                   "wgrad_on_second_stream": None if ms_overlap is None else {
                       "ms_per_step": round(ms_overlap, 4),
                       "TOPS": round(useful_ops / (ms_overlap * 1e-3) / 1e12, 3),
                       "what": "same step and step count, weight gradients issued on a second stream; not the headline"}},
        "roofline": roofline,
        "calls": calls,
        "stream_ceiling": stream_ceiling(q8t, torch),
    }
    if not args.no_layer_step:
        res["layer_step"] = layer_step_record(q8t, torch, args.seed)
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(tuple(args.cpu_batches), args.seed)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
