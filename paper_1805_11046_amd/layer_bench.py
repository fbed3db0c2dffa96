"""Per-layer timing of the three products on the conv shapes of the workloads
(ResNet-18 at batch 256, the ResNet-50 bottleneck at batch 128).

    python -m paper_1805_11046_amd.layer_bench                 # table over all shapes
    python -m paper_1805_11046_amd.layer_bench l3 l4           # shapes whose name contains a word
    python -m paper_1805_11046_amd.layer_bench --case 256,256,14,14,256,3,3,1,1 --which wgrad --reps 3
                                                               # a few calls of one product (for profilers)

Operands are random codes already resident in HBM; times are hipEvent averages over back-to-back
calls (the Infinity Cache keeps small operands between calls, see the bandwidth notes of the
project documentation).  Needs a GPU.
"""
import argparse

import torch

from . import binding as q8t

SHAPES = [
    ("c2 3x3 64->64 @56 b128", (128, 64, 56, 56, 64, 3, 3, 1, 1)),
    ("c3a 1x1 256->64 @56 b128", (128, 256, 56, 56, 64, 1, 1, 1, 0)),
    ("c3c 1x1 64->256 @56 b128", (128, 64, 56, 56, 256, 1, 1, 1, 0)),
    ("c4 conv1 7x7/2 3->64 b256", (256, 3, 224, 224, 64, 7, 7, 2, 3)),
    ("c4 l1 3x3 64->64 @56 b256", (256, 64, 56, 56, 64, 3, 3, 1, 1)),
    ("c4 l2 3x3 128->128 @28", (256, 128, 28, 28, 128, 3, 3, 1, 1)),
    ("c4 l3 3x3 256->256 @14", (256, 256, 14, 14, 256, 3, 3, 1, 1)),
    ("c4 l4 3x3 512->512 @7", (256, 512, 7, 7, 512, 3, 3, 1, 1)),
    ("c4 3x3/2 64->128 @56", (256, 64, 56, 56, 128, 3, 3, 2, 1)),
    ("c4 3x3/2 128->256 @28", (256, 128, 28, 28, 256, 3, 3, 2, 1)),
    ("c4 3x3/2 256->512 @14", (256, 256, 14, 14, 512, 3, 3, 2, 1)),
    ("c4 1x1/2 64->128 @56", (256, 64, 56, 56, 128, 1, 1, 2, 0)),
    ("c4 1x1/2 128->256 @28", (256, 128, 28, 28, 256, 1, 1, 2, 0)),
    ("c4 1x1/2 256->512 @14", (256, 256, 14, 14, 512, 1, 1, 2, 0)),
]


def _timeit(fn, iters, warm):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters * 1e3


class Layer:
    def __init__(self, case, dev):
        N, C, H, W, K, R, S, st, pad = case
        self.d = q8t.conv_desc(*case)
        P, Q = self.d.P, self.d.Q
        self.ops = 2.0 * N * P * Q * K * C * R * S
        ri = lambda lo, hi, shape, dt: torch.randint(lo, hi, shape, dtype=dt, device=dev)
        self.x = ri(-128, 127, (N, C, H, W), torch.int8)
        self.w = ri(-128, 127, (K, C, R, S), torch.int8)
        self.g8 = ri(-128, 127, (N, K, P, Q), torch.int8)
        self.g16 = ri(-32768, 32767, (N, K, P, Q), torch.int16)
        f = torch.randn(1024, device=dev)
        _, self.px = q8t.quantize(f, 8)
        _, self.pw = q8t.quantize(f * 0.1, 8)
        _, self.pg = q8t.quantize(f * 1e-3, 8, True, 1)
        _, self.pg16 = q8t.quantize(f * 1e-3, 16, True, 2)
        self.y = torch.empty((N, K, P, Q), device=dev)
        self.dx = torch.empty((N, C, H, W), device=dev)
        self.dw = torch.empty((K, C, R, S), device=dev)

    def fwd(self):
        q8t.qconv_fwd(self.d, self.x, self.px, self.w, self.pw, out=self.y)

    def dgrad(self):
        q8t.qconv_dgrad(self.d, self.g8, self.pg, self.w, self.pw, out=self.dx)

    def wgrad(self):
        q8t.qconv_wgrad(self.d, self.x, self.px, self.g16, self.pg16, out=self.dw)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("words", nargs="*")
    ap.add_argument("--case", default=None)
    ap.add_argument("--which", default="fwd", choices=["fwd", "dgrad", "wgrad"])
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--iters", type=int, default=5)
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    if args.case:
        L = Layer(tuple(int(v) for v in args.case.split(",")), dev)
        for _ in range(args.reps):
            getattr(L, args.which)()
        torch.cuda.synchronize()
        return
    for name, case in SHAPES:
        if args.words and not any(w in name for w in args.words):
            continue
        if name.startswith("c4 conv1"):
            L = Layer(case, dev)
            t = [_timeit(L.fwd, args.iters, 2), float("nan"), _timeit(L.wgrad, args.iters, 2)]   # the input needs no gradient
        else:
            L = Layer(case, dev)
            t = [_timeit(L.fwd, args.iters, 2), _timeit(L.dgrad, args.iters, 2), _timeit(L.wgrad, args.iters, 2)]
        print("%-28s %6.1f GOP  fwd %8.1f us %7.1f TOPS | dgrad %8.1f us %7.1f TOPS | wgrad %8.1f us %7.1f TOPS"
              % (name, L.ops / 1e9, t[0], L.ops / t[0] / 1e6, t[1], L.ops / t[1] / 1e6, t[2], L.ops / t[2] / 1e6), flush=True)
        del L


if __name__ == "__main__":
    main()
