"""GPU parity: FC and convolution products (forward, layer gradient, 16x8-bit weight gradient)
vs the oracle.  Integer accumulators bit-exact, float outputs within 1e-5 / 1e-6."""
import numpy as np
import pytest

import oracle
import synth
from gpu_util import same_ints, close, dev, host, qp_dev_from, require_gpu

pytestmark = pytest.mark.gpu


def _rand_q(g, shape, bits=8, zp=None):
    half = 2 ** (bits - 1)
    lv = g.integers(0, 2 ** bits, size=shape)
    zp = int(g.integers(0, 2 ** bits)) if zp is None else zp
    dt = np.int8 if bits <= 8 else np.int16
    qp = oracle.QParams(0.0, 0.0, float(np.float32(g.uniform(0.01, 0.1))), 1.0, zp, bits)
    return (lv - half).astype(dt), qp


FC_SHAPES = [(64, 128, 256), (1, 1, 1), (70, 50, 130), (5, 200, 64), (130, 65, 1000), (256, 1000, 512)]


@pytest.mark.parametrize("M,N,K", FC_SHAPES)
def test_fc_products(M, N, K):
    q8t = require_gpu()
    g = synth.rng(M * 1000 + N + K)
    sx, px = _rand_q(g, (M, K))
    sw, pw = _rand_q(g, (K, N))
    sg, pg = _rand_q(g, (M, N))
    sg16, pg16 = _rand_q(g, (M, N), bits=16)
    dpx, dpw, dpg, dpg16 = (qp_dev_from(p) for p in (px, pw, pg, pg16))
    y, acc = q8t.qgemm_fwd(dev(sx), dpx, dev(sw), dpw, want_acc=True)
    oy, oacc = oracle.qgemm_fwd(sx, px, sw, pw)
    same_ints(host(acc), oacc)
    close(host(y), oy)
    dx, acc = q8t.qgemm_dgrad(dev(sg), dpg, dev(sw), dpw, want_acc=True)
    odx, oacc = oracle.qgemm_dgrad(sg, pg, sw, pw)
    same_ints(host(acc), oacc)
    close(host(dx), odx)
    dw, acc = q8t.qgemm_wgrad(dev(sx), dpx, dev(sg16), dpg16, want_acc=True)
    odw, oacc = oracle.qgemm_wgrad(sx, px, sg16, pg16)
    same_ints(host(acc), oacc)
    close(host(dw), odw)


def test_fc_extreme_codes_do_not_overflow():
    # all codes at the far end from the zero point, reduction length at the contract's limit
    q8t = require_gpu()
    M, N, K = 16, 16, 33025
    sx = np.full((M, K), 127, np.int8)
    sw = np.full((K, N), 127, np.int8)
    px = oracle.QParams(0, 0, 1.0, 1.0, 0, 8)
    pw = oracle.QParams(0, 0, 1.0, 1.0, 0, 8)
    y, acc = q8t.qgemm_fwd(dev(sx), qp_dev_from(px), dev(sw), qp_dev_from(pw), want_acc=True)
    assert (host(acc) == 255 * 255 * K).all()
    with pytest.raises(q8t.binding.Q8TError) as e:
        q8t.qgemm_fwd(dev(np.zeros((2, K + 1), np.int8)), qp_dev_from(px), dev(np.zeros((K + 1, 2), np.int8)),
                      qp_dev_from(pw))
    assert e.value.code == -4


def test_config0_layer_step():
    # FC 64x256x128: quantize -> forward; bifurcated dY -> dgrad, wgrad; all through the C ABI
    q8t = require_gpu()
    x, w, dy = synth.fc_layer(seed=0)
    qx, px = q8t.quantize(dev(x), 8)
    qw, pw = q8t.quantize(dev(w), 8)
    g8, pg8, g16, pg16 = q8t.quantize_bifurcate(dev(dy), seed8=11, seed16=12)
    y, acc = q8t.qgemm_fwd(qx, px, qw, pw, want_acc=True)
    dx, accd = q8t.qgemm_dgrad(g8, pg8, qw, pw, want_acc=True)
    dw, accw = q8t.qgemm_wgrad(qx, px, g16, pg16, want_acc=True)
    sx, _, opx = oracle.quantize(x, 8)
    sw, _, opw = oracle.quantize(w, 8)
    s8, _, o8 = oracle.quantize(dy, 8, True, seed=11)
    s16, _, o16 = oracle.quantize(dy, 16, True, seed=12)
    oy, oacc = oracle.qgemm_fwd(sx, opx, sw, opw)
    odx, oaccd = oracle.qgemm_dgrad(s8, o8, sw, opw)
    odw, oaccw = oracle.qgemm_wgrad(sx, opx, s16, o16)
    same_ints(host(acc), oacc)
    same_ints(host(accd), oaccd)
    same_ints(host(accw), oaccw)
    close(host(y), oy)
    close(host(dx), odx)
    close(host(dw), odw)


CONV_CASES = [
    # N, C, H, W, K, R, S, stride, pad
    (2, 3, 7, 6, 4, 3, 3, 1, 1),
    (1, 2, 9, 9, 3, 3, 3, 2, 1),
    (2, 4, 5, 5, 3, 1, 1, 1, 0),
    (1, 3, 8, 8, 2, 1, 1, 2, 0),
    (1, 3, 23, 22, 5, 7, 7, 2, 3),
    (2, 64, 14, 14, 64, 3, 3, 1, 1),     # specialised-kernel shape, small
    (3, 64, 56, 56, 64, 3, 3, 1, 1),     # config-2 layer at batch 3
    (2, 128, 12, 12, 64, 3, 3, 1, 1),
    (2, 256, 10, 10, 64, 1, 1, 1, 0),    # bottleneck 1x1 reduce
    (2, 64, 10, 10, 256, 1, 1, 1, 0),    # bottleneck 1x1 expand
    (2, 64, 16, 16, 128, 3, 3, 2, 1),    # stride-2 3x3
    (2, 64, 16, 16, 128, 1, 1, 2, 0),    # stride-2 1x1 downsample
    (2, 16, 9, 9, 24, 3, 3, 1, 1),
    (1, 80, 7, 7, 72, 3, 3, 1, 1),       # channels not a multiple of 64
    (5, 32, 8, 8, 128, 3, 3, 1, 1),      # specialised weight gradient: 2 row groups, short images
    (3, 64, 28, 28, 64, 3, 3, 1, 1),
    (20, 16, 4, 8, 64, 3, 3, 1, 1),      # more images than one per workgroup, non-square
    (2, 192, 8, 12, 192, 3, 3, 1, 1),
    (1, 64, 60, 56, 64, 3, 3, 1, 1),     # last chunk of the image is ragged
    (2, 32, 30, 56, 64, 3, 3, 1, 1),     # width 56, height not a multiple of the 4 rows per staged chunk
    (2, 16, 5, 28, 128, 3, 3, 1, 1),     # width 28, image shorter than one staged chunk
    (2, 32, 5, 28, 64, 3, 3, 1, 1),      # shifted-gradient weight gradient: image shorter than one chunk
    (1, 32, 9, 28, 64, 3, 3, 1, 1),      # ... second chunk holds a single image row
    (3, 32, 3, 56, 64, 3, 3, 1, 1),      # ... width 56, three rows
    (5, 96, 8, 56, 128, 3, 3, 1, 1),     # ... three channel groups, two row groups, two whole chunks per image
    (2, 64, 56, 56, 256, 1, 1, 1, 0),    # 1x1 at the full plane size
    (40, 64, 6, 6, 64, 3, 3, 1, 1),      # one 256-row tile spans several small images
    (9, 64, 14, 14, 128, 3, 3, 1, 1),
    (3, 128, 28, 28, 128, 3, 3, 1, 1),
    (2, 64, 10, 18, 64, 3, 3, 1, 1),     # width not a multiple of 4
    # channel-contiguous general MFMA path (channels multiples of 64, shape not covered by the 3x3 / 1x1 kernels)
    (3, 128, 7, 7, 64, 3, 3, 1, 1),      # 49-position planes: byte relayout, unaligned result rows
    (2, 64, 9, 11, 128, 3, 3, 2, 1),     # odd sizes at stride 2: uneven stride classes in the layer gradient
    (2, 64, 13, 13, 64, 5, 5, 3, 2),     # stride 3, 5x5
    (1, 64, 20, 20, 64, 7, 7, 2, 3),     # 49 taps
    (2, 128, 7, 7, 128, 1, 1, 1, 0),
    (2, 64, 8, 8, 64, 2, 2, 2, 0),       # even filter size, no padding
    (130, 64, 3, 3, 64, 3, 3, 1, 1),     # many tiny images, ragged last tile
    (2, 64, 11, 9, 64, 3, 3, 2, 0),      # input rows and columns no output touches (zero layer gradient there)
    (2, 64, 9, 12, 128, 3, 3, 2, 1),     # stride 2, even width: class pairs per workgroup, odd height (uneven row parities)
    (3, 64, 14, 18, 128, 1, 1, 2, 0),    # 1x1 at stride 2: three stride classes without taps, zero-filled by the fourth
    (2, 64, 15, 16, 64, 1, 1, 2, 0),     # the same with an odd height: empty classes handled on their own
    # wide-tile kernel (3x3 stride 1, reduction channels % 64, output channels % 256 -- or % 128 on planes whose size
    # is not a multiple of 4 --, small planes)
    (3, 256, 14, 14, 256, 3, 3, 1, 1),   # 588 rows: four full tiles and a ragged one
    (5, 512, 7, 7, 512, 3, 3, 1, 1),     # 49-position planes (pieces cut out of unaligned dwords), two column tiles
    (2, 128, 14, 14, 256, 3, 3, 1, 1),   # two chunks; the layer gradient (128 outputs) stays on the 64-column kernel
    (2, 256, 9, 11, 256, 3, 3, 1, 1),    # odd plane, width 11
    (2, 256, 16, 16, 256, 3, 3, 1, 1),   # one tile = half an image
    (9, 256, 4, 4, 256, 3, 3, 1, 1),     # a tile spans eight tiny images
    (6, 256, 5, 5, 256, 3, 3, 1, 1),     # ... with unaligned planes
    (3, 64, 14, 14, 256, 3, 3, 1, 1),    # a single 64-channel chunk
    (7, 128, 7, 7, 128, 3, 3, 1, 1),     # 128-column tiles (one 32-column tile per wavefront)
    (4, 64, 7, 7, 384, 3, 3, 1, 1),      # ... three of them, one chunk
    # GEMM form of the weight gradient (byte planes x im2col rows)
    (16, 3, 32, 32, 64, 7, 7, 2, 3),     # first-layer shape: 3 input channels, 147 columns
    (8, 256, 14, 14, 256, 3, 3, 1, 1),   # 14x14 planes, 256 channels
    (16, 512, 7, 7, 512, 3, 3, 1, 1),    # 7x7 planes, 512 channels
    (24, 64, 56, 56, 64, 1, 1, 1, 0),    # reduction longer than one overflow-free slice
    (4, 3, 30, 26, 64, 7, 7, 2, 3),      # few input channels, fused forward: odd result width (scalar stores)
    (1, 4, 8, 300, 64, 3, 3, 1, 1),      # ... result rows longer than one 128-position pass
    (2, 8, 20, 20, 128, 3, 3, 1, 1),     # ... two blocks of 64 output channels
    (4, 3, 64, 64, 64, 7, 7, 2, 3),      # few input channels: weight gradient in one kernel (operands cut out in LDS)
    (8, 4, 16, 32, 64, 3, 3, 1, 1),      # ... stride 1, groups of 4 taps
    (4, 3, 32, 32, 128, 7, 7, 2, 3),     # ... two blocks of 64 output channels
    (13, 24, 17, 13, 40, 3, 2, 2, 1),    # nothing a multiple of anything; 63-position planes in groups of 4 images
    (6, 128, 7, 7, 128, 3, 3, 1, 1),     # 49-position planes, last image group incomplete
    (5, 64, 9, 10, 64, 3, 3, 1, 1),      # 90-position planes in pairs, last pair incomplete
    # weight gradient on padded 14x14 / 7x7 planes in LDS (stride 1 and 2)
    (2, 64, 28, 28, 128, 3, 3, 2, 1),    # stride 2 -> 14x14: the input plane is split into its four parity classes
    (5, 64, 14, 14, 64, 3, 3, 2, 1),     # stride 2 -> 7x7: chunks of four planes, the last one with a single image
    (40, 64, 28, 28, 64, 3, 3, 2, 1),    # one image range per image
    (37, 64, 7, 7, 64, 3, 3, 1, 1),      # ten image ranges, the last chunk incomplete
    (19, 64, 14, 14, 128, 3, 3, 1, 1),   # two row groups
    (3, 64, 28, 28, 128, 1, 1, 2, 0),    # 1x1 at stride 2 -> 14x14: one tap on the (even row, even column) class
    (6, 128, 14, 14, 64, 1, 1, 2, 0),    # 1x1 at stride 2 -> 7x7: chunks of four planes, the last one with two images
    (33, 64, 14, 14, 64, 1, 1, 2, 0),    # ... nine image ranges
    (2, 64, 56, 56, 128, 3, 3, 2, 1),    # stride 2 -> 28x28: four bands of 8 rows per plane, the last one half empty
    (5, 128, 56, 56, 64, 3, 3, 2, 1),    # ... two channel groups, image ranges of unequal length
    (3, 128, 56, 56, 64, 1, 1, 2, 0),    # ... one tap
    # forward with few input channels: explicit im2col rows + GEMM
    (4, 16, 20, 20, 128, 3, 3, 1, 1),    # 144 columns -> 192, 128-wide tiles
    (8, 5, 30, 17, 64, 5, 3, 2, 2),      # non-square filter, stride 2, 75 columns -> 128
    # forward with few input channels and 64 output channels: fragments read from a staged band of input rows
    (3, 2, 20, 24, 64, 5, 5, 3, 2),      # stride 3, 10 groups of 5 taps (two K-steps), ragged last band
    (2, 1, 12, 16, 64, 3, 8, 1, 0),      # one channel, rows of 8 taps, no padding (a single K-step)
    (2, 6, 40, 40, 64, 5, 3, 1, 1),      # 30 groups (four K-steps), 40 positions per row: a ragged last tile
    (1, 3, 224, 224, 64, 7, 7, 2, 3),    # the first layer of a ResNet at its real plane size
    # 1x1 with a stride, no padding: forward as the stride-1 layer on the gathered positions
    (3, 64, 56, 56, 128, 1, 1, 2, 0),    # rows of a multiple of 8 codes: gathered with byte permutes
    (2, 64, 20, 12, 64, 1, 1, 2, 0),     # ... scalar gather
    (2, 64, 17, 29, 128, 1, 1, 3, 0),    # stride 3, sizes that are no multiples of it (6 x 10 positions)
]


def _conv_operands(g, case):
    N, C, H, W, K, R, S, st, pad = case
    od = oracle.conv_desc(*case)
    sx, px = _rand_q(g, (N, C, H, W))
    sw, pw = _rand_q(g, (K, C, R, S))
    sg, pg = _rand_q(g, (N, K, od.P, od.Q))
    sg16, pg16 = _rand_q(g, (N, K, od.P, od.Q), bits=16)
    return od, (sx, px), (sw, pw), (sg, pg), (sg16, pg16)


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_products(case):
    q8t = require_gpu()
    g = synth.rng(sum(case))
    od, (sx, px), (sw, pw), (sg, pg), (sg16, pg16) = _conv_operands(g, case)
    d = q8t.conv_desc(*case)
    dpx, dpw, dpg, dpg16 = (qp_dev_from(p) for p in (px, pw, pg, pg16))
    y, acc = q8t.qconv_fwd(d, dev(sx), dpx, dev(sw), dpw, want_acc=True)
    oy, oacc = oracle.qconv_fwd(od, sx, px, sw, pw)
    same_ints(host(acc), oacc)
    close(host(y), oy)
    dx, acc = q8t.qconv_dgrad(d, dev(sg), dpg, dev(sw), dpw, want_acc=True)
    odx, oacc = oracle.qconv_dgrad(od, sg, pg, sw, pw)
    same_ints(host(acc), oacc)
    close(host(dx), odx)
    dw, acc = q8t.qconv_wgrad(d, dev(sx), dpx, dev(sg16), dpg16, want_acc=True)
    odw, oacc = oracle.qconv_wgrad(od, sx, px, sg16, pg16)
    same_ints(host(acc), oacc)
    close(host(dw), odw)


@pytest.mark.parametrize("case", [(2, 64, 14, 14, 64, 3, 3, 1, 1), (2, 64, 9, 11, 128, 3, 3, 2, 1),
                                  (2, 16, 9, 9, 24, 3, 3, 1, 1), (2, 64, 10, 10, 128, 1, 1, 1, 0),
                                  (2, 3, 16, 16, 64, 7, 7, 2, 3)])
def test_conv_products_below_8_and_16_bits(case):
    # widths M < 8 (and < 16 for the weight-gradient operand) are stored as level - 2^(M-1) in the
    # same containers; every kernel family has to take the stored zero point from the width
    q8t = require_gpu()
    g = synth.rng(77 + sum(case))
    N, C, H, W, K, R, S, st, pad = case
    od = oracle.conv_desc(*case)
    sx, px = _rand_q(g, (N, C, H, W), bits=5)
    sw, pw = _rand_q(g, (K, C, R, S), bits=4)
    sg, pg = _rand_q(g, (N, K, od.P, od.Q), bits=6)
    sg16, pg16 = _rand_q(g, (N, K, od.P, od.Q), bits=12)
    d = q8t.conv_desc(*case)
    dpx, dpw, dpg, dpg16 = (qp_dev_from(p) for p in (px, pw, pg, pg16))
    y, acc = q8t.qconv_fwd(d, dev(sx), dpx, dev(sw), dpw, want_acc=True)
    oy, oacc = oracle.qconv_fwd(od, sx, px, sw, pw)
    same_ints(host(acc), oacc)
    close(host(y), oy)
    dx, acc = q8t.qconv_dgrad(d, dev(sg), dpg, dev(sw), dpw, want_acc=True)
    odx, oacc = oracle.qconv_dgrad(od, sg, pg, sw, pw)
    same_ints(host(acc), oacc)
    close(host(dx), odx)
    dw, acc = q8t.qconv_wgrad(d, dev(sx), dpx, dev(sg16), dpg16, want_acc=True)
    odw, oacc = oracle.qconv_wgrad(od, sx, px, sg16, pg16)
    same_ints(host(acc), oacc)
    close(host(dw), odw)


def test_conv_float_only_and_acc_only_outputs_agree():
    q8t = require_gpu()
    case = (2, 64, 14, 14, 64, 3, 3, 1, 1)
    g = synth.rng(5)
    od, (sx, px), (sw, pw), _, _ = _conv_operands(g, case)
    d = q8t.conv_desc(*case)
    dpx, dpw = qp_dev_from(px), qp_dev_from(pw)
    y1, acc1 = q8t.qconv_fwd(d, dev(sx), dpx, dev(sw), dpw, want_acc=True)
    y2, _ = q8t.qconv_fwd(d, dev(sx), dpx, dev(sw), dpw, want_acc=False)
    assert np.array_equal(host(y1), host(y2))
