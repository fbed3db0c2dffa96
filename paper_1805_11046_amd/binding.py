"""Thin ctypes binding over libq8t.so (the C ABI declared in include/q8t.h).

Argument marshalling only: torch supplies device memory and the current stream, every step of
the method runs in the library's HIP kernels.  There is no CPU fallback: if the library is not
built the import fails.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libq8t.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libq8t.so is not built (%s): run `python -c 'import __graft_entry__ as g; g.build()'` "
        "or `python paper_1805_11046_amd/build.py`" % LIB_PATH)

_lib = C.CDLL(LIB_PATH)

ERRORS = {-1: "Q8T_ERR_NULL", -2: "Q8T_ERR_SHAPE", -3: "Q8T_ERR_BITS", -4: "Q8T_ERR_OVERFLOW",
          -5: "Q8T_ERR_WORKSPACE", -6: "Q8T_ERR_HIP"}


class Q8TError(RuntimeError):
    def __init__(self, code, where):
        super().__init__("%s failed: %s (%d)" % (where, ERRORS.get(code, "?"), code))
        self.code = code


class ConvDesc(C.Structure):
    """q8t_conv_desc: input [N,C,H,W], filter [K,C,R,S]."""
    _fields_ = [(k, C.c_int) for k in ("N", "C", "H", "W", "K", "R", "S", "stride", "pad")]

    @property
    def P(self):
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self):
        return (self.W + 2 * self.pad - self.S) // self.stride + 1


QPARAMS_BYTES = 24
_vp, _i, _i64, _u64, _f, _sz = C.c_void_p, C.c_int, C.c_int64, C.c_uint64, C.c_float, C.c_size_t

_SIGS = {
    "q8t_quantize_workspace_size": (_sz, [_i64]),
    "q8t_quantize": (_i, [_vp, _i64, _i, _i, _u64, _vp, _vp, _vp, _vp]),
    "q8t_quantize_multi_workspace_size": (_sz, [_i, _vp]),
    "q8t_quantize_multi": (_i, [_i, _vp, _vp, _i, _vp, _vp, _vp, _vp]),
    "q8t_init": (_i, []),
    "q8t_quantize_noalloc": (_i, [_vp, _i64, _i, _i, _u64, _vp, _vp, _vp]),
    "q8t_quantize_with_range": (_i, [_vp, _i64, _i, _i, _u64, _vp, _vp, _vp, _vp]),
    "q8t_quantize_bifurcate": (_i, [_vp, _i64, _u64, _u64, _vp, _vp, _vp, _vp, _vp, _vp]),
    "q8t_dequantize": (_i, [_vp, _vp, _i64, _vp, _vp]),
    "q8t_qgemm_workspace_size": (_sz, [_i, _i, _i, _i]),
    "q8t_qgemm_fwd": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _vp, _vp, _vp, _vp]),
    "q8t_qgemm_dgrad": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _vp, _vp, _vp, _vp]),
    "q8t_qgemm_wgrad": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _vp, _vp, _vp, _vp]),
    "q8t_qconv_workspace_size": (_sz, [C.POINTER(ConvDesc), _i]),
    "q8t_qconv_fwd": (_i, [C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "q8t_qconv_dgrad": (_i, [C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "q8t_qconv_dgrad_relu_sum": (_i, [C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "q8t_qconv_wgrad": (_i, [C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "q8t_qconv_pack_size": (_sz, [C.POINTER(ConvDesc), _i]),
    "q8t_qconv_pack_multi": (_i, [_i, C.POINTER(ConvDesc), C.POINTER(C.c_int), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), _vp]),
    "q8t_qconv_fwd_bn_stats_packed": (_i, [C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "q8t_qconv_dgrad_packed": (_i, [C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "q8t_qconv_dgrad_relu_sum_packed": (_i, [C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "q8t_range_bn_workspace_size": (_sz, [_i, _i, _i, _i]),
    "q8t_range_bn_fwd": (_i, [_vp, _i, _i, _i, _i, _vp, _vp, _f, _vp, _vp, _vp, _vp, _vp, _vp]),
    "q8t_range_bn_bwd": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _vp, _f, _vp, _vp, _vp, _vp, _vp]),
    "q8t_chunk_range_workspace_size": (_sz, [_i64, _i]),
    "q8t_chunk_range": (_i, [_vp, _i64, _i, _vp, _vp, _vp]),
    "q8t_quant_angle_workspace_size": (_sz, [_i64]),
    "q8t_quant_angle": (_i, [_vp, _vp, _vp, _i64, _vp, _vp, _vp]),
    "q8t_qconv_fwd_bn_stats_workspace_size": (_sz, [C.POINTER(ConvDesc)]),
    "q8t_qconv_fwd_bn_stats": (_i, [C.POINTER(ConvDesc), _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "q8t_range_bn_fwd_apply": (_i, [_vp, _i, _i, _i, _i, _vp, _vp, _f, _vp, _vp, _vp, _vp, _vp]),
    "q8t_range_bn_relu_fwd_apply": (_i, [_vp, _i, _i, _i, _i, _vp, _vp, _f, _vp, _vp, _vp, _vp, _vp]),
    "q8t_range_bn_relu_bwd_bifurcate": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _vp, _vp, _f, _vp, _vp, _vp, _u64, _u64, _vp,
                                              _vp, _vp, _vp, _vp, _vp]),
    "q8t_range_bn_bwd_bifurcate_workspace_size": (_sz, [_i, _i, _i, _i]),
    "q8t_range_bn_bwd_bifurcate": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _vp, _f, _vp, _vp, _vp, _u64, _u64, _vp, _vp,
                                        _vp, _vp, _vp, _vp]),
    "q8t_probe_stream": (_i, [_i, _vp, _vp, _i64, _vp]),
    "q8t_range_bn_relu_maxpool_fwd": (_i, [_vp, _i, _i, _i, _i, _vp, _vp, _f, _vp, _vp, _vp, _vp]),
    "q8t_maxpool_relu_bwd": (_i, [_vp, _vp, _i, _i, _i, _i, _vp, _vp]),
    "q8t_maxpool_range_bn_bwd_bifurcate_workspace_size": (_sz, [_i, _i, _i, _i]),
    "q8t_maxpool_range_bn_bwd_bifurcate": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _vp, _f, _vp, _vp, _u64, _u64, _vp, _vp,
                                                _vp, _vp, _vp, _vp]),
    "q8t_add_relu_quantize_workspace_size": (_sz, [_i64]),
    "q8t_add_relu_quantize": (_i, [_vp, _vp, _i64, _vp, _vp, _vp, _vp, _vp]),
    "q8t_range_bn_add_relu_quantize": (_i, [_vp] * 8 + [_i, _i, _i, _i, _f, _vp, _vp, _vp, _vp, _vp]),
    "q8t_relu_bwd_add": (_i, [_vp, _vp, _vp, _i64, _vp, _vp]),
    "q8t_relu_bwd_sum": (_i, [_vp, _vp, _vp, _i64, _vp, _vp]),
    "q8t_relu_bwd_sum_lattice": (_i, [_vp, _vp, _vp, _i, _i, _i, _i, _i, _vp, _vp]),
    "q8t_ternarize_workspace_size": (_sz, [_i64]),
    "q8t_ternarize": (_i, [_vp, _i64, _u64, _vp, _vp, _vp, _vp]),
    "q8t_binarize": (_i, [_vp, _i64, _vp, _vp]),
    "q8t_pack_bits": (_i, [_vp, _i, _i, _i, _vp, _vp]),
    "q8t_xnor_gemm": (_i, [_vp, _vp, _i, _i, _i, _vp, _vp]),
    "q8t_tern_wgrad_multi_workspace_size": (_sz, [_i, _i, _i]),
    "q8t_tern_wgrad_multi": (_i, [_vp, _vp, _i, _i, _i, _i, _u64, _vp, _vp, _vp, _vp]),
    "q8t_range_bn_scale": (C.c_double, [_i64]),
    "q8t_version": (C.c_char_p, []),
}
for _name, (_res, _args) in _SIGS.items():
    _fn = getattr(_lib, _name)  # AttributeError here = the library does not export the symbol
    _fn.restype = _res
    _fn.argtypes = _args

EXPORTED = tuple(sorted(_SIGS))


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)
_raw_device = getattr(torch._C, "_cuda_getDevice", None) or torch.cuda.current_device


def _stream():
    """torch's current stream on the current device as a raw handle.  torch.cuda.current_stream() costs
    ~0.2 ms of host time per call (it re-checks the environment), which starves the GPU when a step makes
    hundreds of library calls; the raw accessor is a plain C call."""
    if _raw_stream is not None:
        return C.c_void_p(_raw_stream(_raw_device()))
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc, where):
    if rc != 0:
        raise Q8TError(rc, where)


def _dev(t):
    if not t.is_cuda:
        raise ValueError("q8t works on device tensors only (got a CPU tensor)")
    if not t.is_contiguous():
        raise ValueError("q8t needs contiguous tensors")
    return t


_ws_cache = {}


def workspace(nbytes, device):
    """A reusable device scratch buffer of at least nbytes (grown on demand, one per device)."""
    key = (device.type, device.index)
    buf = _ws_cache.get(key)
    need = max(int(nbytes), 256)
    if buf is None or buf.numel() < need:
        buf = torch.empty(need, dtype=torch.uint8, device=device)
        _ws_cache[key] = buf
    return buf


def new_qparams(device):
    """Device-resident q8t_qparams (24 bytes) as an int32[6] tensor."""
    return torch.empty(6, dtype=torch.int32, device=device)


def qparams_to_host(qp):
    """(vmin, vmax, scale, inv_scale, zero_point, bits) read back from the device."""
    h = qp.cpu()
    f = h[:4].view(torch.float32)
    return (float(f[0]), float(f[1]), float(f[2]), float(f[3]), int(h[4]), int(h[5]))


def version():
    return _lib.q8t_version().decode()


def probe_stream(mode, src, dst, nbytes):
    """Plain streaming kernel of known traffic (0 copy, 1 read only, 2 fill); see q8t.h."""
    _check(_lib.q8t_probe_stream(int(mode), _ptr(src), _ptr(dst), int(nbytes), _stream()), "q8t_probe_stream")


def range_bn_scale(n):
    return float(_lib.q8t_range_bn_scale(int(n)))


# ------------------------------------------------------------------ quantization
def quantize(x, bits=8, stochastic=False, seed=0, q_out=None, qp_out=None, ws=None):
    _dev(x)
    n = x.numel()
    q = q_out if q_out is not None else torch.empty(x.shape, dtype=torch.int8 if bits <= 8 else torch.int16,
                                                     device=x.device)
    qp = qp_out if qp_out is not None else new_qparams(x.device)
    ws = ws if ws is not None else workspace(_lib.q8t_quantize_workspace_size(n), x.device)
    _check(_lib.q8t_quantize(_ptr(x), n, bits, int(bool(stochastic)), int(seed) & (2 ** 64 - 1), _ptr(q),
                             _ptr(qp), _ptr(ws), _stream()), "q8t_quantize")
    return q, qp


def quantize_multi(tensors, bits=8):
    """Nearest-rounding quantization of several tensors (each with its own range) in two launches.
    Returns [(codes, qparams), ...] in the order of `tensors`."""
    count = len(tensors)
    for t in tensors:
        _dev(t)
    dev = tensors[0].device
    qs = [torch.empty(t.shape, dtype=torch.int8, device=dev) for t in tensors]
    qps = torch.empty((count, 6), dtype=torch.int32, device=dev)     # one q8t_qparams (24 bytes) per row
    xs = (C.c_void_p * count)(*[t.data_ptr() for t in tensors])
    ns = (C.c_int64 * count)(*[t.numel() for t in tensors])
    qo = (C.c_void_p * count)(*[q.data_ptr() for q in qs])
    po = (C.c_void_p * count)(*[qps[i].data_ptr() for i in range(count)])
    ws = workspace(_lib.q8t_quantize_multi_workspace_size(count, ns), dev)
    _check(_lib.q8t_quantize_multi(count, xs, ns, bits, qo, po, _ptr(ws), _stream()), "q8t_quantize_multi")
    return [(qs[i], qps[i]) for i in range(count)]


def init():
    """Per-device set-up of the allocation-free entry point (the current device)."""
    _check(_lib.q8t_init(), "q8t_init")


def quantize_noalloc(x, q_out, qp_out, bits=8, stochastic=False, seed=0):
    """q8t_quantize without a workspace: the library's static scratch array holds the partial results.
    The caller supplies every buffer; nothing is allocated here either."""
    _dev(x)
    _check(_lib.q8t_quantize_noalloc(_ptr(x), x.numel(), bits, int(bool(stochastic)), int(seed) & (2 ** 64 - 1),
                                     _ptr(q_out), _ptr(qp_out), _stream()), "q8t_quantize_noalloc")
    return q_out, qp_out


def quantize_with_range(x, vmin_vmax, bits=8, stochastic=False, seed=0, q_out=None, qp_out=None):
    _dev(x)
    _dev(vmin_vmax)
    n = x.numel()
    q = q_out if q_out is not None else torch.empty(x.shape, dtype=torch.int8 if bits <= 8 else torch.int16,
                                                     device=x.device)
    qp = qp_out if qp_out is not None else new_qparams(x.device)
    _check(_lib.q8t_quantize_with_range(_ptr(x), n, bits, int(bool(stochastic)), int(seed) & (2 ** 64 - 1),
                                        _ptr(vmin_vmax), _ptr(q), _ptr(qp), _stream()),
           "q8t_quantize_with_range")
    return q, qp


def quantize_bifurcate(g, seed8=0, seed16=1, q8_out=None, qp8_out=None, q16_out=None, qp16_out=None, ws=None):
    _dev(g)
    n = g.numel()
    q8 = q8_out if q8_out is not None else torch.empty(g.shape, dtype=torch.int8, device=g.device)
    q16 = q16_out if q16_out is not None else torch.empty(g.shape, dtype=torch.int16, device=g.device)
    qp8 = qp8_out if qp8_out is not None else new_qparams(g.device)
    qp16 = qp16_out if qp16_out is not None else new_qparams(g.device)
    ws = ws if ws is not None else workspace(_lib.q8t_quantize_workspace_size(n), g.device)
    _check(_lib.q8t_quantize_bifurcate(_ptr(g), n, int(seed8) & (2 ** 64 - 1), int(seed16) & (2 ** 64 - 1),
                                       _ptr(q8), _ptr(qp8), _ptr(q16), _ptr(qp16), _ptr(ws), _stream()),
           "q8t_quantize_bifurcate")
    return q8, qp8, q16, qp16


def dequantize(q, qp, out=None):
    _dev(q)
    out = out if out is not None else torch.empty(q.shape, dtype=torch.float32, device=q.device)
    _check(_lib.q8t_dequantize(_ptr(q), _ptr(qp), q.numel(), _ptr(out), _stream()), "q8t_dequantize")
    return out


# ------------------------------------------------------------------ FC products
def _fc(fn, name, a, pa, b, pb, M, N, K, out_shape, which, acc_dtype, want_acc, out, ws):
    dev = a.device
    y = out if out is not None else torch.empty(out_shape, dtype=torch.float32, device=dev)
    acc = torch.empty(out_shape, dtype=acc_dtype, device=dev) if want_acc else None
    ws = ws if ws is not None else workspace(_lib.q8t_qgemm_workspace_size(M, N, K, which), dev)
    _check(fn(_ptr(a), _ptr(pa), _ptr(b), _ptr(pb), M, N, K, _ptr(y), _ptr(acc), _ptr(ws), _stream()), name)
    return y, acc


def qgemm_fwd(qx, px, qw, pw, want_acc=False, out=None, ws=None):
    """Y[M,N] = X[M,K] W[K,N]"""
    _dev(qx), _dev(qw)
    M, K = qx.shape
    K2, N = qw.shape
    assert K == K2
    return _fc(_lib.q8t_qgemm_fwd, "q8t_qgemm_fwd", qx, px, qw, pw, M, N, K, (M, N), 0, torch.int32, want_acc,
               out, ws)


def qgemm_dgrad(qdy, pg, qw, pw, want_acc=False, out=None, ws=None):
    """dX[M,K] = dY[M,N] W[K,N]^T"""
    _dev(qdy), _dev(qw)
    M, N = qdy.shape
    K, N2 = qw.shape
    assert N == N2
    return _fc(_lib.q8t_qgemm_dgrad, "q8t_qgemm_dgrad", qdy, pg, qw, pw, M, N, K, (M, K), 1, torch.int32,
               want_acc, out, ws)


def qgemm_wgrad(qx, px, qdy16, pg16, want_acc=False, out=None, ws=None):
    """dW[K,N] = X[M,K]^T dY16[M,N]"""
    _dev(qx), _dev(qdy16)
    M, K = qx.shape
    M2, N = qdy16.shape
    assert M == M2 and qdy16.dtype == torch.int16
    return _fc(_lib.q8t_qgemm_wgrad, "q8t_qgemm_wgrad", qx, px, qdy16, pg16, M, N, K, (K, N), 2, torch.int64,
               want_acc, out, ws)


def chunk_range(x, K, ws=None):
    """Clamping range averaged over K contiguous chunks (App. B).  Returns a device tensor {vmin, vmax}."""
    _dev(x)
    n = x.numel()
    out = torch.empty(2, dtype=torch.float32, device=x.device)
    ws = ws if ws is not None else workspace(_lib.q8t_chunk_range_workspace_size(n, int(K)), x.device)
    _check(_lib.q8t_chunk_range(_ptr(x), n, int(K), _ptr(out), _ptr(ws), _stream()), "q8t_chunk_range")
    return out


def quant_angle(x, q, qp, ws=None):
    """Sec. 5.1 (Problem Statement), eq. (1).  Returns a device tensor of 4 doubles {x.Q(x), |x|^2, |Q(x)|^2, cos(theta)}."""
    _dev(x), _dev(q)
    n = x.numel()
    assert q.numel() == n
    out = torch.empty(4, dtype=torch.float64, device=x.device)
    ws = ws if ws is not None else workspace(_lib.q8t_quant_angle_workspace_size(n), x.device)
    _check(_lib.q8t_quant_angle(_ptr(x), _ptr(q), _ptr(qp), n, _ptr(out), _ptr(ws), _stream()), "q8t_quant_angle")
    return out


# ------------------------------------------------------------------ convolution products
def conv_desc(N, Cin, H, W, K, R, S, stride, pad):
    return ConvDesc(N, Cin, H, W, K, R, S, stride, pad)


def _conv(fn, name, d, a, pa, b, pb, out_shape, which, acc_dtype, want_acc, out, ws):
    dev = a.device
    y = out if out is not None else torch.empty(out_shape, dtype=torch.float32, device=dev)
    acc = torch.empty(out_shape, dtype=acc_dtype, device=dev) if want_acc else None
    ws = ws if ws is not None else workspace(_lib.q8t_qconv_workspace_size(C.byref(d), which), dev)
    _check(fn(C.byref(d), _ptr(a), _ptr(pa), _ptr(b), _ptr(pb), _ptr(y), _ptr(acc), _ptr(ws), _stream()), name)
    return y, acc


def qconv_workspace_size(d, which):
    """Bytes of workspace q8t_qconv_fwd (0) / dgrad (1) / wgrad (2) need for this layer."""
    return int(_lib.q8t_qconv_workspace_size(C.byref(d), int(which)))


def qconv_fwd(d, qx, px, qw, pw, want_acc=False, out=None, ws=None):
    _dev(qx), _dev(qw)
    assert tuple(qx.shape) == (d.N, d.C, d.H, d.W) and tuple(qw.shape) == (d.K, d.C, d.R, d.S)
    return _conv(_lib.q8t_qconv_fwd, "q8t_qconv_fwd", d, qx, px, qw, pw, (d.N, d.K, d.P, d.Q), 0, torch.int32,
                 want_acc, out, ws)


def qconv_pack_size(d, which):
    """Bytes of the packed filter for the forward (0) / layer-gradient (1) product of this shape; 0: nothing to pack."""
    return int(_lib.q8t_qconv_pack_size(C.byref(d), int(which)))


def qconv_pack_multi(jobs, out=None):
    """jobs: list of (desc, which, qw).  Packs the filters of all of them in one launch and returns one buffer per job
    (None where the shape packs nothing ahead) for the packed= argument of the products.  out: buffers to reuse."""
    n = len(jobs)
    if n == 0:
        return []
    descs = (ConvDesc * n)(*[j[0] for j in jobs])
    which = (C.c_int * n)(*[int(j[1]) for j in jobs])
    bufs = []
    for i, (d, w, qw) in enumerate(jobs):
        _dev(qw)
        assert tuple(qw.shape) == (d.K, d.C, d.R, d.S) and qw.dtype == torch.int8
        size = qconv_pack_size(d, w)
        if size == 0:
            bufs.append(None)
        elif out is not None and out[i] is not None:
            assert out[i].numel() >= size and out[i].dtype == torch.uint8
            bufs.append(out[i])
        else:
            bufs.append(torch.empty(size, dtype=torch.uint8, device=qw.device))
    qws = (C.c_void_p * n)(*[_ptr(j[2]) for j in jobs])
    pks = (C.c_void_p * n)(*[_ptr(b) for b in bufs])
    _check(_lib.q8t_qconv_pack_multi(n, descs, which, qws, pks, _stream()), "q8t_qconv_pack_multi")
    return bufs


def qconv_fwd_bn_stats(d, qx, px, qw, pw, want_acc=False, out=None, stats_out=None, ws=None, packed=None):
    """Forward convolution + Range BN statistics of its result.  Returns (y, acc or None, stats[3,K]).
    packed: the layer's filter from qconv_pack_multi (same desc, which = 0, same codes)."""
    _dev(qx), _dev(qw)
    assert tuple(qx.shape) == (d.N, d.C, d.H, d.W) and tuple(qw.shape) == (d.K, d.C, d.R, d.S)
    dev = qx.device
    shape = (d.N, d.K, d.P, d.Q)
    y = out if out is not None else torch.empty(shape, dtype=torch.float32, device=dev)
    acc = torch.empty(shape, dtype=torch.int32, device=dev) if want_acc else None
    stats = stats_out if stats_out is not None else torch.empty((3, d.K), dtype=torch.float32, device=dev)
    ws = ws if ws is not None else workspace(_lib.q8t_qconv_fwd_bn_stats_workspace_size(C.byref(d)), dev)
    if packed is not None:
        _check(_lib.q8t_qconv_fwd_bn_stats_packed(C.byref(d), _ptr(qx), _ptr(px), _ptr(qw), _ptr(pw), _ptr(packed), _ptr(y),
                                                  _ptr(acc), _ptr(stats), _ptr(ws), _stream()), "q8t_qconv_fwd_bn_stats_packed")
    else:
        _check(_lib.q8t_qconv_fwd_bn_stats(C.byref(d), _ptr(qx), _ptr(px), _ptr(qw), _ptr(pw), _ptr(y), _ptr(acc),
                                           _ptr(stats), _ptr(ws), _stream()), "q8t_qconv_fwd_bn_stats")
    return y, acc, stats


def qconv_dgrad(d, qdy, pg, qw, pw, want_acc=False, out=None, ws=None, packed=None):
    """packed: the layer's filter from qconv_pack_multi (same desc, which = 1, same codes)."""
    _dev(qdy), _dev(qw)
    assert tuple(qdy.shape) == (d.N, d.K, d.P, d.Q) and tuple(qw.shape) == (d.K, d.C, d.R, d.S)
    if packed is not None:
        dev = qdy.device
        shape = (d.N, d.C, d.H, d.W)
        dx = out if out is not None else torch.empty(shape, dtype=torch.float32, device=dev)
        acc = torch.empty(shape, dtype=torch.int32, device=dev) if want_acc else None
        ws = ws if ws is not None else workspace(_lib.q8t_qconv_workspace_size(C.byref(d), 1), dev)
        _check(_lib.q8t_qconv_dgrad_packed(C.byref(d), _ptr(qdy), _ptr(pg), _ptr(qw), _ptr(pw), _ptr(packed), _ptr(dx), _ptr(acc),
                                           _ptr(ws), _stream()), "q8t_qconv_dgrad_packed")
        return dx, acc
    return _conv(_lib.q8t_qconv_dgrad, "q8t_qconv_dgrad", d, qdy, pg, qw, pw, (d.N, d.C, d.H, d.W), 1,
                 torch.int32, want_acc, out, ws)


def qconv_dgrad_relu_sum(d, qdy, pg, qw, pw, other, act, out=None, ws=None, packed=None):
    """act > 0 ? dgrad + other : 0 (other may be None): the layer gradient of a residual block's first convolution
    with the end of the block's backward pass in its epilogue.  Returns dx."""
    _dev(qdy), _dev(qw), _dev(act)
    shape = (d.N, d.C, d.H, d.W)
    assert tuple(qdy.shape) == (d.N, d.K, d.P, d.Q) and tuple(qw.shape) == (d.K, d.C, d.R, d.S)
    assert tuple(act.shape) == shape and act.dtype == torch.float32 and act.is_contiguous()
    if other is not None:
        _dev(other)
        assert tuple(other.shape) == shape and other.dtype == torch.float32 and other.is_contiguous()
    dx = out if out is not None else torch.empty(shape, dtype=torch.float32, device=qdy.device)
    ws = ws if ws is not None else workspace(_lib.q8t_qconv_workspace_size(C.byref(d), 1), qdy.device)
    if packed is not None:
        _check(_lib.q8t_qconv_dgrad_relu_sum_packed(C.byref(d), _ptr(qdy), _ptr(pg), _ptr(qw), _ptr(pw), _ptr(packed), _ptr(other),
                                                    _ptr(act), _ptr(dx), _ptr(ws), _stream()), "q8t_qconv_dgrad_relu_sum_packed")
    else:
        _check(_lib.q8t_qconv_dgrad_relu_sum(C.byref(d), _ptr(qdy), _ptr(pg), _ptr(qw), _ptr(pw), _ptr(other), _ptr(act), _ptr(dx),
                                             _ptr(ws), _stream()), "q8t_qconv_dgrad_relu_sum")
    return dx


def qconv_wgrad(d, qx, px, qdy16, pg16, want_acc=False, out=None, ws=None):
    _dev(qx), _dev(qdy16)
    assert tuple(qx.shape) == (d.N, d.C, d.H, d.W) and tuple(qdy16.shape) == (d.N, d.K, d.P, d.Q)
    assert qdy16.dtype == torch.int16
    return _conv(_lib.q8t_qconv_wgrad, "q8t_qconv_wgrad", d, qx, px, qdy16, pg16, (d.K, d.C, d.R, d.S), 2,
                 torch.int64, want_acc, out, ws)


# ------------------------------------------------------------------ Range BN
def range_bn_fwd(x, gamma=None, beta=None, eps=0.0, quantized=False, want_y=True, y_out=None, stats_out=None,
                 q_out=None, qp_out=None, ws=None):
    """Returns (y or None, stats[3,C], q or None, qp or None)."""
    _dev(x)
    N, Cc, H, W = x.shape
    dev = x.device
    y = y_out if y_out is not None else (torch.empty_like(x) if want_y else None)
    stats = stats_out if stats_out is not None else torch.empty((3, Cc), dtype=torch.float32, device=dev)
    q = qp = None
    if quantized:
        q = q_out if q_out is not None else torch.empty(x.shape, dtype=torch.int8, device=dev)
        qp = qp_out if qp_out is not None else new_qparams(dev)
    ws = ws if ws is not None else workspace(_lib.q8t_range_bn_workspace_size(N, Cc, H, W), dev)
    _check(_lib.q8t_range_bn_fwd(_ptr(x), N, Cc, H, W, _ptr(gamma), _ptr(beta), float(eps), _ptr(y), _ptr(stats),
                                 _ptr(q), _ptr(qp), _ptr(ws), _stream()), "q8t_range_bn_fwd")
    return y, stats, q, qp


def range_bn_fwd_apply(x, stats, gamma=None, beta=None, eps=0.0, quantized=False, want_y=True, y_out=None, q_out=None,
                       qp_out=None):
    """Range BN forward from given statistics.  Returns (y or None, q or None, qp or None)."""
    _dev(x), _dev(stats)
    N, Cc, H, W = x.shape
    dev = x.device
    y = y_out if y_out is not None else (torch.empty_like(x) if want_y else None)
    q = qp = None
    if quantized:
        q = q_out if q_out is not None else torch.empty(x.shape, dtype=torch.int8, device=dev)
        qp = qp_out if qp_out is not None else new_qparams(dev)
    _check(_lib.q8t_range_bn_fwd_apply(_ptr(x), N, Cc, H, W, _ptr(gamma), _ptr(beta), float(eps), _ptr(stats), _ptr(y),
                                       _ptr(q), _ptr(qp), _stream()), "q8t_range_bn_fwd_apply")
    return y, q, qp


def range_bn_relu_fwd_apply(x, stats, gamma=None, beta=None, eps=0.0, quantized=False, want_y=True, y_out=None,
                            q_out=None, qp_out=None):
    """Range BN + ReLU forward from given statistics.  Returns (y or None, q or None, qp or None)."""
    _dev(x), _dev(stats)
    N, Cc, H, W = x.shape
    dev = x.device
    y = y_out if y_out is not None else (torch.empty_like(x) if want_y else None)
    q = qp = None
    if quantized:
        q = q_out if q_out is not None else torch.empty(x.shape, dtype=torch.int8, device=dev)
        qp = qp_out if qp_out is not None else new_qparams(dev)
    _check(_lib.q8t_range_bn_relu_fwd_apply(_ptr(x), N, Cc, H, W, _ptr(gamma), _ptr(beta), float(eps), _ptr(stats),
                                            _ptr(y), _ptr(q), _ptr(qp), _stream()), "q8t_range_bn_relu_fwd_apply")
    return y, q, qp


def range_bn_bwd(x, dy, stats, gamma=None, eps=0.0, dx_out=None, ws=None):
    """Returns (dx, dgamma, dbeta)."""
    _dev(x), _dev(dy), _dev(stats)
    N, Cc, H, W = x.shape
    dev = x.device
    dx = dx_out if dx_out is not None else torch.empty_like(x)
    dgamma = torch.empty(Cc, dtype=torch.float32, device=dev)
    dbeta = torch.empty(Cc, dtype=torch.float32, device=dev)
    ws = ws if ws is not None else workspace(_lib.q8t_range_bn_workspace_size(N, Cc, H, W), dev)
    _check(_lib.q8t_range_bn_bwd(_ptr(x), _ptr(dy), _ptr(stats), N, Cc, H, W, _ptr(gamma), float(eps), _ptr(dx),
                                 _ptr(dgamma), _ptr(dbeta), _ptr(ws), _stream()), "q8t_range_bn_bwd")
    return dx, dgamma, dbeta


def _bn_bwd_bifurcate_buffers(x, dx_out, q8_out, qp8_out, q16_out, qp16_out, ws, want_dx, want_q8=True, ws_size=None):
    """output buffers and workspace shared by the fused backward calls (want_q8=False: no 8-bit copy, q8 = qp8 = None)"""
    N, Cc, H, W = x.shape
    dev = x.device
    dx = dx_out if dx_out is not None else (torch.empty_like(x) if want_dx else None)
    dgamma = torch.empty(Cc, dtype=torch.float32, device=dev)
    dbeta = torch.empty(Cc, dtype=torch.float32, device=dev)
    q8 = qp8 = None
    if want_q8:
        q8 = q8_out if q8_out is not None else torch.empty(x.shape, dtype=torch.int8, device=dev)
        qp8 = qp8_out if qp8_out is not None else new_qparams(dev)
    q16 = q16_out if q16_out is not None else torch.empty(x.shape, dtype=torch.int16, device=dev)
    qp16 = qp16_out if qp16_out is not None else new_qparams(dev)
    size = (ws_size or _lib.q8t_range_bn_bwd_bifurcate_workspace_size)(N, Cc, H, W)
    ws = ws if ws is not None else workspace(size, dev)
    return dx, dgamma, dbeta, q8, qp8, q16, qp16, ws


def range_bn_relu_bwd_bifurcate(x, dy, stats, gamma=None, beta=None, eps=0.0, seed8=0, seed16=1, dx_out=None,
                                q8_out=None, qp8_out=None, q16_out=None, qp16_out=None, ws=None, want_dx=True):
    """Backward of Range BN + ReLU + bifurcated quantization of dx in one call.
    Returns (dx or None, dgamma, dbeta, q8, qp8, q16, qp16)."""
    _dev(x), _dev(dy), _dev(stats)
    N, Cc, H, W = x.shape
    dx, dgamma, dbeta, q8, qp8, q16, qp16, ws = _bn_bwd_bifurcate_buffers(x, dx_out, q8_out, qp8_out, q16_out, qp16_out,
                                                                          ws, want_dx)
    _check(_lib.q8t_range_bn_relu_bwd_bifurcate(_ptr(x), _ptr(dy), _ptr(stats), N, Cc, H, W, _ptr(gamma), _ptr(beta),
                                                float(eps), _ptr(dx), _ptr(dgamma), _ptr(dbeta),
                                                int(seed8) & (2 ** 64 - 1), int(seed16) & (2 ** 64 - 1), _ptr(q8),
                                                _ptr(qp8), _ptr(q16), _ptr(qp16), _ptr(ws), _stream()),
           "q8t_range_bn_relu_bwd_bifurcate")
    return dx, dgamma, dbeta, q8, qp8, q16, qp16


def range_bn_bwd_bifurcate(x, dy, stats, gamma=None, eps=0.0, seed8=0, seed16=1, dx_out=None, q8_out=None,
                           qp8_out=None, q16_out=None, qp16_out=None, ws=None, want_dx=True, want_q8=True):
    """Range BN backward + bifurcated quantization of dx in one call.
    Returns (dx or None, dgamma, dbeta, q8, qp8, q16, qp16); want_q8=False leaves q8 = qp8 = None."""
    _dev(x), _dev(dy), _dev(stats)
    N, Cc, H, W = x.shape
    dx, dgamma, dbeta, q8, qp8, q16, qp16, ws = _bn_bwd_bifurcate_buffers(x, dx_out, q8_out, qp8_out, q16_out, qp16_out,
                                                                          ws, want_dx, want_q8)
    _check(_lib.q8t_range_bn_bwd_bifurcate(_ptr(x), _ptr(dy), _ptr(stats), N, Cc, H, W, _ptr(gamma), float(eps),
                                           _ptr(dx), _ptr(dgamma), _ptr(dbeta), int(seed8) & (2 ** 64 - 1),
                                           int(seed16) & (2 ** 64 - 1), _ptr(q8), _ptr(qp8), _ptr(q16), _ptr(qp16),
                                           _ptr(ws), _stream()), "q8t_range_bn_bwd_bifurcate")
    return dx, dgamma, dbeta, q8, qp8, q16, qp16


# ------------------------------------------------------------------ ternarized back-propagation
def ternarize(g, seed=0, ws=None):
    """Stochastic ternarization.  Returns (codes int8 in {-1,0,1}, scale: device tensor of 1 float = max|g|)."""
    _dev(g)
    n = g.numel()
    t = torch.empty(g.shape, dtype=torch.int8, device=g.device)
    scale = torch.empty(1, dtype=torch.float32, device=g.device)
    ws = ws if ws is not None else workspace(_lib.q8t_ternarize_workspace_size(n), g.device)
    _check(_lib.q8t_ternarize(_ptr(g), n, int(seed) & (2 ** 64 - 1), _ptr(t), _ptr(scale), _ptr(ws), _stream()),
           "q8t_ternarize")
    return t, scale


def binarize(x):
    """+1 for x >= 0, -1 otherwise (int8)."""
    _dev(x)
    codes = torch.empty(x.shape, dtype=torch.int8, device=x.device)
    _check(_lib.q8t_binarize(_ptr(x), x.numel(), _ptr(codes), _stream()), "q8t_binarize")
    return codes


def pack_bits(codes, transpose=False):
    """Bit rows (int32 tensor holding the uint32 words) of a 2-D matrix of +-1 codes."""
    _dev(codes)
    rows, cols = codes.shape
    nr, nc = (cols, rows) if transpose else (rows, cols)
    out = torch.empty((nr, (nc + 31) // 32), dtype=torch.int32, device=codes.device)
    _check(_lib.q8t_pack_bits(_ptr(codes), rows, cols, int(bool(transpose)), _ptr(out), _stream()), "q8t_pack_bits")
    return out


def xnor_gemm(a_bits, w_bits, K):
    """y[m,n] = sum_k a[m,k] w[n,k] over +-1 values given as bit rows of K bits (int32)."""
    _dev(a_bits), _dev(w_bits)
    M, N = a_bits.shape[0], w_bits.shape[0]
    assert a_bits.shape[1] == w_bits.shape[1] == (K + 31) // 32
    y = torch.empty((M, N), dtype=torch.int32, device=a_bits.device)
    _check(_lib.q8t_xnor_gemm(_ptr(a_bits), _ptr(w_bits), M, N, int(K), _ptr(y), _stream()), "q8t_xnor_gemm")
    return y


def tern_wgrad_multi(g, a_codes, S, seed=0, want_acc=False, ws=None):
    """Algorithm 1 (multiple stochastic ternarization sampling) for an FC layer.  Returns (dW [K,N], acc or None)."""
    _dev(g), _dev(a_codes)
    M, N = g.shape
    M2, K = a_codes.shape
    assert M == M2 and a_codes.dtype == torch.int8
    dw = torch.empty((K, N), dtype=torch.float32, device=g.device)
    acc = torch.empty((K, N), dtype=torch.int64, device=g.device) if want_acc else None
    ws = ws if ws is not None else workspace(_lib.q8t_tern_wgrad_multi_workspace_size(M, N, K), g.device)
    _check(_lib.q8t_tern_wgrad_multi(_ptr(g), _ptr(a_codes), M, N, K, int(S), int(seed) & (2 ** 64 - 1), _ptr(dw),
                                     _ptr(acc), _ptr(ws), _stream()), "q8t_tern_wgrad_multi")
    return dw, acc


# ------------------------------------------------------------------ network plumbing (not from the paper)
def range_bn_relu_maxpool_fwd(x, stats, gamma=None, beta=None, eps=0.0):
    """relu(Range BN(x)) + 3x3 / stride 2 / pad 1 max pooling in one pass.  Returns (pooled fp32, idx uint8)."""
    _dev(x), _dev(stats)
    N, Cc, H, W = x.shape
    P, Q = (H - 1) // 2 + 1, (W - 1) // 2 + 1
    out = torch.empty((N, Cc, P, Q), dtype=torch.float32, device=x.device)
    idx = torch.empty((N, Cc, P, Q), dtype=torch.uint8, device=x.device)
    _check(_lib.q8t_range_bn_relu_maxpool_fwd(_ptr(x), N, Cc, H, W, _ptr(gamma), _ptr(beta), float(eps), _ptr(stats), _ptr(out),
                                              _ptr(idx), _stream()), "q8t_range_bn_relu_maxpool_fwd")
    return out, idx


def maxpool_relu_bwd(gpool, idx, H, W):
    """Upstream gradient of the Range BN in front of ReLU + max pooling, from the pooled gradient and idx."""
    _dev(gpool), _dev(idx)
    N, Cc = gpool.shape[:2]
    dy = torch.empty((N, Cc, H, W), dtype=torch.float32, device=gpool.device)
    _check(_lib.q8t_maxpool_relu_bwd(_ptr(gpool), _ptr(idx), N, Cc, H, W, _ptr(dy), _stream()), "q8t_maxpool_relu_bwd")
    return dy


def maxpool_range_bn_bwd_bifurcate(x, gpool, idx, stats, gamma=None, eps=0.0, seed8=0, seed16=1, want_q8=True, ws=None):
    """maxpool_relu_bwd followed by range_bn_bwd_bifurcate without the unpooled gradient in memory.
    Returns (dgamma, dbeta, q8, qp8, q16, qp16); want_q8=False leaves q8 = qp8 = None."""
    _dev(x), _dev(gpool), _dev(idx), _dev(stats)
    N, Cc, H, W = x.shape
    assert tuple(gpool.shape) == (N, Cc, (H - 1) // 2 + 1, (W - 1) // 2 + 1) and gpool.shape == idx.shape
    _, dgamma, dbeta, q8, qp8, q16, qp16, ws = _bn_bwd_bifurcate_buffers(
        x, None, None, None, None, None, ws, False, want_q8, _lib.q8t_maxpool_range_bn_bwd_bifurcate_workspace_size)
    _check(_lib.q8t_maxpool_range_bn_bwd_bifurcate(_ptr(x), _ptr(gpool), _ptr(idx), _ptr(stats), N, Cc, H, W, _ptr(gamma),
                                                   float(eps), _ptr(dgamma), _ptr(dbeta), int(seed8) & (2 ** 64 - 1),
                                                   int(seed16) & (2 ** 64 - 1), _ptr(q8), _ptr(qp8), _ptr(q16), _ptr(qp16),
                                                   _ptr(ws), _stream()), "q8t_maxpool_range_bn_bwd_bifurcate")
    return dgamma, dbeta, q8, qp8, q16, qp16


def add_relu_quantize(a, b, quantized=True, ws=None):
    """relu(a + b) and (optionally) its 8-bit codes + parameters.  Returns (out, q or None, qp or None)."""
    _dev(a), _dev(b)
    assert a.shape == b.shape
    n = a.numel()
    out = torch.empty_like(a)
    q = torch.empty(a.shape, dtype=torch.int8, device=a.device) if quantized else None
    qp = new_qparams(a.device) if quantized else None
    ws = ws if ws is not None else workspace(_lib.q8t_add_relu_quantize_workspace_size(n), a.device)
    _check(_lib.q8t_add_relu_quantize(_ptr(a), _ptr(b), n, _ptr(out), _ptr(q), _ptr(qp), _ptr(ws), _stream()),
           "q8t_add_relu_quantize")
    return out, q, qp


def range_bn_add_relu_quantize(x, stats, other, gamma=None, beta=None, other_stats=None, other_gamma=None,
                               other_beta=None, eps=0.0, quantized=True):
    """relu(bn(x; stats) + o), o = other or bn(other; other_stats), and the 8-bit codes of the result.
    Returns (out, codes or None, qparams or None)."""
    _dev(x), _dev(other), _dev(stats)
    N, Cc, H, W = x.shape
    out = torch.empty_like(x)
    q = torch.empty(x.shape, dtype=torch.int8, device=x.device) if quantized else None
    qp = new_qparams(x.device) if quantized else None
    ws = workspace(_lib.q8t_add_relu_quantize_workspace_size(x.numel()), x.device)
    _check(_lib.q8t_range_bn_add_relu_quantize(_ptr(x), _ptr(stats), _ptr(gamma), _ptr(beta), _ptr(other), _ptr(other_stats),
                                               _ptr(other_gamma), _ptr(other_beta), N, Cc, H, W, float(eps), _ptr(out),
                                               _ptr(q), _ptr(qp), _ptr(ws), _stream()), "q8t_range_bn_add_relu_quantize")
    return out, q, qp


def relu_bwd_sum(g1, g2=None, out=None):
    """out > 0 ? g1 + g2 : 0 (out None: no mask; g2 None: nothing added)."""
    _dev(g1)
    res = torch.empty_like(g1)
    _check(_lib.q8t_relu_bwd_sum(_ptr(g1), _ptr(g2), _ptr(out), g1.numel(), _ptr(res), _stream()), "q8t_relu_bwd_sum")
    return res


def relu_bwd_sum_lattice(g1, g2s, out, stride):
    """out > 0 ? g1 + t : 0, t = g2s on the lattice of rows / columns that are multiples of stride, 0 elsewhere."""
    _dev(g1), _dev(g2s)
    N, Cc, H, W = g1.shape
    assert tuple(g2s.shape) == (N, Cc, (H + stride - 1) // stride, (W + stride - 1) // stride)
    res = torch.empty_like(g1)
    _check(_lib.q8t_relu_bwd_sum_lattice(_ptr(g1), _ptr(g2s), _ptr(out), N, Cc, H, W, int(stride), _ptr(res), _stream()),
           "q8t_relu_bwd_sum_lattice")
    return res


def relu_bwd_add(g, out, other=None):
    """(out > 0 ? g : 0) + other."""
    _dev(g), _dev(out)
    res = torch.empty_like(g)
    _check(_lib.q8t_relu_bwd_add(_ptr(g), _ptr(out), _ptr(other), g.numel(), _ptr(res), _stream()), "q8t_relu_bwd_add")
    return res
