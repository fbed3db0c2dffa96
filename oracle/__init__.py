"""ctypes/numpy access to the CPU oracle (oracle/q8t_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's
cpu-baseline leg.  The product package never imports this module and this module
never imports the product package.  It holds argument marshalling only; every
piece of arithmetic lives in the C file.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "q8t_oracle.c")
_LIB = os.path.join(_HERE, "libq8t_oracle.so")


class QParams(C.Structure):
    _fields_ = [("vmin", C.c_float), ("vmax", C.c_float), ("scale", C.c_float),
                ("inv_scale", C.c_float), ("zero_point", C.c_int32), ("bits", C.c_int32)]

    def as_tuple(self):
        return (self.vmin, self.vmax, self.scale, self.inv_scale, self.zero_point, self.bits)

    def __repr__(self):
        return "QParams(vmin=%r, vmax=%r, scale=%r, inv_scale=%r, zp=%d, bits=%d)" % self.as_tuple()


class ConvDesc(C.Structure):
    _fields_ = [(k, C.c_int) for k in ("N", "C", "H", "W", "K", "R", "S", "stride", "pad")]

    @property
    def P(self):
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self):
        return (self.W + 2 * self.pad - self.S) // self.stride + 1


def build(force=False):
    """Compile the oracle with gcc (plain C, OpenMP on outer loops, no FMA contraction)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC",
           "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.orc_range_bn_scale.restype = C.c_double
        _lib.orc_range_bn_scale.argtypes = [C.c_int64]
        _lib.orc_r16.restype = C.c_uint32
        _lib.orc_r16.argtypes = [C.c_uint64, C.c_uint64]
        _lib.orc_rng_words.argtypes = [C.c_uint64, C.c_uint64, C.POINTER(C.c_uint32),
                                       C.POINTER(C.c_uint32)]
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def num_threads():
    return int(lib().orc_num_threads())


def range_bn_scale(n):
    return float(lib().orc_range_bn_scale(int(n)))


def r16(i, seed):
    return int(lib().orc_r16(C.c_uint64(int(i)), C.c_uint64(int(seed))))


def rng_words(g, seed):
    w0, w1 = C.c_uint32(), C.c_uint32()
    lib().orc_rng_words(C.c_uint64(int(g)), C.c_uint64(int(seed)), C.byref(w0), C.byref(w1))
    return w0.value, w1.value


def minmax(x):
    x = _f32(x).ravel()
    mn, mx = C.c_float(), C.c_float()
    lib().orc_minmax(_p(x), C.c_int64(x.size), C.byref(mn), C.byref(mx))
    return np.float32(mn.value), np.float32(mx.value)


def qparams_from_range(vmin, vmax, bits):
    qp = QParams()
    lib().orc_qparams_from_range(C.c_float(vmin), C.c_float(vmax), C.c_int(bits), C.byref(qp))
    return qp


def _stored_dtype(bits):
    return np.int8 if bits <= 8 else np.int16


def quantize(x, bits=8, stochastic=False, seed=0, vrange=None):
    """Returns (stored codes, levels int32, QParams), shaped like x."""
    x = _f32(x)
    n = x.size
    levels = np.empty(x.shape, dtype=np.int32)
    stored = np.empty(x.shape, dtype=_stored_dtype(bits))
    qp = QParams()
    if vrange is None:
        lib().orc_quantize(_p(x), C.c_int64(n), C.c_int(bits), C.c_int(int(stochastic)),
                           C.c_uint64(int(seed)), _p(levels), _p(stored), C.byref(qp))
    else:
        lib().orc_quantize_with_range(_p(x), C.c_int64(n), C.c_int(bits), C.c_int(int(stochastic)),
                                      C.c_uint64(int(seed)), C.c_float(vrange[0]),
                                      C.c_float(vrange[1]), _p(levels), _p(stored), C.byref(qp))
    return stored, levels, qp


def dequantize(stored, qp):
    stored = np.ascontiguousarray(stored, dtype=_stored_dtype(qp.bits))
    out = np.empty(stored.shape, dtype=np.float32)
    lib().orc_dequantize(_p(stored), C.byref(qp), C.c_int64(stored.size), _p(out))
    return out


def quant_angle(x, stored, qp):
    """Sec. 5.1 (Problem Statement), eq. (1).  Returns (x.Q(x), |x|^2, |Q(x)|^2, cos(theta)) as fp64."""
    x = _f32(x)
    stored = np.ascontiguousarray(stored, dtype=_stored_dtype(qp.bits))
    assert x.size == stored.size
    out = np.empty(4, np.float64)
    lib().orc_quant_angle(_p(x), _p(stored), C.byref(qp), C.c_int64(x.size), _p(out))
    return tuple(float(v) for v in out)


def chunk_range(x, K):
    """App. B: clamping range averaged over K contiguous chunks.  Returns (vmin, vmax) as fp32."""
    x = _f32(x)
    out = np.empty(2, np.float32)
    lib().orc_chunk_range(_p(x), C.c_int64(x.size), C.c_int(int(K)), _p(out))
    return np.float32(out[0]), np.float32(out[1])


def _i8(a):
    return np.ascontiguousarray(a, dtype=np.int8)


def _i16(a):
    return np.ascontiguousarray(a, dtype=np.int16)


def qgemm_fwd(qx, px, qw, pw):
    qx, qw = _i8(qx), _i8(qw)
    M, K = qx.shape
    K2, N = qw.shape
    assert K == K2
    y = np.empty((M, N), np.float32)
    acc = np.empty((M, N), np.int64)
    lib().orc_qgemm_fwd(_p(qx), C.byref(px), _p(qw), C.byref(pw), M, N, K, _p(y), _p(acc))
    return y, acc


def qgemm_dgrad(qdy, pg, qw, pw):
    qdy, qw = _i8(qdy), _i8(qw)
    M, N = qdy.shape
    K, N2 = qw.shape
    assert N == N2
    dx = np.empty((M, K), np.float32)
    acc = np.empty((M, K), np.int64)
    lib().orc_qgemm_dgrad(_p(qdy), C.byref(pg), _p(qw), C.byref(pw), M, N, K, _p(dx), _p(acc))
    return dx, acc


def qgemm_wgrad(qx, px, qdy16, pg):
    qx, qdy16 = _i8(qx), _i16(qdy16)
    M, K = qx.shape
    M2, N = qdy16.shape
    assert M == M2
    dw = np.empty((K, N), np.float32)
    acc = np.empty((K, N), np.int64)
    lib().orc_qgemm_wgrad(_p(qx), C.byref(px), _p(qdy16), C.byref(pg), M, N, K, _p(dw), _p(acc))
    return dw, acc


def conv_desc(N, Cin, H, W, K, R, S, stride, pad):
    return ConvDesc(N, Cin, H, W, K, R, S, stride, pad)


def qconv_fwd(d, qx, px, qw, pw):
    qx, qw = _i8(qx), _i8(qw)
    assert qx.shape == (d.N, d.C, d.H, d.W) and qw.shape == (d.K, d.C, d.R, d.S)
    shape = (d.N, d.K, d.P, d.Q)
    y = np.empty(shape, np.float32)
    acc = np.empty(shape, np.int64)
    lib().orc_qconv_fwd(C.byref(d), _p(qx), C.byref(px), _p(qw), C.byref(pw), _p(y), _p(acc))
    return y, acc


def qconv_dgrad(d, qdy, pg, qw, pw):
    qdy, qw = _i8(qdy), _i8(qw)
    assert qdy.shape == (d.N, d.K, d.P, d.Q) and qw.shape == (d.K, d.C, d.R, d.S)
    shape = (d.N, d.C, d.H, d.W)
    dx = np.empty(shape, np.float32)
    acc = np.empty(shape, np.int64)
    lib().orc_qconv_dgrad(C.byref(d), _p(qdy), C.byref(pg), _p(qw), C.byref(pw), _p(dx), _p(acc))
    return dx, acc


def qconv_wgrad(d, qx, px, qdy16, pg):
    qx, qdy16 = _i8(qx), _i16(qdy16)
    assert qx.shape == (d.N, d.C, d.H, d.W) and qdy16.shape == (d.N, d.K, d.P, d.Q)
    shape = (d.K, d.C, d.R, d.S)
    dw = np.empty(shape, np.float32)
    acc = np.empty(shape, np.int64)
    lib().orc_qconv_wgrad(C.byref(d), _p(qx), C.byref(px), _p(qdy16), C.byref(pg), _p(dw), _p(acc))
    return dw, acc


def _opt_f32(a):
    return None if a is None else _f32(a)


def range_bn_stats(x):
    x = _f32(x)
    N, Cc, H, W = x.shape
    stats = np.empty((3, Cc), np.float32)
    lib().orc_range_bn_stats(_p(x), N, Cc, H, W, _p(stats))
    return stats


def range_bn_fwd(x, gamma=None, beta=None, eps=0.0, stats=None, quantized=False):
    """Returns (y, stats[3,C], q_stored or None, QParams or None).
    With `stats` given, only the elementwise stage runs (on those statistics)."""
    x = _f32(x)
    N, Cc, H, W = x.shape
    gamma, beta = _opt_f32(gamma), _opt_f32(beta)
    y = np.empty(x.shape, np.float32)
    q = np.empty(x.shape, np.int8) if quantized else None
    qp = QParams()
    if stats is None:
        stats = np.empty((3, Cc), np.float32)
        lib().orc_range_bn_fwd(_p(x), N, Cc, H, W, _p(gamma), _p(beta), C.c_float(eps), _p(y),
                               _p(stats), _p(q), C.byref(qp))
    else:
        stats = _f32(stats)
        lib().orc_range_bn_fwd_apply(_p(x), N, Cc, H, W, _p(gamma), _p(beta), C.c_float(eps),
                                     _p(stats), _p(y), _p(q), C.byref(qp))
    return y, stats, q, (qp if quantized else None)


def range_bn_bwd_sums(x, dy, stats, eps=0.0):
    x, dy, stats = _f32(x), _f32(dy), _f32(stats)
    N, Cc, H, W = x.shape
    sums = np.empty((2, Cc), np.float64)
    lib().orc_range_bn_bwd_sums(_p(x), _p(dy), _p(stats), N, Cc, H, W, C.c_float(eps), _p(sums))
    return sums


def range_bn_bwd(x, dy, stats, gamma=None, eps=0.0, sums=None):
    """Returns (dx, dgamma, dbeta).  With `sums` given ([2,C] float64: sum dy,
    sum dy*xhat) only the elementwise stage runs."""
    x, dy, stats = _f32(x), _f32(dy), _f32(stats)
    N, Cc, H, W = x.shape
    gamma = _opt_f32(gamma)
    dx = np.empty(x.shape, np.float32)
    dgamma = np.empty(Cc, np.float32)
    dbeta = np.empty(Cc, np.float32)
    if sums is None:
        lib().orc_range_bn_bwd(_p(x), _p(dy), _p(stats), N, Cc, H, W, _p(gamma), C.c_float(eps),
                               _p(dx), _p(dgamma), _p(dbeta))
    else:
        sums = np.ascontiguousarray(sums, dtype=np.float64)
        lib().orc_range_bn_bwd_apply(_p(x), _p(dy), _p(stats), _p(sums), N, Cc, H, W, _p(gamma),
                                     C.c_float(eps), _p(dx), _p(dgamma), _p(dbeta))
    return dx, dgamma, dbeta


def range_bn_relu_fwd(x, stats, gamma=None, beta=None, eps=0.0, quantized=False):
    """Range BN followed by ReLU for given statistics.
    Returns (y, q_stored or None, QParams or None)."""
    x, stats = _f32(x), _f32(stats)
    N, Cc, H, W = x.shape
    gamma, beta = _opt_f32(gamma), _opt_f32(beta)
    y = np.empty(x.shape, np.float32)
    q = np.empty(x.shape, np.int8) if quantized else None
    qp = QParams()
    lib().orc_range_bn_relu_fwd_apply(_p(x), N, Cc, H, W, _p(gamma), _p(beta), C.c_float(eps),
                                      _p(stats), _p(y), _p(q), C.byref(qp))
    return y, q, (qp if quantized else None)


def range_bn_relu_mask(x, dy, stats, gamma=None, beta=None, eps=0.0):
    """The upstream gradient after the backward of the ReLU that follows a Range BN."""
    x, dy, stats = _f32(x), _f32(dy), _f32(stats)
    N, Cc, H, W = x.shape
    gamma, beta = _opt_f32(gamma), _opt_f32(beta)
    out = np.empty(x.shape, np.float32)
    lib().orc_range_bn_relu_mask(_p(x), _p(dy), _p(stats), N, Cc, H, W, _p(gamma), _p(beta),
                                 C.c_float(eps), _p(out))
    return out


def range_bn_relu_bwd(x, dy, stats, gamma=None, beta=None, eps=0.0, sums=None):
    """Backward of Range BN + ReLU: the ReLU mask, then the Range BN backward on the masked
    gradient.  Returns (dx, dgamma, dbeta)."""
    return range_bn_bwd(x, range_bn_relu_mask(x, dy, stats, gamma, beta, eps), stats, gamma, eps, sums)


def range_bn_fwd_f64(x, gamma=None, beta=None, eps=0.0):
    x = np.ascontiguousarray(x, dtype=np.float64)
    N, Cc, H, W = x.shape
    g = None if gamma is None else np.ascontiguousarray(gamma, dtype=np.float64)
    b = None if beta is None else np.ascontiguousarray(beta, dtype=np.float64)
    y = np.empty(x.shape, np.float64)
    lib().orc_range_bn_fwd_f64(_p(x), N, Cc, H, W, _p(g), _p(b), C.c_double(eps), _p(y))
    return y


def standard_bn_f64(x):
    x = np.ascontiguousarray(x, dtype=np.float64)
    N, Cc, H, W = x.shape
    y = np.empty(x.shape, np.float64)
    lib().orc_standard_bn_f64(_p(x), N, Cc, H, W, _p(y))
    return y


# ------------------------------------------------------------------ ternarized back-propagation
def ternarize(x, seed=0):
    """Stochastic ternarization (appendix "Additional Experiments").  Returns (codes int8 in
    {-1,0,1} shaped like x, scale = max|x| as fp32)."""
    x = _f32(x)
    codes = np.empty(x.shape, np.int8)
    scale = C.c_float()
    lib().orc_ternarize(_p(x), C.c_int64(x.size), C.c_uint64(int(seed)), _p(codes), C.byref(scale))
    return codes, np.float32(scale.value)


def binarize(x):
    """+1 for x >= 0, -1 otherwise (int8)."""
    x = _f32(x)
    codes = np.empty(x.shape, np.int8)
    lib().orc_binarize(_p(x), C.c_int64(x.size), _p(codes))
    return codes


def pack_bits(codes, transpose=False):
    """Bit rows (uint32 words) of a 2-D matrix of +-1 codes; see orc_pack_bits."""
    codes = _i8(codes)
    rows, cols = codes.shape
    nr, nc = (cols, rows) if transpose else (rows, cols)
    out = np.empty((nr, (nc + 31) // 32), np.uint32)
    lib().orc_pack_bits(_p(codes), rows, cols, int(bool(transpose)), _p(out))
    return out


def xnor_gemm(abits, wbits, K):
    """y[m,n] = sum_k a[m,k] w[n,k] over +-1 values given as bit rows of K bits (int32)."""
    abits = np.ascontiguousarray(abits, dtype=np.uint32)
    wbits = np.ascontiguousarray(wbits, dtype=np.uint32)
    M, N = abits.shape[0], wbits.shape[0]
    assert abits.shape[1] == wbits.shape[1] == (K + 31) // 32
    y = np.empty((M, N), np.int32)
    lib().orc_xnor_gemm(_p(abits), _p(wbits), M, N, int(K), _p(y))
    return y


def tern_wgrad_multi(g, a_codes, S, seed=0):
    """Algorithm 1 for an FC layer: g [M,N] fp32, a_codes [M,K] +-1.  Returns (dW [K,N] fp32, acc int64)."""
    g = _f32(g)
    a_codes = _i8(a_codes)
    M, N = g.shape
    M2, K = a_codes.shape
    assert M == M2
    dw = np.empty((K, N), np.float32)
    acc = np.empty((K, N), np.int64)
    lib().orc_tern_wgrad_multi(_p(g), _p(a_codes), M, N, K, int(S), C.c_uint64(int(seed)), _p(dw), _p(acc))
    return dw, acc


# ------------------------------------------------------------------ network plumbing (not from the paper)
def range_bn_relu_maxpool_fwd(x, stats, gamma=None, beta=None, eps=0.0):
    """relu(Range BN(x)) followed by 3x3 / stride 2 / pad 1 max pooling.  Returns (pooled fp32, idx uint8)."""
    x, stats = _f32(x), _f32(stats)
    N, Cc, H, W = x.shape
    gamma, beta = _opt_f32(gamma), _opt_f32(beta)
    P, Q = (H - 1) // 2 + 1, (W - 1) // 2 + 1
    out = np.empty((N, Cc, P, Q), np.float32)
    idx = np.empty((N, Cc, P, Q), np.uint8)
    lib().orc_range_bn_relu_maxpool_fwd(_p(x), N, Cc, H, W, _p(gamma), _p(beta), C.c_float(eps), _p(stats), _p(out), _p(idx))
    return out, idx


def maxpool_relu_bwd(gpool, idx, H, W):
    gpool = _f32(gpool)
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    N, Cc = gpool.shape[:2]
    dy = np.empty((N, Cc, H, W), np.float32)
    lib().orc_maxpool_relu_bwd(_p(gpool), _p(idx), N, Cc, H, W, _p(dy))
    return dy


def add_relu(a, b):
    """Returns (relu(a + b), its maximum as fp32)."""
    a, b = _f32(a), _f32(b)
    out = np.empty(a.shape, np.float32)
    mx = C.c_float()
    lib().orc_add_relu(_p(a), _p(b), C.c_int64(a.size), _p(out), C.byref(mx))
    return out, np.float32(mx.value)


def range_bn_add_relu(x, stats, other, gamma=None, beta=None, other_stats=None, other_gamma=None, other_beta=None,
                      eps=0.0):
    """relu(bn(x; stats) + o), o = other or bn(other; other_stats); returns (out, max of out)"""
    x, other, stats = _f32(x), _f32(other), _f32(stats)
    N, Cc, H, W = x.shape
    out = np.empty(x.shape, np.float32)
    mx = C.c_float(0.0)
    lib().orc_range_bn_add_relu(_p(x), _p(stats), _p(_opt_f32(gamma)), _p(_opt_f32(beta)), _p(other),
                                _p(_opt_f32(other_stats)), _p(_opt_f32(other_gamma)), _p(_opt_f32(other_beta)),
                                N, Cc, H, W, C.c_float(eps), _p(out), C.byref(mx))
    return out, float(np.float32(mx.value))


def relu_bwd_sum(g1, g2=None, out=None):
    g1 = _f32(g1)
    g2, out = _opt_f32(g2), _opt_f32(out)
    res = np.empty(g1.shape, np.float32)
    lib().orc_relu_bwd_sum(_p(g1), _p(g2), _p(out), C.c_int64(g1.size), _p(res))
    return res


def relu_bwd_sum_lattice(g1, g2s, out, stride):
    g1, g2s = _f32(g1), _f32(g2s)
    out = _opt_f32(out)
    N, Cc, H, W = g1.shape
    assert g2s.shape == (N, Cc, (H + stride - 1) // stride, (W + stride - 1) // stride)
    res = np.empty(g1.shape, np.float32)
    lib().orc_relu_bwd_sum_lattice(_p(g1), _p(g2s), _p(out), N, Cc, H, W, int(stride), _p(res))
    return res


def relu_bwd_add(g, out, other=None):
    g, out = _f32(g), _f32(out)
    other = _opt_f32(other)
    res = np.empty(g.shape, np.float32)
    lib().orc_relu_bwd_add(_p(g), _p(out), _p(other), C.c_int64(g.size), _p(res))
    return res
