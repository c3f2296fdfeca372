"""ctypes access to the plain C oracle (oracle/vt_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the bench's cpu_baseline
leg.  The product package never imports this module.  No arithmetic of the method lives in
this file: it compiles the C source with gcc, loads it, and marshals numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "vt_oracle.c")
_LIB = os.path.join(_HERE, "libvt_oracle.so")
_lib = None

CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fno-unsafe-math-optimizations",
          "-shared", "-fPIC", "-std=c11", "-Wall", "-Wextra"]


class Conv2d(C.Structure):
    """vto_conv2d: geometry of a channels-last 2-D convolution."""
    _fields_ = [(k, C.c_int64) for k in ("N", "H", "W", "C", "KH", "KW", "stride_h", "stride_w", "pad_h", "pad_w",
                                         "dil_h", "dil_w")]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (scalar, no contraction, no fast-math)."""
    hdr = os.path.join(_HERE, "vt_oracle.h")
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= max(os.path.getmtime(_SRC), os.path.getmtime(hdr))):
        return _LIB
    subprocess.check_call(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        dp, fp = C.POINTER(C.c_double), C.POINTER(C.c_float)
        u32p, u64p = C.POINTER(C.c_uint32), C.POINTER(C.c_uint64)
        L.vto_rnd32_bits.restype = C.c_uint32
        L.vto_rnd32_bits.argtypes = [C.c_double]
        L.vto_thr_from_tau.restype = C.c_uint32
        L.vto_thr_from_tau.argtypes = [C.c_double]
        L.vto_scaled_round_error.restype = C.c_double
        L.vto_scaled_round_error.argtypes = [C.c_double]
        L.vto_boundary_distance.restype = C.c_uint32
        L.vto_boundary_distance.argtypes = [C.c_double]
        L.vto_ternary_code.restype = C.c_int
        L.vto_ternary_code.argtypes = [C.c_double, C.c_uint32]
        L.vto_round_log.restype = C.c_int
        L.vto_round_log.argtypes = [dp, C.c_uint64, C.c_double, fp, u32p, u32p, C.c_uint64, u64p]
        L.vto_round_replay.restype = C.c_int
        L.vto_round_replay.argtypes = [dp, C.c_uint64, u32p, u32p, C.c_uint64, fp]
        L.vto_gemm_f64.restype = C.c_int
        L.vto_gemm_f64.argtypes = [C.c_int, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_double,
                                   dp, C.c_int64, dp, C.c_int64, dp, dp, C.c_int64, C.c_int]
        u8p = C.POINTER(C.c_uint8)
        L.vto_ternary_pack5.restype = C.c_uint8
        L.vto_ternary_pack5.argtypes = [u8p]
        L.vto_ternary_unpack5.restype = None
        L.vto_ternary_unpack5.argtypes = [C.c_uint8, u8p]
        L.vto_round_log_dense.restype = C.c_int
        L.vto_round_log_dense.argtypes = [dp, C.c_uint64, C.c_double, fp, u8p, u64p]
        L.vto_round_replay_dense.restype = C.c_int
        L.vto_round_replay_dense.argtypes = [dp, C.c_uint64, u8p, fp]
        L.vto_rnd_b_bits.restype = C.c_uint32
        L.vto_rnd_b_bits.argtypes = [C.c_double, C.c_int]
        L.vto_scaled_round_error_b.restype = C.c_double
        L.vto_scaled_round_error_b.argtypes = [C.c_double, C.c_int]
        L.vto_boundary_distance_b.restype = C.c_uint32
        L.vto_boundary_distance_b.argtypes = [C.c_double, C.c_int]
        L.vto_ternary_code_b.restype = C.c_int
        L.vto_ternary_code_b.argtypes = [C.c_double, C.c_uint32, C.c_int]
        L.vto_round_log_b.restype = C.c_int
        L.vto_round_log_b.argtypes = [dp, C.c_uint64, C.c_double, C.c_int, fp, u32p, u32p, C.c_uint64, u64p]
        L.vto_round_replay_b.restype = C.c_int
        L.vto_round_replay_b.argtypes = [dp, C.c_uint64, u32p, u32p, C.c_uint64, C.c_int, fp]
        L.vto_round_log_dense_b.restype = C.c_int
        L.vto_round_log_dense_b.argtypes = [dp, C.c_uint64, C.c_double, C.c_int, fp, u8p, u64p]
        L.vto_round_replay_dense_b.restype = C.c_int
        L.vto_round_replay_dense_b.argtypes = [dp, C.c_uint64, u8p, C.c_int, fp]
        L.vto_threshold_stats_b.restype = C.c_int
        L.vto_threshold_stats_b.argtypes = [dp, dp, C.c_uint64, C.c_int, u64p]
        L.vto_elementwise_f64.restype = C.c_int
        L.vto_elementwise_f64.argtypes = [C.c_int, dp, dp, C.c_uint64, dp, C.c_int]
        L.vto_layernorm_f64.restype = C.c_int
        L.vto_layernorm_f64.argtypes = [dp, C.c_int64, C.c_int64, dp, dp, C.c_double, dp, C.c_int]
        L.vto_batchnorm_f64.restype = C.c_int
        L.vto_batchnorm_f64.argtypes = [dp, C.c_int64, C.c_int64, dp, dp, C.c_double, C.c_int, dp, C.c_int]
        L.vto_softmax_f64.restype = C.c_int
        L.vto_softmax_f64.argtypes = [dp, C.c_int64, C.c_int64, C.c_double, C.c_int64, dp, C.c_int]
        L.vto_conv2d_out_size.restype = C.c_int
        L.vto_conv2d_out_size.argtypes = [C.POINTER(Conv2d), C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        L.vto_conv2d_fwd_f64.restype = C.c_int
        L.vto_conv2d_fwd_f64.argtypes = [C.POINTER(Conv2d), C.c_int64, dp, dp, dp, dp, C.c_int]
        L.vto_conv2d_wgrad_f64.restype = C.c_int
        L.vto_conv2d_wgrad_f64.argtypes = [C.POINTER(Conv2d), C.c_int64, dp, dp, dp, C.c_int]
        L.vto_conv2d_dgrad_f64.restype = C.c_int
        L.vto_conv2d_dgrad_f64.argtypes = [C.POINTER(Conv2d), C.c_int64, dp, dp, dp, C.c_int]
        L.vto_threshold_stats.restype = C.c_int
        L.vto_threshold_stats.argtypes = [dp, dp, C.c_uint64, u64p]
        _lib = L
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct)) if a is not None else None


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def rnd32_bits(x: float) -> int:
    return int(lib().vto_rnd32_bits(float(x)))


def thr_from_tau(tau_ulp: float) -> int:
    return int(lib().vto_thr_from_tau(float(tau_ulp)))


def rnd_bits(x: float, b_r: int = 32) -> int:
    return int(lib().vto_rnd_b_bits(float(x), int(b_r)))


def scaled_round_error(x: float, b_r: int = 32) -> float:
    return float(lib().vto_scaled_round_error_b(float(x), int(b_r)))


def boundary_distance(x: float, b_r: int = 32) -> int:
    return int(lib().vto_boundary_distance_b(float(x), int(b_r)))


def ternary_code(x: float, thr: int, b_r: int = 32) -> int:
    return int(lib().vto_ternary_code_b(float(x), int(thr), int(b_r)))


def round_log(x, tau_ulp: float, cap: int | None = None, b_r: int = 32):
    """Returns (y float32[n], idx uint32[min(count,cap)], dir words uint32[ceil(cap/32)], count)."""
    x = _f64(x).ravel()
    n = x.size
    cap = n if cap is None else int(cap)
    y = np.empty(n, np.float32)
    idx = np.zeros(max(cap, 1), np.uint32)
    dirw = np.zeros(max((cap + 31) // 32, 1), np.uint32)
    cnt = C.c_uint64(0)
    rc = lib().vto_round_log_b(_p(x, C.c_double), n, float(tau_ulp), int(b_r), _p(y, C.c_float),
                               _p(idx, C.c_uint32), _p(dirw, C.c_uint32), cap, C.byref(cnt))
    if rc != 0:
        raise ValueError(f"vto_round_log: error {rc}")
    c = int(cnt.value)
    k = min(c, cap)
    return y, idx[:k].copy(), dirw[:(k + 31) // 32].copy(), c


def round_replay(x, idx, dirw, count: int | None = None, b_r: int = 32):
    x = _f64(x).ravel()
    idx = np.ascontiguousarray(idx, dtype=np.uint32)
    dirw = np.ascontiguousarray(dirw, dtype=np.uint32)
    count = idx.size if count is None else int(count)
    assert dirw.size * 32 >= count and idx.size >= count
    y = np.empty(x.size, np.float32)
    rc = lib().vto_round_replay_b(_p(x, C.c_double), x.size, _p(idx, C.c_uint32),
                                  _p(dirw, C.c_uint32), count, int(b_r), _p(y, C.c_float))
    if rc != 0:
        raise ValueError(f"vto_round_replay: error {rc}")
    return y


def ternary_pack5(codes) -> int:
    c = np.ascontiguousarray(codes, np.uint8)
    assert c.size == 5
    return int(lib().vto_ternary_pack5(_p(c, C.c_uint8)))


def ternary_unpack5(byte: int):
    c = np.zeros(5, np.uint8)
    lib().vto_ternary_unpack5(int(byte), _p(c, C.c_uint8))
    return c


def round_log_dense(x, tau_ulp: float, b_r: int = 32):
    """Returns (y float32[n], tlog uint8[ceil(n/5)], n_logged)."""
    x = _f64(x).ravel()
    n = x.size
    y = np.empty(n, np.float32)
    tlog = np.zeros(max((n + 4) // 5, 1), np.uint8)
    cnt = C.c_uint64(0)
    rc = lib().vto_round_log_dense_b(_p(x, C.c_double), n, float(tau_ulp), int(b_r), _p(y, C.c_float),
                                     _p(tlog, C.c_uint8), C.byref(cnt))
    if rc != 0:
        raise ValueError(f"vto_round_log_dense: error {rc}")
    return y, tlog[:(n + 4) // 5].copy(), int(cnt.value)


def round_replay_dense(x, tlog, b_r: int = 32):
    x = _f64(x).ravel()
    n = x.size
    t = np.ascontiguousarray(tlog, np.uint8)
    assert t.size >= (n + 4) // 5
    if t.size == 0:
        t = np.zeros(1, np.uint8)
    y = np.empty(n, np.float32)
    rc = lib().vto_round_replay_dense_b(_p(x, C.c_double), n, _p(t, C.c_uint8), int(b_r), _p(y, C.c_float))
    if rc != 0:
        raise ValueError(f"vto_round_replay_dense: error {rc}")
    return y


def gemm_f64(A, B, *, transA=False, transB=False, alpha=1.0, bias=None, order=0):
    """A, B are 2-D row-major arrays as stored; transX says the stored array is op(X)^T."""
    A, B = _f64(A), _f64(B)
    M, K = (A.shape[1], A.shape[0]) if transA else A.shape
    K2, N = (B.shape[1], B.shape[0]) if transB else B.shape
    assert K == K2
    if bias is not None:
        bias = _f64(bias)
        assert bias.size == N
    Cm = np.empty((M, N), np.float64)
    rc = lib().vto_gemm_f64(int(transA), int(transB), M, N, K, float(alpha),
                            _p(A, C.c_double), A.shape[1], _p(B, C.c_double), B.shape[1],
                            _p(bias, C.c_double), _p(Cm, C.c_double), N, int(order))
    if rc != 0:
        raise ValueError(f"vto_gemm_f64: error {rc}")
    return Cm


def conv2d_geometry(xshape, KH, KW, stride=1, pad=0, dil=1):
    """(Conv2d, Ho, Wo) for an input of shape (N, H, W, C); stride/pad/dil: int or (h, w) pair."""
    pair = lambda v: (int(v), int(v)) if np.isscalar(v) else (int(v[0]), int(v[1]))
    (sh, sw), (ph, pw), (dh, dw) = pair(stride), pair(pad), pair(dil)
    N, H, W, Cin = (int(v) for v in xshape)
    d = Conv2d(N, H, W, Cin, int(KH), int(KW), sh, sw, ph, pw, dh, dw)
    ho, wo = C.c_int64(), C.c_int64()
    if lib().vto_conv2d_out_size(C.byref(d), C.byref(ho), C.byref(wo)) != 0:
        raise ValueError("vto_conv2d_out_size: invalid geometry")
    return d, ho.value, wo.value


def conv2d_fwd(X, Wt, *, stride=1, pad=0, dil=1, bias=None, order=0):
    """X (N,H,W,C), Wt (KH,KW,C,Cout) -> Y (N,Ho,Wo,Cout)."""
    X, Wt = _f64(X), _f64(Wt)
    assert X.ndim == 4 and Wt.ndim == 4 and Wt.shape[2] == X.shape[3]
    d, Ho, Wo = conv2d_geometry(X.shape, Wt.shape[0], Wt.shape[1], stride, pad, dil)
    Cout = Wt.shape[3]
    if bias is not None:
        bias = _f64(bias)
        assert bias.size == Cout
    Y = np.empty((X.shape[0], Ho, Wo, Cout), np.float64)
    rc = lib().vto_conv2d_fwd_f64(C.byref(d), Cout, _p(X, C.c_double), _p(Wt, C.c_double), _p(bias, C.c_double),
                                  _p(Y, C.c_double), int(order))
    if rc != 0:
        raise ValueError(f"vto_conv2d_fwd_f64: error {rc}")
    return Y


def conv2d_wgrad(X, dY, KH, KW, *, stride=1, pad=0, dil=1, order=0):
    """X (N,H,W,C), dY (N,Ho,Wo,Cout) -> dW (KH,KW,C,Cout)."""
    X, dY = _f64(X), _f64(dY)
    d, Ho, Wo = conv2d_geometry(X.shape, KH, KW, stride, pad, dil)
    assert dY.shape[:3] == (X.shape[0], Ho, Wo)
    Cout = dY.shape[3]
    dW = np.empty((KH, KW, X.shape[3], Cout), np.float64)
    rc = lib().vto_conv2d_wgrad_f64(C.byref(d), Cout, _p(X, C.c_double), _p(dY, C.c_double), _p(dW, C.c_double),
                                    int(order))
    if rc != 0:
        raise ValueError(f"vto_conv2d_wgrad_f64: error {rc}")
    return dW


def conv2d_dgrad(dY, Wt, xshape, *, stride=1, pad=0, dil=1, order=0):
    """dY (N,Ho,Wo,Cout), Wt (KH,KW,C,Cout), input shape (N,H,W,C) -> dX (N,H,W,C)."""
    dY, Wt = _f64(dY), _f64(Wt)
    d, Ho, Wo = conv2d_geometry(xshape, Wt.shape[0], Wt.shape[1], stride, pad, dil)
    assert Wt.shape[2] == xshape[3] and dY.shape == (xshape[0], Ho, Wo, Wt.shape[3])
    dX = np.empty(tuple(int(v) for v in xshape), np.float64)
    rc = lib().vto_conv2d_dgrad_f64(C.byref(d), Wt.shape[3], _p(dY, C.c_double), _p(Wt, C.c_double),
                                    _p(dX, C.c_double), int(order))
    if rc != 0:
        raise ValueError(f"vto_conv2d_dgrad_f64: error {rc}")
    return dX


EW_ADD, EW_RELU, EW_GELU_TANH, EW_GELU_ERF = 0, 1, 2, 3


def elementwise(op: int, a, b=None, exact: bool = False):
    a = _f64(a)
    if b is not None:
        b = _f64(b)
        assert b.shape == a.shape
    y = np.empty(a.shape, np.float64)
    rc = lib().vto_elementwise_f64(int(op), _p(a, C.c_double), _p(b, C.c_double), a.size, _p(y, C.c_double),
                                   int(bool(exact)))
    if rc != 0:
        raise ValueError(f"vto_elementwise_f64: error {rc}")
    return y


def layernorm(x, gamma=None, beta=None, eps: float = 1e-5, order: int = 0):
    x = _f64(x)
    assert x.ndim == 2
    gamma = _f64(gamma) if gamma is not None else None
    beta = _f64(beta) if beta is not None else None
    y = np.empty(x.shape, np.float64)
    rc = lib().vto_layernorm_f64(_p(x, C.c_double), x.shape[0], x.shape[1], _p(gamma, C.c_double),
                                 _p(beta, C.c_double), float(eps), _p(y, C.c_double), int(order))
    if rc != 0:
        raise ValueError(f"vto_layernorm_f64: error {rc}")
    return y


def batchnorm(x, gamma=None, beta=None, eps: float = 1e-5, relu: bool = False, order: int = 0):
    """x: (rows, channels); statistics per channel over the rows (training mode)."""
    x = _f64(x)
    assert x.ndim == 2
    gamma = _f64(gamma) if gamma is not None else None
    beta = _f64(beta) if beta is not None else None
    y = np.empty(x.shape, np.float64)
    rc = lib().vto_batchnorm_f64(_p(x, C.c_double), x.shape[0], x.shape[1], _p(gamma, C.c_double),
                                 _p(beta, C.c_double), float(eps), int(bool(relu)), _p(y, C.c_double), int(order))
    if rc != 0:
        raise ValueError(f"vto_batchnorm_f64: error {rc}")
    return y


def softmax(x, scale: float = 1.0, causal_period: int = 0, order: int = 0):
    x = _f64(x)
    assert x.ndim == 2
    y = np.empty(x.shape, np.float64)
    rc = lib().vto_softmax_f64(_p(x, C.c_double), x.shape[0], x.shape[1], float(scale), int(causal_period),
                               _p(y, C.c_double), int(order))
    if rc != 0:
        raise ValueError(f"vto_softmax_f64: error {rc}")
    return y


def threshold_stats(y1, y2, b_r: int = 32):
    y1, y2 = _f64(y1).ravel(), _f64(y2).ravel()
    assert y1.size == y2.size
    out = np.zeros(68, np.uint64)
    rc = lib().vto_threshold_stats_b(_p(y1, C.c_double), _p(y2, C.c_double), y1.size, int(b_r),
                                     _p(out, C.c_uint64))
    if rc != 0:
        raise ValueError(f"vto_threshold_stats: error {rc}")
    return {"n_flip": int(out[0]), "thr_flip": int(out[1]), "max_ulp64_diff": int(out[2]),
            "hist": out[3:].astype(np.uint64).copy()}
