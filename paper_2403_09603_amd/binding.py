"""ctypes binding of libvt_hip.so -- argument marshalling only.

Function names and argument meaning follow include/vt.h one to one.  Tensors must live on the
GPU and be contiguous; PyTorch supplies device memory and the current HIP stream, nothing else.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libvt_hip.so")
_lib = None

VT_OP_ROUND_LOG, VT_OP_ROUND_REPLAY, VT_OP_GEMM_ROUND_LOG, VT_OP_THRESHOLD_STATS, VT_OP_GEMM_ROUND_LOG_BR = 0, 1, 2, 3, 4
VT_CONV_FORWARD, VT_CONV_WEIGHT_GRAD, VT_CONV_DATA_GRAD = 0, 1, 2
VT_A_ROW_MAJOR, VT_A_TRANSPOSED, VT_A_IM2COL_T = 0, 1, 3
VT_OP_LAYER_ROUND_LOG = 5
VT_LAYER_ADD, VT_LAYER_RELU, VT_LAYER_GELU_TANH, VT_LAYER_GELU_ERF, VT_LAYER_NORM, VT_LAYER_SOFTMAX = 0, 1, 2, 3, 4, 5
VT_LAYER_BATCHNORM, VT_LAYER_BATCHNORM_RELU = 6, 7
VT_OP_SHA256_TREE, VT_OP_MERKLE_ROOT = 6, 7
VT_OP_CONV_DGRAD_ROUND_LOG, VT_OP_CONV_DGRAD_ROUND_LOG_BR = 8, 9
VT_ROUND_LOG_STATIC_MAX_N = 1 << 30
VT_COUNT_ABANDONED = (1 << 64) - 1


class VtError(RuntimeError):
    pass


class _VtLog(C.Structure):
    _fields_ = [("idx", C.c_void_p), ("dir", C.c_void_p), ("cap", C.c_uint64), ("count", C.c_void_p),
                ("dense", C.c_void_p), ("b_r", C.c_int32)]


class Conv2d(C.Structure):
    """vt_conv2d of include/vt.h: geometry of a channels-last 2-D convolution."""
    _fields_ = [(k, C.c_int64) for k in ("N", "H", "W", "C", "KH", "KW", "stride_h", "stride_w", "pad_h", "pad_w",
                                         "dil_h", "dil_w")]


class _VtLayer(C.Structure):
    """vt_layer of include/vt.h."""
    _fields_ = [("op", C.c_int32), ("a", C.c_void_p), ("b", C.c_void_p), ("gamma", C.c_void_p), ("beta", C.c_void_p),
                ("rows", C.c_int64), ("cols", C.c_int64), ("eps", C.c_double), ("scale", C.c_double),
                ("causal_period", C.c_int64)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the HIP library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise VtError(f"{_LIB_PATH} is missing: build it with `python -m paper_2403_09603_amd.build` "
                      "(or __graft_entry__.build()); there is no CPU fallback")
    L = C.CDLL(_LIB_PATH)
    vp, i64, u64, dbl, cint = C.c_void_p, C.c_int64, C.c_uint64, C.c_double, C.c_int
    L.vt_round_log.restype = cint
    L.vt_round_log.argtypes = [vp, u64, dbl, vp, C.POINTER(_VtLog), vp, C.c_size_t, vp]
    L.vt_round_log_static.restype = cint
    L.vt_round_log_static.argtypes = [vp, u64, dbl, vp, C.POINTER(_VtLog), vp]
    L.vt_round_replay.restype = cint
    L.vt_round_replay.argtypes = [vp, u64, vp, vp, u64, vp, vp, C.c_size_t, vp]
    L.vt_round_replay_dense.restype = cint
    L.vt_round_replay_dense.argtypes = [vp, u64, vp, vp, vp]
    L.vt_round_replay_br.restype = cint
    L.vt_round_replay_br.argtypes = [vp, u64, vp, vp, u64, cint, vp, vp]
    L.vt_round_replay_dense_br.restype = cint
    L.vt_round_replay_dense_br.argtypes = [vp, u64, vp, cint, vp, vp]
    L.vt_threshold_stats_br.restype = cint
    L.vt_threshold_stats_br.argtypes = [vp, vp, u64, cint, vp, vp]
    L.vt_gemm_f64_round_log.restype = cint
    L.vt_gemm_f64_round_log.argtypes = [cint, cint, i64, i64, i64, dbl, vp, i64, i64, vp, i64, i64, vp, i64,
                                        vp, i64, i64, vp, cint, dbl, C.POINTER(_VtLog), vp, C.c_size_t, vp]
    L.vt_gemm_f64_round_log_nested.restype = cint
    L.vt_gemm_f64_round_log_nested.argtypes = [cint, cint, i64, i64, i64, dbl, vp, i64, i64, i64, vp, i64, i64, i64, vp,
                                               i64, i64, vp, i64, i64, vp, cint, dbl, C.POINTER(_VtLog), vp,
                                               C.c_size_t, vp]
    L.vt_conv2d_f64_round_log.restype = cint
    L.vt_conv2d_f64_round_log.argtypes = [cint, C.POINTER(Conv2d), i64, vp, vp, vp, vp, vp, cint, dbl,
                                          C.POINTER(_VtLog), vp, C.c_size_t, vp]
    L.vt_conv2d_gemm_shape.restype = cint
    L.vt_conv2d_gemm_shape.argtypes = [C.POINTER(Conv2d), i64, cint, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]
    L.vt_layer_f64_round_log.restype = cint
    L.vt_layer_f64_round_log.argtypes = [C.POINTER(_VtLayer), vp, vp, cint, dbl, C.POINTER(_VtLog), vp, C.c_size_t, vp]
    L.vt_threshold_stats.restype = cint
    L.vt_threshold_stats.argtypes = [vp, vp, u64, vp, vp]
    L.vt_sha256_tree.restype = cint
    L.vt_sha256_tree.argtypes = [vp, u64, u64, vp, vp, C.c_size_t, vp]
    L.vt_merkle_root.restype = cint
    L.vt_merkle_root.argtypes = [vp, u64, vp, vp, C.c_size_t, vp]
    L.vt_workspace_bytes.restype = C.c_size_t
    L.vt_workspace_bytes.argtypes = [cint, i64, i64, i64, i64]
    L.vt_thr_from_tau.restype = C.c_uint32
    L.vt_thr_from_tau.argtypes = [dbl]
    L.vt_thr_layer_from_stats.restype = C.c_uint32
    L.vt_thr_layer_from_stats.argtypes = [C.c_uint64, C.c_uint64]
    L.vt_gemm_plan.restype = cint
    L.vt_gemm_plan.argtypes = [cint, i64, i64, i64, i64, i64, i64, C.POINTER(cint), C.POINTER(cint), C.POINTER(cint)]
    L.vt_gemm_tail_plan.restype = cint
    L.vt_gemm_tail_plan.argtypes = [cint, i64, i64, i64, i64, i64, i64, C.POINTER(cint), C.POINTER(cint)]
    L.vt_set_kernel_events.restype = cint
    L.vt_set_kernel_events.argtypes = [vp, vp]
    L.vt_strerror.restype = C.c_char_p
    L.vt_strerror.argtypes = [cint]
    _lib = L
    return L


def vt_strerror(code: int) -> str:
    return load_library().vt_strerror(int(code)).decode()


def _check(code: int, what: str):
    if code != 0:
        raise VtError(f"{what}: {vt_strerror(code)} (status {code})")


def _ptr(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise VtError("tensor must be on the GPU")
    if not t.is_contiguous():
        raise VtError("tensor must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise VtError(f"expected {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


@dataclass
class Log:
    """Caller-owned device buffers of one log segment (the vt_log struct of include/vt.h)."""
    idx: torch.Tensor      # int32 [cap]  (bit pattern of uint32 indices)
    dir: torch.Tensor      # int32 [ceil(cap/32)]
    count: torch.Tensor    # int64 [1]
    cap: int
    dense: torch.Tensor | None = None   # uint8 [ceil(total/5)]: packed ternary log (then cap is 0)
    b_r: int = 32          # rounding amount the trainer call uses (10 .. 32)

    def read_count(self, check_cap: bool = True) -> int:
        """Synchronising read of the count word (see check_count)."""
        return check_count(self.count.item(), self.cap if check_cap and self.dense is None else None)

    def _c(self) -> _VtLog:
        if self.dense is not None and (not self.dense.is_cuda or self.dense.dtype != torch.uint8):
            raise VtError("dense log must be a uint8 tensor on the GPU")
        return _VtLog(self.idx.data_ptr() if self.cap else None, self.dir.data_ptr() if self.cap else None,
                      self.cap, self.count.data_ptr(), self.dense.data_ptr() if self.dense is not None else None,
                      int(self.b_r))


class VtLogAbandoned(VtError):
    """*count == VT_COUNT_ABANDONED: the ordered-log pass gave up a bounded wait; outputs valid, log not."""


def check_count(raw: int, cap: int | None = None) -> int:
    """The value read from a log's count word as a number of entries.  Raises VtLogAbandoned for the
    VT_COUNT_ABANDONED sentinel (run the call again) and VtError when the log overflowed `cap`
    (run it again with a larger log)."""
    raw = int(raw) & ((1 << 64) - 1)
    if raw == VT_COUNT_ABANDONED:
        raise VtLogAbandoned("ordered-log pass abandoned (count == VT_COUNT_ABANDONED): FP32 outputs are valid, "
                             "idx/dir are not; repeat the call")
    if cap is not None and raw > int(cap):
        raise VtError(f"log overflow: {raw} entries for a capacity of {int(cap)}; repeat the call with a larger log")
    return raw


def alloc_log(cap: int, device="cuda") -> Log:
    cap = int(cap)
    return Log(torch.empty(max(cap, 1), dtype=torch.int32, device=device),
               torch.empty(max((cap + 31) // 32, 1), dtype=torch.int32, device=device),
               torch.zeros(1, dtype=torch.int64, device=device), cap)


def alloc_dense_log(total: int, device="cuda") -> Log:
    """Buffers for the packed ternary form of the log of `total` outputs (five entries per byte)."""
    total = int(total)
    return Log(torch.empty(1, dtype=torch.int32, device=device), torch.empty(1, dtype=torch.int32, device=device),
               torch.zeros(1, dtype=torch.int64, device=device), 0,
               torch.empty(max((total + 4) // 5, 4), dtype=torch.uint8, device=device))


def vt_workspace_bytes(op: int, M: int, N: int, K: int = 0, batch: int = 1) -> int:
    return int(load_library().vt_workspace_bytes(int(op), int(M), int(N), int(K), int(batch)))


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def vt_thr_from_tau(tau_ulp: float) -> int:
    return int(load_library().vt_thr_from_tau(float(tau_ulp)))


def vt_round_log(x: torch.Tensor, tau_ulp: float, y: torch.Tensor, log: Log, ws: torch.Tensor, stream=None):
    n = x.numel()
    if y.numel() != n:
        raise VtError("y must have as many elements as x")
    if log.dense is not None and log.dense.numel() < (n + 4) // 5:
        raise VtError("dense log is smaller than ceil(n/5) bytes")
    clog = log._c()
    _check(load_library().vt_round_log(_ptr(x, torch.float64), n, float(tau_ulp), _ptr(y, torch.float32),
                                       C.byref(clog), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)),
           "vt_round_log")


def vt_round_log_static(x: torch.Tensor, tau_ulp: float, y: torch.Tensor, log: Log, stream=None):
    """vt_round_log with the library's own static scratch instead of a workspace (allocates nothing)."""
    n = x.numel()
    if y.numel() != n:
        raise VtError("y must have as many elements as x")
    if log.dense is not None and log.dense.numel() < (n + 4) // 5:
        raise VtError("dense log is smaller than ceil(n/5) bytes")
    clog = log._c()
    _check(load_library().vt_round_log_static(_ptr(x, torch.float64), n, float(tau_ulp), _ptr(y, torch.float32),
                                              C.byref(clog), _stream(stream)), "vt_round_log_static")


def vt_round_replay(x: torch.Tensor, idx: torch.Tensor, dir: torch.Tensor, count: int, y: torch.Tensor,
                    stream=None, b_r: int = 32):
    n = x.numel()
    if y.numel() != n:
        raise VtError("y must have as many elements as x")
    count = int(count)
    if count > idx.numel() or (count + 31) // 32 > dir.numel():
        raise VtError("count exceeds the log buffers")
    if b_r == 32:
        _check(load_library().vt_round_replay(_ptr(x, torch.float64), n, _ptr(idx, torch.int32),
                                              _ptr(dir, torch.int32), count, _ptr(y, torch.float32), None, 0,
                                              _stream(stream)), "vt_round_replay")
    else:
        _check(load_library().vt_round_replay_br(_ptr(x, torch.float64), n, _ptr(idx, torch.int32),
                                                 _ptr(dir, torch.int32), count, int(b_r), _ptr(y, torch.float32),
                                                 _stream(stream)), "vt_round_replay_br")


def vt_round_replay_dense(x: torch.Tensor, tlog: torch.Tensor, y: torch.Tensor, stream=None, b_r: int = 32):
    n = x.numel()
    if y.numel() != n:
        raise VtError("y must have as many elements as x")
    if tlog.dtype != torch.uint8 or tlog.numel() < (n + 4) // 5:
        raise VtError("tlog must be a uint8 tensor of ceil(n/5) bytes")
    if b_r == 32:
        _check(load_library().vt_round_replay_dense(_ptr(x, torch.float64), n, _ptr(tlog), _ptr(y, torch.float32),
                                                    _stream(stream)), "vt_round_replay_dense")
    else:
        _check(load_library().vt_round_replay_dense_br(_ptr(x, torch.float64), n, _ptr(tlog), int(b_r),
                                                       _ptr(y, torch.float32), _stream(stream)),
               "vt_round_replay_dense_br")


def vt_gemm_f64_round_log(transA: bool, transB: bool, M: int, N: int, K: int, alpha: float,
                          A: torch.Tensor, lda: int, strideA: int, B: torch.Tensor, ldb: int, strideB: int,
                          bias, batch: int, C32: torch.Tensor, ldc: int, strideC: int, C64_debug,
                          variant: int, tau_ulp: float, log: Log, ws: torch.Tensor, stream=None):
    # extent checks: the kernels trust lda/ldb/ldc/strides, so make sure the tensors cover them
    def need(rows, cols, ld, stride):
        return 0 if rows == 0 or cols == 0 or batch == 0 else (batch - 1) * stride + (rows - 1) * ld + cols
    if A.numel() < need(K if transA else M, M if transA else K, lda, strideA):
        raise VtError("A is smaller than M, K, lda, strideA, batch imply")
    if B.numel() < need(N if transB else K, K if transB else N, ldb, strideB):
        raise VtError("B is smaller than K, N, ldb, strideB, batch imply")
    if C32.numel() < need(M, N, ldc, strideC):
        raise VtError("C32 is smaller than M, N, ldc, strideC, batch imply")
    if bias is not None and bias.numel() < N:
        raise VtError("bias is shorter than N")
    if C64_debug is not None and C64_debug.numel() < M * N * batch:
        raise VtError("C64_debug is smaller than M*N*batch")
    if log.dense is not None and log.dense.numel() < (M * N * batch + 4) // 5:
        raise VtError("dense log is smaller than ceil(M*N*batch/5) bytes")
    clog = log._c()
    _check(load_library().vt_gemm_f64_round_log(
        int(bool(transA)), int(bool(transB)), int(M), int(N), int(K), float(alpha),
        _ptr(A, torch.float64), int(lda), int(strideA), _ptr(B, torch.float64), int(ldb), int(strideB),
        _ptr(bias, torch.float64), int(batch), _ptr(C32, torch.float32), int(ldc), int(strideC),
        _ptr(C64_debug, torch.float64), int(variant), float(tau_ulp), C.byref(clog),
        _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)), "vt_gemm_f64_round_log")


def vt_gemm_f64_round_log_nested(transA: bool, transB: bool, M: int, N: int, K: int, alpha: float,
                                 A: torch.Tensor, lda: int, strideA: int, strideA_outer: int,
                                 B: torch.Tensor, ldb: int, strideB: int, strideB_outer: int,
                                 bias, batch_inner: int, batch_outer: int, C32: torch.Tensor, ldc: int, strideC: int,
                                 C64_debug, variant: int, tau_ulp: float, log: Log, ws: torch.Tensor, stream=None):
    batch = batch_inner * batch_outer

    def need(rows, cols, ld, s_in, s_out):
        if rows == 0 or cols == 0 or batch == 0:
            return 0
        return (batch_outer - 1) * s_out + (batch_inner - 1) * s_in + (rows - 1) * ld + cols
    if A.numel() < need(K if transA else M, M if transA else K, lda, strideA, strideA_outer):
        raise VtError("A is smaller than the shape, pitches and batch strides imply")
    if B.numel() < need(N if transB else K, K if transB else N, ldb, strideB, strideB_outer):
        raise VtError("B is smaller than the shape, pitches and batch strides imply")
    if batch and M and N and C32.numel() < (batch - 1) * strideC + (M - 1) * ldc + N:
        raise VtError("C32 is smaller than M, N, ldc, strideC and the batch imply")
    if bias is not None and bias.numel() < N:
        raise VtError("bias is shorter than N")
    if C64_debug is not None and C64_debug.numel() < M * N * batch:
        raise VtError("C64_debug is smaller than M*N*batch")
    if log.dense is not None and log.dense.numel() < (M * N * batch + 4) // 5:
        raise VtError("dense log is smaller than ceil(M*N*batch/5) bytes")
    clog = log._c()
    _check(load_library().vt_gemm_f64_round_log_nested(
        int(bool(transA)), int(bool(transB)), int(M), int(N), int(K), float(alpha),
        _ptr(A, torch.float64), int(lda), int(strideA), int(strideA_outer),
        _ptr(B, torch.float64), int(ldb), int(strideB), int(strideB_outer),
        _ptr(bias, torch.float64), int(batch_inner), int(batch_outer), _ptr(C32, torch.float32), int(ldc), int(strideC),
        _ptr(C64_debug, torch.float64), int(variant), float(tau_ulp), C.byref(clog),
        _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)), "vt_gemm_f64_round_log_nested")


def vt_conv2d_gemm_shape(d: Conv2d, Cout: int, mode: int):
    """(M, N, K) of the GEMM the convolution runs as (sizes the workspace and the outputs)."""
    M, N, K = C.c_int64(), C.c_int64(), C.c_int64()
    _check(load_library().vt_conv2d_gemm_shape(C.byref(d), int(Cout), int(mode), C.byref(M), C.byref(N), C.byref(K)),
           "vt_conv2d_gemm_shape")
    return M.value, N.value, K.value


def vt_conv2d_f64_round_log(mode: int, d: Conv2d, Cout: int, X: torch.Tensor, B: torch.Tensor, bias,
                            C32: torch.Tensor, C64_debug, variant: int, tau_ulp: float, log: Log,
                            ws: torch.Tensor, stream=None):
    M, N, K = vt_conv2d_gemm_shape(d, Cout, mode)
    if mode == VT_CONV_DATA_GRAD:
        Mf, _, _ = vt_conv2d_gemm_shape(d, Cout, VT_CONV_FORWARD)
        if X.numel() < Mf * Cout:
            raise VtError("dY is smaller than N*Ho*Wo*Cout")
    elif X.numel() < d.N * d.H * d.W * d.C:
        raise VtError("X is smaller than N*H*W*C")
    if B.numel() < K * N:
        raise VtError("B is smaller than the geometry implies")
    if C32.numel() < M * N or (C64_debug is not None and C64_debug.numel() < M * N):
        raise VtError("output is smaller than the geometry implies")
    if bias is not None and bias.numel() < N:
        raise VtError("bias is shorter than Cout")
    if log.dense is not None and log.dense.numel() < (M * N + 4) // 5:
        raise VtError("dense log is smaller than ceil(outputs/5) bytes")
    clog = log._c()
    _check(load_library().vt_conv2d_f64_round_log(
        int(mode), C.byref(d), int(Cout), _ptr(X, torch.float64), _ptr(B, torch.float64), _ptr(bias, torch.float64),
        _ptr(C32, torch.float32), _ptr(C64_debug, torch.float64), int(variant), float(tau_ulp), C.byref(clog),
        _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)), "vt_conv2d_f64_round_log")


def vt_layer_f64_round_log(op: int, a: torch.Tensor, b, gamma, beta, rows: int, cols: int, y: torch.Tensor, y64_debug,
                           variant: int, tau_ulp: float, log: Log, ws: torch.Tensor, *, eps: float = 1e-5,
                           scale: float = 1.0, causal_period: int = 0, stream=None):
    n = int(rows) * int(cols)
    if a.numel() < n or y.numel() < n or (b is not None and b.numel() < n):
        raise VtError("a, b and y must hold rows*cols elements")
    if (gamma is not None and gamma.numel() < cols) or (beta is not None and beta.numel() < cols):
        raise VtError("gamma and beta must hold cols elements")
    if y64_debug is not None and y64_debug.numel() < n:
        raise VtError("y64_debug must hold rows*cols elements")
    if log.dense is not None and log.dense.numel() < (n + 4) // 5:
        raise VtError("dense log is smaller than ceil(rows*cols/5) bytes")
    layer = _VtLayer(int(op), a.data_ptr() if n else None, b.data_ptr() if b is not None and n else None,
                     gamma.data_ptr() if gamma is not None else None, beta.data_ptr() if beta is not None else None,
                     int(rows), int(cols), float(eps), float(scale), int(causal_period))
    for t in (a, b, gamma, beta):
        if t is not None:
            _ptr(t, torch.float64)
    clog = log._c()
    _check(load_library().vt_layer_f64_round_log(C.byref(layer), _ptr(y, torch.float32), _ptr(y64_debug, torch.float64),
                                                 int(variant), float(tau_ulp), C.byref(clog), _ptr(ws),
                                                 ws.numel() * ws.element_size(), _stream(stream)),
           "vt_layer_f64_round_log")


def vt_gemm_plan(M: int, N: int, K: int, batch: int = 1, ldc: int | None = None, strideC: int | None = None,
                 transA=False):
    """(tile_m, tile_n, splits) the GEMM entry point uses for this shape.  transA: False / True, or
    VT_A_IM2COL_T for the weight gradient of a convolution that is not 1 x 1 at every position."""
    tm, tn, sp = C.c_int(), C.c_int(), C.c_int()
    _check(load_library().vt_gemm_plan(int(transA), int(M), int(N), int(K), int(batch), int(N if ldc is None else ldc),
                                       int(M * N if strideC is None else strideC), C.byref(tm), C.byref(tn),
                                       C.byref(sp)), "vt_gemm_plan")
    return tm.value, tn.value, sp.value


def vt_gemm_tail_plan(M: int, N: int, K: int, batch: int = 1, ldc: int | None = None, strideC: int | None = None,
                      transA=False):
    """(tail_tiles, slices): see vt_gemm_tail_plan in include/vt.h."""
    tiles, slices = C.c_int(0), C.c_int(0)
    ldc = N if ldc is None else ldc
    strideC = M * N if strideC is None else strideC
    _check(load_library().vt_gemm_tail_plan(int(transA), M, N, K, batch, ldc, strideC, C.byref(tiles), C.byref(slices)),
           "vt_gemm_tail_plan")
    return tiles.value, slices.value


def vt_set_kernel_events(ev_begin, ev_end):
    """ev_begin / ev_end: raw hipEvent_t handles (ints) or None to clear."""
    _check(load_library().vt_set_kernel_events(C.c_void_p(ev_begin) if ev_begin else None,
                                               C.c_void_p(ev_end) if ev_end else None), "vt_set_kernel_events")


def vt_threshold_stats(y1: torch.Tensor, y2: torch.Tensor, out: torch.Tensor, stream=None, b_r: int = 32):
    if y1.numel() != y2.numel():
        raise VtError("y1 and y2 differ in size")
    if out.numel() < 68 or out.dtype != torch.int64:
        raise VtError("out must be an int64 tensor of 68 elements")
    if b_r == 32:
        _check(load_library().vt_threshold_stats(_ptr(y1, torch.float64), _ptr(y2, torch.float64), y1.numel(),
                                                 _ptr(out), _stream(stream)), "vt_threshold_stats")
    else:
        _check(load_library().vt_threshold_stats_br(_ptr(y1, torch.float64), _ptr(y2, torch.float64), y1.numel(),
                                                    int(b_r), _ptr(out), _stream(stream)), "vt_threshold_stats_br")


VT_THR_LAYER_MAX = 1 << 27


def vt_thr_layer_from_stats(thr_flip: int, max_ulp64_diff: int) -> int:
    return int(load_library().vt_thr_layer_from_stats(int(thr_flip), int(max_ulp64_diff)))


def vt_sha256_tree(data: torch.Tensor, chunk: int, digest: torch.Tensor, ws: torch.Tensor, stream=None):
    """Hash the bytes of `data` (any dtype, on the GPU) into the 32-byte uint8 tensor `digest`."""
    if digest.dtype != torch.uint8 or digest.numel() < 32:
        raise VtError("digest must be a uint8 tensor of 32 bytes")
    nbytes = data.numel() * data.element_size()
    _check(load_library().vt_sha256_tree(_ptr(data) if nbytes else None, nbytes, int(chunk), _ptr(digest), _ptr(ws),
                                         ws.numel() * ws.element_size(), _stream(stream)), "vt_sha256_tree")


def vt_merkle_root(leaves: torch.Tensor, root: torch.Tensor, ws: torch.Tensor, stream=None):
    """Merkle root of the 32-byte leaves (uint8 tensor of n x 32 bytes) into the 32-byte uint8 tensor `root`."""
    if leaves.dtype != torch.uint8 or root.dtype != torch.uint8 or leaves.numel() % 32 or root.numel() < 32:
        raise VtError("leaves must be n x 32 uint8 and root 32 uint8")
    _check(load_library().vt_merkle_root(_ptr(leaves), leaves.numel() // 32, _ptr(root), _ptr(ws),
                                         ws.numel() * ws.element_size(), _stream(stream)), "vt_merkle_root")
