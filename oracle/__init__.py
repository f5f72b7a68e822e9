"""ctypes access to the CPU oracle (oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the bench's CPU-baseline leg may import this
package.  It shares nothing with the HIP library and never imports it.

Arrays are numpy, in host memory: float32 for F32 inputs, uint16 bit
patterns for BF16 / F16 inputs, uint8 for the FP8 formats.  Results come back as float64, unrounded.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

F32, BF16, F16, FP8_E4M3, FP8_E5M2 = 0, 1, 2, 3, 4
EPI_NONE, EPI_BIAS, EPI_RELU, EPI_BIAS_RELU, EPI_BIAS_GELU_TANH, EPI_GELU_TANH = range(6)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_HDR = os.path.join(_HERE, "oracle.h")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc into liboracle.so (next to the source)."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_HDR)))
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        i64, vp, f32, i32 = ctypes.c_int64, ctypes.c_void_p, ctypes.c_float, ctypes.c_int
        L.oracle_matmul.argtypes = [vp, vp, vp, vp, vp] + [i64] * 6 + [i32, i32, f32, i32]
        L.oracle_batched_matmul.argtypes = [vp, vp, vp, vp, vp] + [i64] * 10 + [i32, i32, f32, i32]
        L.oracle_conv2d_nhwc.argtypes = [vp, vp, vp, vp, vp] + [i64] * 13 + [i32, f32, i32]
        L.oracle_batched_matmul_at.argtypes = ([vp, vp, vp, vp, vp] + [i64] * 8
                                               + [i32, i32, f32, i32, i64, vp, vp, vp])
        L.oracle_conv2d_nhwc_at.argtypes = ([vp, vp, vp, vp, vp] + [i64] * 13
                                            + [i32, f32, i32, i64, vp, vp, vp, vp])
        L.oracle_conv2d_nhwc_pad4.argtypes = [vp, vp, vp, vp, vp] + [i64] * 15 + [i32, f32, i32]
        L.oracle_conv2d_transpose_nhwc.argtypes = [vp, vp, vp, vp, vp] + [i64] * 15 + [i32, f32, i32]
        L.oracle_conv2d_transpose_nhwc_at.argtypes = ([vp, vp, vp, vp, vp] + [i64] * 15
                                                      + [i32, f32, i32, i64, vp, vp, vp, vp])
        L.oracle_conv_transpose_out_dim.argtypes = [i64] * 6
        L.oracle_conv_transpose_out_dim.restype = i64
        L.oracle_matmul_int8.argtypes = ([vp, vp, vp, vp] + [i64] * 6 + [i32, vp, vp, f32, vp, vp, i32, f32, i32])
        L.oracle_conv2d_nhwc_int8.argtypes = ([vp, vp, vp, vp] + [i64] * 13 + [vp, vp, f32, vp, vp, i32, f32, i32])
        L.oracle_matmul_int8_bn.argtypes = ([vp, vp, vp, vp] + [i64] * 6 + [i32, vp, vp, f32, vp, vp, f32, vp, vp, i32, f32, i32])
        L.oracle_conv2d_nhwc_int8_bn.argtypes = ([vp, vp, vp, vp] + [i64] * 13
                                                 + [vp, vp, f32, vp, vp, f32, vp, vp, i32, f32, i32])
        L.oracle_matmul_residual.argtypes = [vp, vp, vp, vp, vp, vp] + [i64] * 7 + [i32, i32, i32, f32, f32, i32]
        L.oracle_conv2d_nhwc_residual.argtypes = [vp, vp, vp, vp, vp, vp] + [i64] * 13 + [i32, i32, f32, f32, i32]
        L.oracle_attention.argtypes = [vp, vp, vp, vp, vp] + [i64] * 14 + [i32, f32]
        L.oracle_attention_rows.argtypes = [vp, vp, vp, vp, vp] + [i64] * 12 + [i32, f32, i64, vp, vp]
        L.oracle_attention_causal.argtypes = [vp, vp, vp, vp] + [i64] * 12 + [i32, f32]
        L.oracle_attention_causal_rows.argtypes = [vp, vp, vp, vp] + [i64] * 10 + [i32, f32, i64, vp, vp]
        L.oracle_conv_out_dim.argtypes = [i64] * 5
        L.oracle_conv_out_dim.restype = i64
        L.oracle_epilogue.argtypes = [ctypes.c_double, ctypes.c_double, f32, i32]
        L.oracle_epilogue.restype = ctypes.c_double
        L.oracle_gelu_tanh.argtypes = [ctypes.c_double]
        L.oracle_gelu_tanh.restype = ctypes.c_double
        L.oracle_widen.argtypes = [ctypes.c_uint32, i32]
        L.oracle_widen.restype = ctypes.c_double
        L.oracle_round_bf16.argtypes = [ctypes.c_double]
        L.oracle_round_bf16.restype = ctypes.c_uint16
        L.oracle_round_f16.argtypes = [ctypes.c_double]
        L.oracle_round_f16.restype = ctypes.c_uint16
        L.oracle_num_threads.restype = i32
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data


def _check_in(a: np.ndarray, dtype: int) -> np.ndarray:
    want = np.float32 if dtype == F32 else np.uint16 if dtype in (BF16, F16) else np.uint8
    if a.dtype != want:
        raise TypeError(f"dtype code {dtype} needs a {want.__name__} array, got {a.dtype}")
    return a


def _check_bias(bias):
    if bias is None:
        return None
    if bias.dtype != np.float32 or not bias.flags.c_contiguous:
        raise TypeError("bias must be contiguous float32")
    return bias


def _rc(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"{what}: oracle rejected the arguments (code {rc})")


def matmul(A, B, bias=None, *, dtype, trans_b=0, alpha=1.0, epi=EPI_NONE,
           M=None, N=None, K=None, lda=None, ldb=None, want_preact=False):
    """act(alpha*A.B + bias) as float64 [M][N]; A, B are 2-d arrays (or views
    described by M, N, K, lda, ldb over a contiguous parent)."""
    out = batched_matmul(A, B, bias, dtype=dtype, trans_b=trans_b, alpha=alpha, epi=epi,
                         batch=1, M=M if M is not None else A.shape[0],
                         N=N if N is not None else (B.shape[0] if trans_b else B.shape[1]),
                         K=K if K is not None else A.shape[1],
                         lda=lda if lda is not None else A.shape[1],
                         ldb=ldb if ldb is not None else B.shape[1],
                         stride_a=0, stride_b=0, want_preact=want_preact)
    if want_preact:
        return out[0][0], out[1][0]
    return out[0]


def batched_matmul(A, B, bias=None, *, dtype, trans_b=0, alpha=1.0, epi=EPI_NONE,
                   batch=None, M=None, N=None, K=None, lda=None, ldb=None,
                   stride_a=None, stride_b=None, want_preact=False):
    A = _check_in(np.ascontiguousarray(A), dtype)
    B = _check_in(np.ascontiguousarray(B), dtype)
    bias = _check_bias(bias)
    if batch is None:
        batch = A.shape[0]
    if M is None:
        M = A.shape[-2]
    if K is None:
        K = A.shape[-1]
    if N is None:
        N = B.shape[-2] if trans_b else B.shape[-1]
    if lda is None:
        lda = A.shape[-1]
    if ldb is None:
        ldb = B.shape[-1]
    if stride_a is None:
        stride_a = A.shape[-2] * A.shape[-1] if A.ndim == 3 else 0
    if stride_b is None:
        stride_b = B.shape[-2] * B.shape[-1] if B.ndim == 3 else 0
    out = np.empty((batch, M, N), dtype=np.float64)
    pre = np.empty_like(out) if want_preact else None
    rc = lib().oracle_batched_matmul(_ptr(A), _ptr(B), _ptr(bias), _ptr(out), _ptr(pre),
                                     batch, M, N, K, lda, ldb, N, stride_a, stride_b, M * N,
                                     dtype, int(trans_b), float(alpha), epi)
    _rc(rc, "batched_matmul")
    return (out, pre) if want_preact else out


def batched_matmul_at(A, B, bias, sb, si, sj, *, dtype, trans_b=0, alpha=1.0, epi=EPI_NONE,
                      batch, M, N, K, lda=None, ldb=None, stride_a=None, stride_b=None):
    """(out, preact) at the listed (batch, row, col) coordinates only."""
    A = _check_in(np.ascontiguousarray(A), dtype)
    B = _check_in(np.ascontiguousarray(B), dtype)
    bias = _check_bias(bias)
    sb = np.ascontiguousarray(sb, dtype=np.int64)
    si = np.ascontiguousarray(si, dtype=np.int64)
    sj = np.ascontiguousarray(sj, dtype=np.int64)
    if lda is None:
        lda = K
    if ldb is None:
        ldb = K if trans_b else N
    if stride_a is None:
        stride_a = M * lda
    if stride_b is None:
        stride_b = (N if trans_b else K) * ldb
    out = np.empty(len(si), dtype=np.float64)
    pre = np.empty_like(out)
    rc = lib().oracle_batched_matmul_at(_ptr(A), _ptr(B), _ptr(bias), _ptr(out), _ptr(pre),
                                        batch, M, N, K, lda, ldb, stride_a, stride_b,
                                        dtype, int(trans_b), float(alpha), epi,
                                        len(si), _ptr(sb), _ptr(si), _ptr(sj))
    _rc(rc, "batched_matmul_at")
    return out, pre


def conv_out_dim(size, k, stride, pad, dil) -> int:
    return int(lib().oracle_conv_out_dim(size, k, stride, pad, dil))


def conv2d_nhwc(x, w, bias=None, *, dtype, stride=(1, 1), pad=(0, 0), dil=(1, 1),
                alpha=1.0, epi=EPI_NONE, want_preact=False):
    """x [N][H][W][Cin], w [KH][KW][Cin][Cout] -> float64 [N][OH][OW][Cout]."""
    x = _check_in(np.ascontiguousarray(x), dtype)
    w = _check_in(np.ascontiguousarray(w), dtype)
    bias = _check_bias(bias)
    n, H, W, Cin = x.shape
    KH, KW, Cin2, Cout = w.shape
    if Cin2 != Cin:
        raise ValueError("channel mismatch")
    OH = conv_out_dim(H, KH, stride[0], pad[0], dil[0])
    OW = conv_out_dim(W, KW, stride[1], pad[1], dil[1])
    if OH < 0 or OW < 0:
        raise ValueError("empty output")
    out = np.empty((n, OH, OW, Cout), dtype=np.float64)
    pre = np.empty_like(out) if want_preact else None
    rc = lib().oracle_conv2d_nhwc(_ptr(x), _ptr(w), _ptr(bias), _ptr(out), _ptr(pre),
                                  n, H, W, Cin, Cout, KH, KW, stride[0], stride[1],
                                  pad[0], pad[1], dil[0], dil[1], dtype, float(alpha), epi)
    _rc(rc, "conv2d_nhwc")
    return (out, pre) if want_preact else out


def conv2d_nhwc_at(x, w, bias, sn, soh, sow, sco, *, dtype, stride=(1, 1), pad=(0, 0),
                   dil=(1, 1), alpha=1.0, epi=EPI_NONE):
    x = _check_in(np.ascontiguousarray(x), dtype)
    w = _check_in(np.ascontiguousarray(w), dtype)
    bias = _check_bias(bias)
    n, H, W, Cin = x.shape
    KH, KW, _, Cout = w.shape
    idx = [np.ascontiguousarray(v, dtype=np.int64) for v in (sn, soh, sow, sco)]
    out = np.empty(len(idx[0]), dtype=np.float64)
    pre = np.empty_like(out)
    rc = lib().oracle_conv2d_nhwc_at(_ptr(x), _ptr(w), _ptr(bias), _ptr(out), _ptr(pre),
                                     n, H, W, Cin, Cout, KH, KW, stride[0], stride[1],
                                     pad[0], pad[1], dil[0], dil[1], dtype, float(alpha), epi,
                                     len(out), *[_ptr(v) for v in idx])
    _rc(rc, "conv2d_nhwc_at")
    return out, pre


def conv2d_nhwc_pad4(x, w, bias=None, *, dtype, stride=(1, 1), pad=(0, 0, 0, 0), dil=(1, 1),
                     alpha=1.0, epi=EPI_NONE, want_preact=False):
    """Convolution with pad = (top, bottom, left, right); float64 [N][OH][OW][Cout]."""
    x = _check_in(np.ascontiguousarray(x), dtype)
    w = _check_in(np.ascontiguousarray(w), dtype)
    bias = _check_bias(bias)
    N, H, W, Cin = x.shape
    KH, KW, Cin2, Cout = w.shape
    if Cin2 != Cin:
        raise ValueError("channel mismatch")
    OH = (H + pad[0] + pad[1] - dil[0] * (KH - 1) - 1) // stride[0] + 1
    OW = (W + pad[2] + pad[3] - dil[1] * (KW - 1) - 1) // stride[1] + 1
    if OH < 1 or OW < 1:
        raise ValueError("empty output")
    out = np.empty((N, OH, OW, Cout), dtype=np.float64)
    pre = np.empty_like(out) if want_preact else None
    rc = lib().oracle_conv2d_nhwc_pad4(_ptr(x), _ptr(w), _ptr(bias), _ptr(out), _ptr(pre),
                                       N, H, W, Cin, Cout, KH, KW, stride[0], stride[1],
                                       pad[0], pad[1], pad[2], pad[3], dil[0], dil[1],
                                       dtype, float(alpha), epi)
    _rc(rc, "conv2d_nhwc_pad4")
    return (out, pre) if want_preact else out


def conv_transpose_out_dim(size, k, stride, pad, out_pad, dil) -> int:
    return int(lib().oracle_conv_transpose_out_dim(size, k, stride, pad, out_pad, dil))


def conv2d_transpose_nhwc(x, w, bias=None, *, dtype, stride=(1, 1), pad=(0, 0), out_pad=(0, 0),
                          dil=(1, 1), alpha=1.0, epi=EPI_NONE, want_preact=False):
    """Transposed convolution; x [N][H][W][Cin], w [KH][KW][Cin][Cout]; float64 [N][OH][OW][Cout]."""
    x = _check_in(np.ascontiguousarray(x), dtype)
    w = _check_in(np.ascontiguousarray(w), dtype)
    bias = _check_bias(bias)
    N, H, W, Cin = x.shape
    KH, KW, Cin2, Cout = w.shape
    if Cin2 != Cin:
        raise ValueError("channel mismatch")
    OH = conv_transpose_out_dim(H, KH, stride[0], pad[0], out_pad[0], dil[0])
    OW = conv_transpose_out_dim(W, KW, stride[1], pad[1], out_pad[1], dil[1])
    if OH < 1 or OW < 1:
        raise ValueError("empty or invalid output")
    out = np.empty((N, OH, OW, Cout), dtype=np.float64)
    pre = np.empty_like(out) if want_preact else None
    rc = lib().oracle_conv2d_transpose_nhwc(_ptr(x), _ptr(w), _ptr(bias), _ptr(out), _ptr(pre),
                                            N, H, W, Cin, Cout, KH, KW, stride[0], stride[1],
                                            pad[0], pad[1], out_pad[0], out_pad[1], dil[0], dil[1],
                                            dtype, float(alpha), epi)
    _rc(rc, "conv2d_transpose_nhwc")
    return (out, pre) if want_preact else out


def conv2d_transpose_nhwc_at(x, w, bias, sn, soh, sow, sco, *, dtype, stride=(1, 1), pad=(0, 0),
                             out_pad=(0, 0), dil=(1, 1), alpha=1.0, epi=EPI_NONE):
    """(out, preact) of the transposed convolution at listed output coordinates."""
    x = _check_in(np.ascontiguousarray(x), dtype)
    w = _check_in(np.ascontiguousarray(w), dtype)
    bias = _check_bias(bias)
    N, H, W, Cin = x.shape
    KH, KW, _, Cout = w.shape
    idx = [np.ascontiguousarray(a, dtype=np.int64) for a in (sn, soh, sow, sco)]
    out = np.empty(idx[0].size, dtype=np.float64)
    pre = np.empty_like(out)
    rc = lib().oracle_conv2d_transpose_nhwc_at(_ptr(x), _ptr(w), _ptr(bias), _ptr(out), _ptr(pre),
                                               N, H, W, Cin, Cout, KH, KW, stride[0], stride[1],
                                               pad[0], pad[1], out_pad[0], out_pad[1], dil[0], dil[1],
                                               dtype, float(alpha), epi, idx[0].size,
                                               *[_ptr(a) for a in idx])
    _rc(rc, "conv2d_transpose_nhwc_at")
    return out, pre


def matmul_residual(A, B, bias, R, *, dtype, r_dtype, trans_b=0, alpha=1.0, beta=1.0, epi=EPI_NONE,
                    want_preact=False):
    """act(alpha*A.B + bias + beta*R) as float64 [M][N]."""
    A = _check_in(np.ascontiguousarray(A), dtype); B = _check_in(np.ascontiguousarray(B), dtype)
    R = _check_in(np.ascontiguousarray(R), r_dtype); bias = _check_bias(bias)
    M, K = A.shape
    N = B.shape[0] if trans_b else B.shape[1]
    if R.shape != (M, N):
        raise ValueError("R must have the output's shape")
    out = np.empty((M, N), dtype=np.float64)
    pre = np.empty_like(out) if want_preact else None
    rc = lib().oracle_matmul_residual(_ptr(A), _ptr(B), _ptr(bias), _ptr(R), _ptr(out), _ptr(pre), M, N, K,
                                      K, B.shape[1], N, N, dtype, r_dtype, int(trans_b), float(alpha), float(beta), epi)
    _rc(rc, "matmul_residual")
    return (out, pre) if want_preact else out


def conv2d_nhwc_residual(x, w, bias, r, *, dtype, r_dtype, stride=(1, 1), pad=(0, 0), dil=(1, 1), alpha=1.0,
                         beta=1.0, epi=EPI_NONE, want_preact=False):
    x = _check_in(np.ascontiguousarray(x), dtype); w = _check_in(np.ascontiguousarray(w), dtype)
    r = _check_in(np.ascontiguousarray(r), r_dtype); bias = _check_bias(bias)
    N, H, W, Cin = x.shape
    KH, KW, _, Cout = w.shape
    OH = conv_out_dim(H, KH, stride[0], pad[0], dil[0]); OW = conv_out_dim(W, KW, stride[1], pad[1], dil[1])
    if r.shape != (N, OH, OW, Cout):
        raise ValueError("r must have the output's shape")
    out = np.empty((N, OH, OW, Cout), dtype=np.float64)
    pre = np.empty_like(out) if want_preact else None
    rc = lib().oracle_conv2d_nhwc_residual(_ptr(x), _ptr(w), _ptr(bias), _ptr(r), _ptr(out), _ptr(pre), N, H, W, Cin,
                                           Cout, KH, KW, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1],
                                           dtype, r_dtype, float(alpha), float(beta), epi)
    _rc(rc, "conv2d_nhwc_residual")
    return (out, pre) if want_preact else out


def _f32vec(v, n, name):
    if v is None:
        return None
    v = np.ascontiguousarray(v)
    if v.dtype != np.float32 or v.shape != (n,):
        raise TypeError(f"{name} must be float32 [{n}]")
    return v


def matmul_int8(A, B, *, scale, bias=None, mid_scale=0.0, mul=None, add=None, relu=False, out_scale=1.0,
                out_int8=True, trans_b=0, want_acc=False):
    """int8 matmul with the quantised epilogue; returns int8 (or float32) [M][N], and the int32 sums if asked."""
    A = np.ascontiguousarray(A); B = np.ascontiguousarray(B)
    if A.dtype != np.int8 or B.dtype != np.int8:
        raise TypeError("int8 operands expected")
    M, K = A.shape
    N = B.shape[0] if trans_b else B.shape[1]
    scale, bias, mul, add = (_f32vec(v, N, n) for v, n in ((scale, "scale"), (bias, "bias"), (mul, "mul"), (add, "add")))
    out = np.empty((M, N), dtype=np.int8 if out_int8 else np.float32)
    acc = np.empty((M, N), dtype=np.int32) if want_acc else None
    rc = lib().oracle_matmul_int8(_ptr(A), _ptr(B), _ptr(out), _ptr(acc), M, N, K, K, B.shape[1], N, int(trans_b),
                                  _ptr(scale), _ptr(bias), float(mid_scale), _ptr(mul), _ptr(add), int(relu),
                                  float(out_scale), int(out_int8))
    _rc(rc, "matmul_int8")
    return (out, acc) if want_acc else out


def matmul_int8_bn(A, B, *, scale, mean, var, eps, gamma, beta, bias=None, mid_scale=0.0, relu=False, out_scale=1.0,
                   out_int8=True, trans_b=0):
    """int8 matmul with the quantised epilogue whose batch-norm step is unfolded (mean, var, eps, gamma, beta)."""
    A = np.ascontiguousarray(A); B = np.ascontiguousarray(B)
    if A.dtype != np.int8 or B.dtype != np.int8:
        raise TypeError("int8 operands expected")
    M, K = A.shape
    N = B.shape[0] if trans_b else B.shape[1]
    scale, bias, mean, var, gamma, beta = (_f32vec(v, N, n) for v, n in (
        (scale, "scale"), (bias, "bias"), (mean, "mean"), (var, "var"), (gamma, "gamma"), (beta, "beta")))
    out = np.empty((M, N), dtype=np.int8 if out_int8 else np.float32)
    rc = lib().oracle_matmul_int8_bn(_ptr(A), _ptr(B), _ptr(out), None, M, N, K, K, B.shape[1], N, int(trans_b),
                                     _ptr(scale), _ptr(bias), float(mid_scale), _ptr(mean), _ptr(var), float(eps),
                                     _ptr(gamma), _ptr(beta), int(relu), float(out_scale), int(out_int8))
    _rc(rc, "matmul_int8_bn")
    return out


def conv2d_nhwc_int8_bn(x, w, *, scale, mean, var, eps, gamma, beta, bias=None, mid_scale=0.0, relu=False,
                        out_scale=1.0, out_int8=True, stride=(1, 1), pad=(0, 0), dil=(1, 1)):
    x = np.ascontiguousarray(x); w = np.ascontiguousarray(w)
    if x.dtype != np.int8 or w.dtype != np.int8:
        raise TypeError("int8 operands expected")
    N, H, W, Cin = x.shape
    KH, KW, _, Cout = w.shape
    OH = conv_out_dim(H, KH, stride[0], pad[0], dil[0]); OW = conv_out_dim(W, KW, stride[1], pad[1], dil[1])
    scale, bias, mean, var, gamma, beta = (_f32vec(v, Cout, n) for v, n in (
        (scale, "scale"), (bias, "bias"), (mean, "mean"), (var, "var"), (gamma, "gamma"), (beta, "beta")))
    out = np.empty((N, OH, OW, Cout), dtype=np.int8 if out_int8 else np.float32)
    rc = lib().oracle_conv2d_nhwc_int8_bn(_ptr(x), _ptr(w), _ptr(out), None, N, H, W, Cin, Cout, KH, KW,
                                          stride[0], stride[1], pad[0], pad[1], dil[0], dil[1],
                                          _ptr(scale), _ptr(bias), float(mid_scale), _ptr(mean), _ptr(var), float(eps),
                                          _ptr(gamma), _ptr(beta), int(relu), float(out_scale), int(out_int8))
    _rc(rc, "conv2d_nhwc_int8_bn")
    return out


def conv2d_nhwc_int8(x, w, *, scale, bias=None, mid_scale=0.0, mul=None, add=None, relu=False, out_scale=1.0,
                     out_int8=True, stride=(1, 1), pad=(0, 0), dil=(1, 1), want_acc=False):
    x = np.ascontiguousarray(x); w = np.ascontiguousarray(w)
    if x.dtype != np.int8 or w.dtype != np.int8:
        raise TypeError("int8 operands expected")
    N, H, W, Cin = x.shape
    KH, KW, _, Cout = w.shape
    OH = conv_out_dim(H, KH, stride[0], pad[0], dil[0]); OW = conv_out_dim(W, KW, stride[1], pad[1], dil[1])
    scale, bias, mul, add = (_f32vec(v, Cout, n) for v, n in ((scale, "scale"), (bias, "bias"), (mul, "mul"), (add, "add")))
    out = np.empty((N, OH, OW, Cout), dtype=np.int8 if out_int8 else np.float32)
    acc = np.empty((N, OH, OW, Cout), dtype=np.int32) if want_acc else None
    rc = lib().oracle_conv2d_nhwc_int8(_ptr(x), _ptr(w), _ptr(out), _ptr(acc), N, H, W, Cin, Cout, KH, KW,
                                       stride[0], stride[1], pad[0], pad[1], dil[0], dil[1],
                                       _ptr(scale), _ptr(bias), float(mid_scale), _ptr(mul), _ptr(add), int(relu),
                                       float(out_scale), int(out_int8))
    _rc(rc, "conv2d_nhwc_int8")
    return (out, acc) if want_acc else out


def _attention_args(Q, K, V, bias, dtype):
    Q = _check_in(np.ascontiguousarray(Q), dtype)
    K = _check_in(np.ascontiguousarray(K), dtype)
    V = _check_in(np.ascontiguousarray(V), dtype)
    if Q.ndim != 3 or K.ndim != 3 or V.shape != K.shape or Q.shape[0] != K.shape[0] or Q.shape[2] != K.shape[2]:
        raise ValueError("attention expects Q [batch][Nq][D], K and V [batch][Nk][D]")
    batch, Nq, D = Q.shape
    Nk = K.shape[1]
    ld_bias = stride_bias = 0
    if bias is not None:
        if bias.dtype != np.float32 or not bias.flags.c_contiguous:
            raise TypeError("attention bias must be contiguous float32")
        if bias.shape == (Nq, Nk):
            ld_bias, stride_bias = Nk, 0
        elif bias.shape == (batch, Nq, Nk):
            ld_bias, stride_bias = Nk, Nq * Nk
        else:
            raise ValueError("attention bias must be [Nq][Nk] or [batch][Nq][Nk]")
    return Q, K, V, batch, Nq, Nk, D, ld_bias, stride_bias


def attention(Q, K, V, bias=None, *, dtype, alpha=1.0):
    """softmax(alpha * Q K^T + bias) V as float64 [batch][Nq][D]."""
    Q, K, V, batch, Nq, Nk, D, ld_bias, stride_bias = _attention_args(Q, K, V, bias, dtype)
    out = np.empty((batch, Nq, D), dtype=np.float64)
    rc = lib().oracle_attention(_ptr(Q), _ptr(K), _ptr(V), _ptr(bias), _ptr(out),
                                batch, Nq, Nk, D, D, D, D, D, Nq * D, Nk * D, Nk * D, Nq * D,
                                ld_bias, stride_bias, dtype, float(alpha))
    _rc(rc, "attention")
    return out


def attention_rows(Q, K, V, bias, sb, si, *, dtype, alpha=1.0):
    """Rows (sb[s], si[s]) of the same result: float64 [nsamp][D]."""
    Q, K, V, batch, Nq, Nk, D, ld_bias, stride_bias = _attention_args(Q, K, V, bias, dtype)
    sb = np.ascontiguousarray(sb, dtype=np.int64)
    si = np.ascontiguousarray(si, dtype=np.int64)
    out = np.empty((sb.size, D), dtype=np.float64)
    rc = lib().oracle_attention_rows(_ptr(Q), _ptr(K), _ptr(V), _ptr(bias), _ptr(out),
                                     batch, Nq, Nk, D, D, D, D, Nq * D, Nk * D, Nk * D,
                                     ld_bias, stride_bias, dtype, float(alpha),
                                     sb.size, _ptr(sb), _ptr(si))
    _rc(rc, "attention_rows")
    return out


def attention_causal(Q, K, V, *, dtype, alpha=1.0):
    """Causal attention (row i sees keys j <= i + Nk - Nq) as float64 [batch][Nq][D]."""
    Q, K, V, batch, Nq, Nk, D, _, _ = _attention_args(Q, K, V, None, dtype)
    out = np.empty((batch, Nq, D), dtype=np.float64)
    rc = lib().oracle_attention_causal(_ptr(Q), _ptr(K), _ptr(V), _ptr(out),
                                       batch, Nq, Nk, D, D, D, D, D, Nq * D, Nk * D, Nk * D, Nq * D,
                                       dtype, float(alpha))
    _rc(rc, "attention_causal")
    return out


def attention_causal_rows(Q, K, V, sb, si, *, dtype, alpha=1.0):
    """Rows (sb[s], si[s]) of the causal result: float64 [nsamp][D]."""
    Q, K, V, batch, Nq, Nk, D, _, _ = _attention_args(Q, K, V, None, dtype)
    sb = np.ascontiguousarray(sb, dtype=np.int64)
    si = np.ascontiguousarray(si, dtype=np.int64)
    out = np.empty((sb.size, D), dtype=np.float64)
    rc = lib().oracle_attention_causal_rows(_ptr(Q), _ptr(K), _ptr(V), _ptr(out),
                                            batch, Nq, Nk, D, D, D, D, Nq * D, Nk * D, Nk * D,
                                            dtype, float(alpha), sb.size, _ptr(sb), _ptr(si))
    _rc(rc, "attention_causal_rows")
    return out


def epilogue(s, bias, alpha, epi) -> float:
    return float(lib().oracle_epilogue(float(s), float(bias), float(alpha), epi))


def gelu_tanh(t) -> float:
    return float(lib().oracle_gelu_tanh(float(t)))


def widen_bits(bits: int, dtype: int) -> float:
    return float(lib().oracle_widen(int(bits), dtype))


def round_bf16(v: float) -> int:
    return int(lib().oracle_round_bf16(float(v)))


def round_f16(v: float) -> int:
    return int(lib().oracle_round_f16(float(v)))


def num_threads() -> int:
    return int(lib().oracle_num_threads())
