"""ctypes binding of libpbk.so (see include/pbk.h for the contract).

Pointers may be given as Python ints (device addresses) or as objects with a
`data_ptr()` method (torch tensors); `stream` as an int / None, or an object
with a `cuda_stream` attribute (torch.cuda.Stream).
"""
from __future__ import annotations

import ctypes
import os

PBK_OK = 0
PBK_F32, PBK_BF16, PBK_F16, PBK_FP8_E4M3, PBK_FP8_E5M2, PBK_INT8 = 0, 1, 2, 3, 4, 5
(PBK_EPI_NONE, PBK_EPI_BIAS, PBK_EPI_RELU, PBK_EPI_BIAS_RELU,
 PBK_EPI_BIAS_GELU_TANH, PBK_EPI_GELU_TANH) = range(6)

EXPORTED_SYMBOLS = ("pbk_matmul", "pbk_batched_matmul", "pbk_conv2d_nhwc", "pbk_conv2d_nhwc_pad4",
                    "pbk_conv2d_transpose_nhwc", "pbk_attention", "pbk_attention_causal", "pbk_matmul_int8", "pbk_conv2d_nhwc_int8",
                    "pbk_matmul_residual", "pbk_conv2d_nhwc_residual", "pbk_matmul_int8_bn", "pbk_conv2d_nhwc_int8_bn",
                    "pbk_status_string", "pbk_version", "pbk_last_kernel", "pbk_force_kernel")

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpbk.so")
_lib = None


class PbkError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {pbk_status_string(status)} (status {status})")


def lib_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """The loaded library.  Raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it first "
                              "(python -m paper_2603_06731_amd.build, or __graft_entry__.build())")
        # One process must hold ONE HIP runtime: a second copy cannot open the
        # device ("no ROCm-capable device").  torch ships its own libamdhip64, and
        # callers hand this library torch's device pointers and streams, so torch's
        # copy is loaded first and libpbk binds to it by soname.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(_LIB_PATH)
        i64, vp, f32, i32 = ctypes.c_int64, ctypes.c_void_p, ctypes.c_float, ctypes.c_int
        L.pbk_matmul.argtypes = [vp, vp, vp, vp] + [i64] * 6 + [i32, i32, i32, f32, i32, vp]
        L.pbk_matmul.restype = i32
        L.pbk_batched_matmul.argtypes = [vp, vp, vp, vp] + [i64] * 10 + [i32, i32, i32, f32, i32, vp]
        L.pbk_batched_matmul.restype = i32
        L.pbk_conv2d_nhwc.argtypes = [vp, vp, vp, vp] + [i64] * 13 + [i32, i32, f32, i32, vp]
        L.pbk_conv2d_nhwc.restype = i32
        L.pbk_conv2d_nhwc_pad4.argtypes = [vp, vp, vp, vp] + [i64] * 15 + [i32, i32, f32, i32, vp]
        L.pbk_conv2d_nhwc_pad4.restype = i32
        L.pbk_conv2d_transpose_nhwc.argtypes = [vp, vp, vp, vp] + [i64] * 15 + [i32, i32, f32, i32, vp]
        L.pbk_conv2d_transpose_nhwc.restype = i32
        L.pbk_matmul_int8.argtypes = [vp, vp, vp] + [i64] * 6 + [i32, vp, vp, f32, vp, vp, i32, f32, i32, vp]
        L.pbk_matmul_int8.restype = i32
        L.pbk_conv2d_nhwc_int8.argtypes = [vp, vp, vp] + [i64] * 13 + [vp, vp, f32, vp, vp, i32, f32, i32, vp]
        L.pbk_conv2d_nhwc_int8.restype = i32
        L.pbk_matmul_int8_bn.argtypes = [vp, vp, vp] + [i64] * 6 + [i32, vp, vp, f32, vp, vp, f32, vp, vp, i32, f32, i32, vp]
        L.pbk_matmul_int8_bn.restype = i32
        L.pbk_conv2d_nhwc_int8_bn.argtypes = [vp, vp, vp] + [i64] * 13 + [vp, vp, f32, vp, vp, f32, vp, vp, i32, f32, i32, vp]
        L.pbk_conv2d_nhwc_int8_bn.restype = i32
        L.pbk_matmul_residual.argtypes = [vp, vp, vp, vp, vp] + [i64] * 7 + [i32, i32, i32, f32, f32, i32, vp]
        L.pbk_matmul_residual.restype = i32
        L.pbk_conv2d_nhwc_residual.argtypes = [vp, vp, vp, vp, vp] + [i64] * 13 + [i32, i32, f32, f32, i32, vp]
        L.pbk_conv2d_nhwc_residual.restype = i32
        L.pbk_attention.argtypes = [vp, vp, vp, vp, vp] + [i64] * 14 + [i32, f32, vp]
        L.pbk_attention.restype = i32
        L.pbk_attention_causal.argtypes = [vp, vp, vp, vp] + [i64] * 12 + [i32, f32, vp]
        L.pbk_attention_causal.restype = i32
        L.pbk_status_string.argtypes = [i32]
        L.pbk_status_string.restype = ctypes.c_char_p
        L.pbk_version.restype = i32
        L.pbk_last_kernel.restype = ctypes.c_char_p
        L.pbk_force_kernel.argtypes = [ctypes.c_char_p]
        L.pbk_force_kernel.restype = i32
        _lib = L
    return _lib


def _ptr(x):
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


def _stream(s):
    if s is None:
        return None
    if hasattr(s, "cuda_stream"):
        return s.cuda_stream
    return int(s)


def pbk_matmul(A, B, C, bias, M, N, K, lda, ldb, ldc, in_dtype, out_dtype, trans_b,
               alpha, epi, stream=None) -> int:
    return lib().pbk_matmul(_ptr(A), _ptr(B), _ptr(C), _ptr(bias), M, N, K, lda, ldb, ldc,
                            in_dtype, out_dtype, int(trans_b), float(alpha), epi, _stream(stream))


def pbk_batched_matmul(A, B, C, bias, batch, M, N, K, lda, ldb, ldc,
                       stride_a, stride_b, stride_c, in_dtype, out_dtype, trans_b,
                       alpha, epi, stream=None) -> int:
    return lib().pbk_batched_matmul(_ptr(A), _ptr(B), _ptr(C), _ptr(bias), batch, M, N, K,
                                    lda, ldb, ldc, stride_a, stride_b, stride_c,
                                    in_dtype, out_dtype, int(trans_b), float(alpha), epi,
                                    _stream(stream))


def pbk_conv2d_nhwc(x, w, y, bias, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w,
                    pad_h, pad_w, dil_h, dil_w, in_dtype, out_dtype, alpha, epi,
                    stream=None) -> int:
    return lib().pbk_conv2d_nhwc(_ptr(x), _ptr(w), _ptr(y), _ptr(bias), N, H, W, Cin, Cout,
                                 KH, KW, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w,
                                 in_dtype, out_dtype, float(alpha), epi, _stream(stream))


def pbk_conv2d_nhwc_pad4(x, w, y, bias, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w,
                         pad_top, pad_bottom, pad_left, pad_right, dil_h, dil_w,
                         in_dtype, out_dtype, alpha, epi, stream=None) -> int:
    return lib().pbk_conv2d_nhwc_pad4(_ptr(x), _ptr(w), _ptr(y), _ptr(bias), N, H, W, Cin, Cout,
                                      KH, KW, stride_h, stride_w, pad_top, pad_bottom, pad_left, pad_right,
                                      dil_h, dil_w, in_dtype, out_dtype, float(alpha), epi, _stream(stream))


def pbk_conv2d_transpose_nhwc(x, w, y, bias, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w,
                              pad_h, pad_w, out_pad_h, out_pad_w, dil_h, dil_w,
                              in_dtype, out_dtype, alpha, epi, stream=None) -> int:
    return lib().pbk_conv2d_transpose_nhwc(_ptr(x), _ptr(w), _ptr(y), _ptr(bias), N, H, W, Cin, Cout,
                                           KH, KW, stride_h, stride_w, pad_h, pad_w, out_pad_h, out_pad_w,
                                           dil_h, dil_w, in_dtype, out_dtype, float(alpha), epi, _stream(stream))


def pbk_matmul_int8(A, B, C, M, N, K, lda, ldb, ldc, trans_b, scale, bias, mid_scale, mul, add, relu,
                    out_scale, out_dtype, stream=None) -> int:
    return lib().pbk_matmul_int8(_ptr(A), _ptr(B), _ptr(C), M, N, K, lda, ldb, ldc, int(trans_b), _ptr(scale),
                                 _ptr(bias), float(mid_scale), _ptr(mul), _ptr(add), int(relu), float(out_scale),
                                 out_dtype, _stream(stream))


def pbk_conv2d_nhwc_int8(x, w, y, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w,
                         scale, bias, mid_scale, mul, add, relu, out_scale, out_dtype, stream=None) -> int:
    return lib().pbk_conv2d_nhwc_int8(_ptr(x), _ptr(w), _ptr(y), N, H, W, Cin, Cout, KH, KW, stride_h, stride_w,
                                      pad_h, pad_w, dil_h, dil_w, _ptr(scale), _ptr(bias), float(mid_scale),
                                      _ptr(mul), _ptr(add), int(relu), float(out_scale), out_dtype, _stream(stream))


def pbk_matmul_int8_bn(A, B, C, M, N, K, lda, ldb, ldc, trans_b, scale, bias, mid_scale, mean, var, eps, gamma, beta, relu,
                       out_scale, out_dtype, stream=None) -> int:
    return lib().pbk_matmul_int8_bn(_ptr(A), _ptr(B), _ptr(C), M, N, K, lda, ldb, ldc, int(trans_b), _ptr(scale),
                                    _ptr(bias), float(mid_scale), _ptr(mean), _ptr(var), float(eps), _ptr(gamma), _ptr(beta),
                                    int(relu), float(out_scale), out_dtype, _stream(stream))


def pbk_conv2d_nhwc_int8_bn(x, w, y, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w,
                            scale, bias, mid_scale, mean, var, eps, gamma, beta, relu, out_scale, out_dtype, stream=None) -> int:
    return lib().pbk_conv2d_nhwc_int8_bn(_ptr(x), _ptr(w), _ptr(y), N, H, W, Cin, Cout, KH, KW, stride_h, stride_w,
                                         pad_h, pad_w, dil_h, dil_w, _ptr(scale), _ptr(bias), float(mid_scale),
                                         _ptr(mean), _ptr(var), float(eps), _ptr(gamma), _ptr(beta), int(relu),
                                         float(out_scale), out_dtype, _stream(stream))


def pbk_matmul_residual(A, B, C, bias, R, M, N, K, lda, ldb, ldc, ldr, in_dtype, out_dtype, trans_b,
                        alpha, beta, epi, stream=None) -> int:
    return lib().pbk_matmul_residual(_ptr(A), _ptr(B), _ptr(C), _ptr(bias), _ptr(R), M, N, K, lda, ldb, ldc, ldr,
                                     in_dtype, out_dtype, int(trans_b), float(alpha), float(beta), epi, _stream(stream))


def pbk_conv2d_nhwc_residual(x, w, y, bias, r, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w,
                             pad_h, pad_w, dil_h, dil_w, in_dtype, out_dtype, alpha, beta, epi, stream=None) -> int:
    return lib().pbk_conv2d_nhwc_residual(_ptr(x), _ptr(w), _ptr(y), _ptr(bias), _ptr(r), N, H, W, Cin, Cout,
                                          KH, KW, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w,
                                          in_dtype, out_dtype, float(alpha), float(beta), epi, _stream(stream))


def pbk_attention(Q, K, V, bias, O, batch, Nq, Nk, D, ldq, ldk, ldv, ldo,
                  stride_q, stride_k, stride_v, stride_o, ld_bias, stride_bias,
                  dtype, alpha, stream=None) -> int:
    return lib().pbk_attention(_ptr(Q), _ptr(K), _ptr(V), _ptr(bias), _ptr(O), batch, Nq, Nk, D,
                               ldq, ldk, ldv, ldo, stride_q, stride_k, stride_v, stride_o,
                               ld_bias, stride_bias, dtype, float(alpha), _stream(stream))


def pbk_attention_causal(Q, K, V, O, batch, Nq, Nk, D, ldq, ldk, ldv, ldo,
                         stride_q, stride_k, stride_v, stride_o, dtype, alpha, stream=None) -> int:
    return lib().pbk_attention_causal(_ptr(Q), _ptr(K), _ptr(V), _ptr(O), batch, Nq, Nk, D,
                                      ldq, ldk, ldv, ldo, stride_q, stride_k, stride_v, stride_o,
                                      dtype, float(alpha), _stream(stream))


def pbk_status_string(status: int) -> str:
    return lib().pbk_status_string(int(status)).decode()


def pbk_version() -> int:
    return int(lib().pbk_version())


def pbk_last_kernel() -> str:
    return lib().pbk_last_kernel().decode()


def pbk_force_kernel(choice) -> int:
    return lib().pbk_force_kernel(None if choice is None else str(choice).encode())


def check(status: int, where: str = "libpbk") -> None:
    if status != PBK_OK:
        raise PbkError(status, where)
