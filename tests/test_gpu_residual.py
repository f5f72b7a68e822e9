"""Parity of the residual-add epilogue (through the C ABI) with the CPU oracle."""
import numpy as np
import pytest

import workloads as wl
from workloads import configs as C
import pbk_testlib as T

pytestmark = pytest.mark.gpu

BF16, F16, F32 = wl.DTYPE_BF16, wl.DTYPE_F16, wl.DTYPE_F32


def out_tensor(n, dtype):
    return T.device_empty(n, dtype)


@pytest.mark.parametrize("cfg", [None, 0, 1, 5, 6, 7, 9, "generic"])
@pytest.mark.parametrize("mnk", [(300, 264, 200), (256, 512, 64), (33, 520, 136), (130, 257, 72)])
@pytest.mark.parametrize("dtype,out_dtype", [(BF16, BF16), (F16, F32)])
def test_matmul_residual(cfg, mnk, dtype, out_dtype):
    import oracle
    import paper_2603_06731_amd as pbk
    m, n, k = mnk
    A = wl.tensor((m, k), dtype, 1, "normal", 1.0); B = wl.tensor((k, n), dtype, 2, "normal", 1.0 / np.sqrt(k))
    bias = wl.tensor((n,), F32, 3, "normal", 0.5); R = wl.tensor((m, n), out_dtype, 8, "normal", 1.0)
    out = out_tensor(m * n, out_dtype)
    force = None if cfg is None else ("generic" if cfg == "generic" else f"mfma:{cfg}")
    with T.forced_kernel(force):
        st = pbk.pbk_matmul_residual(T.to_device(A), T.to_device(B), out, T.to_device(bias), T.to_device(R), m, n, k,
                                     k, n, n, n, dtype, out_dtype, 0, 0.75, -0.5, C.EPI_BIAS_RELU, None)
    assert st == 0, pbk.pbk_status_string(st)
    ref, pre = oracle.matmul_residual(A, B, bias, R, dtype=dtype, r_dtype=out_dtype, alpha=0.75, beta=-0.5,
                                      epi=C.EPI_BIAS_RELU, want_preact=True)
    got = T.to_host_f64(out, out_dtype).reshape(ref.shape)
    err = T.rel_err(got, ref, pre)
    print(f"residual {mnk} force={force} kernel={pbk.pbk_last_kernel()} err={err:.3e}", flush=True)
    assert err <= T.TIGHT[out_dtype if dtype != F32 else F32], err
    # the residual really takes part: without it the result differs
    ref0 = oracle.matmul(A, B, bias, dtype=dtype, alpha=0.75, epi=C.EPI_BIAS_RELU)
    assert T.rel_err(got, ref0, pre) > 0.05


@pytest.mark.parametrize("cfg", [1, 5, 6])
@pytest.mark.parametrize("dtype,out_dtype", [(BF16, BF16), (F16, F32)])
@pytest.mark.parametrize("n,ldc,ldr", [(257, 257, 257), (264, 267, 269)])
def test_matmul_residual_direct_stores_on_mfma(cfg, dtype, out_dtype, n, ldc, ldr):
    """k-major B keeps a ragged N (or C / R rows that are not 16-byte multiples) on the matrix-unit
    kernel: the epilogue then reads the residual element by element and stores from registers."""
    import oracle
    import paper_2603_06731_amd as pbk
    m, k = 130, 72
    A = wl.tensor((m, k), dtype, 1, "normal", 1.0); B = wl.tensor((n, k), dtype, 2, "normal", 1.0 / np.sqrt(k))
    bias = wl.tensor((n,), F32, 3, "normal", 0.5); R = wl.tensor((m, ldr), out_dtype, 8, "normal", 1.0)
    out = out_tensor(m * ldc, out_dtype)
    with T.forced_kernel(f"mfma:{cfg}"):
        st = pbk.pbk_matmul_residual(T.to_device(A), T.to_device(B), out, T.to_device(bias), T.to_device(R), m, n, k,
                                     k, k, ldc, ldr, dtype, out_dtype, 1, 0.75, -0.5, C.EPI_BIAS_GELU_TANH, None)
    assert st == 0, pbk.pbk_status_string(st)
    assert "mfma" in pbk.pbk_last_kernel()
    ref, pre = oracle.matmul_residual(A, B, bias, np.ascontiguousarray(R[:, :n]), dtype=dtype, r_dtype=out_dtype,
                                      trans_b=1, alpha=0.75, beta=-0.5, epi=C.EPI_BIAS_GELU_TANH, want_preact=True)
    got = T.to_host_f64(out, out_dtype).reshape(m, ldc)[:, :n]
    err = T.rel_err(got, ref, pre)
    print(f"residual direct n={n} ldc={ldc} cfg={cfg} kernel={pbk.pbk_last_kernel()} err={err:.3e}", flush=True)
    assert err <= T.TIGHT[out_dtype], err


def test_matmul_residual_fp32_generic():
    import oracle
    import paper_2603_06731_amd as pbk
    m, n, k = 70, 45, 33
    A = wl.tensor((m, k), F32, 1, "uniform", 1.0); B = wl.tensor((n, k), F32, 2, "uniform", 1.0)
    R = wl.tensor((m, n), F32, 8, "uniform", 2.0)
    out = out_tensor(m * n, F32)
    st = pbk.pbk_matmul_residual(T.to_device(A), T.to_device(B), out, None, T.to_device(R), m, n, k, k, k, n, n,
                                 F32, F32, 1, 1.0, 1.0, C.EPI_GELU_TANH, None)
    assert st == 0
    ref, pre = oracle.matmul_residual(A, B, None, R, dtype=F32, r_dtype=F32, trans_b=1, epi=C.EPI_GELU_TANH, want_preact=True)
    err = T.rel_err(T.to_host_f64(out, F32).reshape(ref.shape), ref, pre)
    assert err <= T.TOL_F32, err


@pytest.mark.parametrize("cfg", [None, 0, 1, "generic"])
def test_conv_residual_block(cfg):
    """The second convolution of a residual block: relu(conv3x3(x) + bias + shortcut)."""
    import oracle
    import paper_2603_06731_amd as pbk
    n, H, W, Cc = 2, 14, 14, 64
    x = wl.tensor((n, H, W, Cc), BF16, 1, "normal", 1.0)
    w = wl.tensor((3, 3, Cc, Cc), BF16, 2, "normal", float(np.sqrt(2.0 / (9 * Cc))))
    bias = wl.tensor((Cc,), F32, 3, "normal", 0.1)
    r = wl.tensor((n, H, W, Cc), BF16, 8, "normal", 1.0)
    out = out_tensor(n * H * W * Cc, BF16)
    force = None if cfg is None else ("generic" if cfg == "generic" else f"mfma:{cfg}")
    with T.forced_kernel(force):
        st = pbk.pbk_conv2d_nhwc_residual(T.to_device(x), T.to_device(w), out, T.to_device(bias), T.to_device(r),
                                          n, H, W, Cc, Cc, 3, 3, 1, 1, 1, 1, 1, 1, BF16, BF16, 1.0, 1.0,
                                          C.EPI_BIAS_RELU, None)
    assert st == 0, pbk.pbk_status_string(st)
    ref, pre = oracle.conv2d_nhwc_residual(x, w, bias, r, dtype=BF16, r_dtype=BF16, pad=(1, 1), epi=C.EPI_BIAS_RELU,
                                           want_preact=True)
    err = T.rel_err(T.to_host_f64(out, BF16).reshape(ref.shape), ref, pre)
    print(f"conv residual force={force} kernel={pbk.pbk_last_kernel()} err={err:.3e}", flush=True)
    assert err <= T.TIGHT[BF16], err


def test_plain_calls_are_unaffected_after_a_residual_call():
    import oracle
    import paper_2603_06731_amd as pbk
    m, n, k = 128, 256, 64
    A = wl.tensor((m, k), BF16, 1, "normal", 1.0); B = wl.tensor((k, n), BF16, 2, "normal", 0.1)
    R = wl.tensor((m, n), BF16, 8, "normal", 5.0)
    dA, dB, dR = T.to_device(A), T.to_device(B), T.to_device(R)
    out = out_tensor(m * n, BF16)
    assert pbk.pbk_matmul_residual(dA, dB, out, None, dR, m, n, k, k, n, n, n, BF16, BF16, 0, 1.0, 1.0, 0, None) == 0
    assert pbk.pbk_matmul(dA, dB, out, None, m, n, k, k, n, n, BF16, BF16, 0, 1.0, 0, None) == 0
    ref, pre = oracle.matmul(A, B, dtype=BF16, want_preact=True)
    assert T.rel_err(T.to_host_f64(out, BF16).reshape(ref.shape), ref, pre) <= T.TIGHT[BF16]


def test_pointwise_conv_residual():
    """The last convolution of a bottleneck block, 1x1: relu(conv1x1(x) + bias + shortcut); the boundary hands it
    to the plain-matrix kernels with the residual operand in place."""
    import oracle
    import paper_2603_06731_amd as pbk
    n, H, W, Cin, Cout = 2, 12, 11, 64, 264
    x = wl.tensor((n, H, W, Cin), BF16, 1, "normal"); w = wl.tensor((1, 1, Cin, Cout), BF16, 2, "normal", 0.17)
    bias = wl.tensor((Cout,), F32, 3, "normal", 0.1); r = wl.tensor((n, H, W, Cout), BF16, 4, "normal")
    out = out_tensor(n * H * W * Cout, BF16)
    st = pbk.pbk_conv2d_nhwc_residual(T.to_device(x), T.to_device(w), out, T.to_device(bias), T.to_device(r),
                                      n, H, W, Cin, Cout, 1, 1, 1, 1, 0, 0, 1, 1, BF16, BF16, 1.0, 1.0, C.EPI_BIAS_RELU, None)
    assert st == 0, pbk.pbk_status_string(st)
    ref, pre = oracle.conv2d_nhwc_residual(x, w, bias, r, dtype=BF16, r_dtype=BF16, pad=(0, 0), epi=C.EPI_BIAS_RELU,
                                           want_preact=True)
    err = T.rel_err(T.to_host_f64(out, BF16).reshape(ref.shape), ref, pre)
    assert "mfma" in pbk.pbk_last_kernel() and err <= T.TIGHT[BF16], (pbk.pbk_last_kernel(), err)
