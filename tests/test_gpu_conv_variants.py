"""Parity of the convolution variants (four-sided padding, transposed
convolution) with the CPU oracle, through the C ABI."""
import numpy as np
import pytest

import workloads as wl
from workloads import configs as C
import pbk_testlib as T

pytestmark = pytest.mark.gpu

BF16, F16, F32 = wl.DTYPE_BF16, wl.DTYPE_F16, wl.DTYPE_F32


def check(w, force=None, expect_kernel=None):
    import paper_2603_06731_amd as pbk
    host = wl.make_inputs(w)
    dev = T.upload(host)
    with T.forced_kernel(force):
        st, out = T.run_workload(w, dev)
    assert st == 0, pbk.pbk_status_string(st)
    if expect_kernel:
        assert expect_kernel in pbk.pbk_last_kernel(), pbk.pbk_last_kernel()
    ref, pre = T.oracle_full(w, host)
    got = T.to_host_f64(out, w.out_dtype).reshape(ref.shape)
    err = T.rel_err(got, ref, pre)
    print(f"{w.name} force={force} kernel={pbk.pbk_last_kernel()} out={ref.shape} err={err:.3e}", flush=True)
    tol = T.TOL_F32 if w.in_dtype == F32 else T.TOL_16BIT
    tight = T.TOL_F32 if w.in_dtype == F32 else T.TIGHT[w.out_dtype]
    assert err <= tol and err <= tight, (w.name, force, err)


def he(kh, kw, cin):
    return float(np.sqrt(2.0 / (kh * kw * cin)))


# ---------------------------------------------------------- four-sided padding

PAD4 = [  # n, H, W, Cin, Cout, KH, KW, stride, pad4, dil
    (2, 16, 16, 32, 64, 3, 3, (2, 2), (0, 1, 0, 1), (1, 1)),      # "same" for an even image at stride 2
    (1, 15, 20, 64, 40, 3, 3, (1, 1), (2, 0, 1, 3), (1, 1)),
    (2, 14, 14, 40, 72, 5, 2, (2, 1), (1, 3, 0, 1), (1, 2)),
]


@pytest.mark.parametrize("case", PAD4)
@pytest.mark.parametrize("cfg", [None, 0, 1, 5, 6, 7, "generic"])
def test_conv_pad4(case, cfg):
    n, H, W, Cin, Cout, KH, KW, stride, pad4, dil = case
    w = wl.Workload("conv_pad4", "conv", BF16, BF16, C.EPI_BIAS_RELU, n=n, H=H, W=W, Cin=Cin, Cout=Cout,
                    KH=KH, KW=KW, stride=stride, pad4=pad4, dil=dil, dist_b=("normal", he(KH, KW, Cin)))
    force = None if cfg is None else ("generic" if cfg == "generic" else f"mfma:{cfg}")
    check(w, force=force, expect_kernel="generic" if cfg == "generic" else "mfma")


def test_conv_pad4_fp32_tiny_channels():
    w = wl.Workload("conv_pad4_f32", "conv", F32, F32, C.EPI_BIAS, n=1, H=20, W=18, Cin=3, Cout=5,
                    KH=3, KW=3, stride=(2, 2), pad4=(0, 1, 1, 0), dist_b=("normal", 0.3))
    check(w, expect_kernel="generic")


# ------------------------------------------------------ transposed convolution

CONVT = [  # n, H, W, Cin, Cout, KH, KW, stride, pad, out_pad, dil
    (2, 12, 12, 32, 64, 3, 3, (1, 1), (1, 1), (0, 0), (1, 1)),
    (2, 12, 10, 64, 32, 3, 3, (2, 2), (1, 1), (1, 1), (1, 1)),     # the usual 2x upsampling layer
    (1, 9, 11, 40, 72, 4, 4, (2, 2), (1, 1), (0, 0), (1, 1)),
    (2, 7, 8, 32, 40, 2, 3, (3, 2), (0, 1), (2, 0), (1, 1)),
    (1, 10, 9, 64, 64, 3, 2, (2, 1), (2, 0), (0, 0), (2, 3)),
    (3, 6, 6, 256, 128, 2, 2, (2, 2), (0, 0), (0, 0), (1, 1)),      # Cin a multiple of the k-tile: one tap per k-tile
]


@pytest.mark.parametrize("case", CONVT)
@pytest.mark.parametrize("cfg", [None, 0, 1, "generic"])
def test_conv_transpose(case, cfg):
    n, H, W, Cin, Cout, KH, KW, stride, pad, out_pad, dil = case
    w = wl.Workload("convT", "conv", BF16, BF16, C.EPI_BIAS_RELU, n=n, H=H, W=W, Cin=Cin, Cout=Cout,
                    KH=KH, KW=KW, stride=stride, pad=pad, out_pad=out_pad, dil=dil, transposed=1,
                    dist_b=("normal", he(KH, KW, Cin)))
    force = None if cfg is None else ("generic" if cfg == "generic" else f"mfma:{cfg}")
    check(w, force=force, expect_kernel="generic" if cfg == "generic" else "mfma")


@pytest.mark.parametrize("dtype,out_dtype", [(F16, F32), (F32, F32), (F16, F16)])
def test_conv_transpose_dtypes(dtype, out_dtype):
    w = wl.Workload("convT_dt", "conv", dtype, out_dtype, C.EPI_BIAS_GELU_TANH, alpha=0.5, n=2, H=8, W=9,
                    Cin=24, Cout=16, KH=3, KW=3, stride=(2, 2), pad=(1, 1), out_pad=(1, 0), transposed=1,
                    dist_b=("normal", he(3, 3, 24)))
    check(w, expect_kernel="generic" if dtype == F32 else "mfma")


def test_conv_transpose_tiny_channels_generic():
    w = wl.Workload("convT_c3", "conv", BF16, BF16, C.EPI_NONE, n=1, H=11, W=7, Cin=3, Cout=3,
                    KH=5, KW=5, stride=(2, 2), pad=(2, 2), out_pad=(1, 1), transposed=1, dist_b=("normal", 0.2))
    check(w, expect_kernel="generic")


def test_conv_transpose_large_sampled():
    """A decoder-sized layer (32 x 28 x 28 x 256 -> 56 x 56 x 128, 4x4 stride 2) in the default
    configuration, checked on sampled outputs."""
    import paper_2603_06731_amd as pbk
    w = wl.Workload("convT_big", "conv", BF16, BF16, C.EPI_BIAS_RELU, n=32, H=28, W=28, Cin=256, Cout=128,
                    KH=4, KW=4, stride=(2, 2), pad=(1, 1), transposed=1, dist_b=("normal", he(2, 2, 256)))
    host = wl.make_inputs(w)
    dev = T.upload(host)
    st, out = T.run_workload(w, dev)
    assert st == 0, pbk.pbk_status_string(st)
    kern = pbk.pbk_last_kernel()
    b, i, j = T.sample_coords(w, 2000)
    ref, pre = T.oracle_sampled(w, host, b, i, j)
    got = T.gather_output(out, w, b, i, j)
    err = T.rel_err(got, ref, pre)
    print(f"convT_big kernel={kern} samples={len(i)} err={err:.3e}", flush=True)
    assert "mfma" in kern and err <= T.TIGHT[BF16], err


# ------------------------------------------------------ pointwise convolutions

@pytest.mark.parametrize("dtype,out_dtype", [(BF16, BF16), (F16, F32), (F32, F32)])
@pytest.mark.parametrize("case", [  # n, H, W, Cin, Cout
    (3, 20, 17, 64, 264),
    (2, 9, 9, 136, 40),
    (1, 30, 30, 24, 8),
])
def test_pointwise_conv_runs_as_the_plain_matmul(case, dtype, out_dtype):
    """A 1x1 filter at stride 1 without padding is the matmul [N H W][Cin] x [Cin][Cout]: the call takes the
    plain-matrix kernels (the B-stationary one, which declines every convolution, accepts it) and matches the
    convolution oracle."""
    n, H, W, Cin, Cout = case
    w = wl.Workload("conv_1x1", "conv", dtype, out_dtype, C.EPI_BIAS_RELU, n=n, H=H, W=W, Cin=Cin, Cout=Cout,
                    KH=1, KW=1, stride=(1, 1), pad=(0, 0), dist_b=("normal", he(1, 1, Cin)))
    check(w)
    if dtype != F32 and Cin <= 128:
        check(w, force="bstat", expect_kernel="bstat")


def test_strided_or_padded_1x1_conv_stays_a_convolution():
    import paper_2603_06731_amd as pbk
    for stride, pad in (((2, 2), (0, 0)), ((1, 1), (1, 1))):
        w = wl.Workload("conv_1x1_s", "conv", BF16, BF16, C.EPI_BIAS, n=2, H=12, W=12, Cin=64, Cout=64,
                        KH=1, KW=1, stride=stride, pad=pad, dist_b=("normal", he(1, 1, 64)))
        check(w)
        host = wl.make_inputs(w)
        with T.forced_kernel("bstat"):
            st, _ = T.run_workload(w, T.upload(host))
        assert st != 0 and "not supported" in pbk.pbk_status_string(st)
