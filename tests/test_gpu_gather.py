"""Parity of the gathering matrix-unit kernel (operands that the direct-to-LDS kernel cannot take: ragged
K, N, leading dimensions, channel counts, unaligned bases) with the CPU oracle, element by element."""
import numpy as np
import pytest

import workloads as wl
from workloads import configs as C
import pbk_testlib as T

pytestmark = pytest.mark.gpu

BF16, F16, F32 = wl.DTYPE_BF16, wl.DTYPE_F16, wl.DTYPE_F32


def run_views(a, b, bias, M, N, K, lda, ldb, ldc, dtype, out_dtype, trans_b, epi, alpha=1.0, force=None, a_off=0, b_off=0):
    """pbk_matmul on views into larger host arrays (element offsets a_off / b_off shift the bases)."""
    import torch
    import oracle
    import paper_2603_06731_amd as pbk
    da = T.to_device(a.reshape(-1)); db = T.to_device(b.reshape(-1))
    esz = 2
    out = T.device_empty(M * ldc + 8, out_dtype, fill=0)
    with T.forced_kernel(force):
        st = pbk.pbk_matmul(da.data_ptr() + a_off * esz, db.data_ptr() + b_off * esz, out,
                            None if bias is None else T.to_device(bias), M, N, K, lda, ldb, ldc,
                            dtype, out_dtype, trans_b, alpha, epi)
    assert st == 0, pbk.pbk_status_string(st)
    torch.cuda.synchronize()
    kern = pbk.pbk_last_kernel()
    av = a.reshape(-1)[a_off:a_off + (M - 1) * lda + K]
    A2 = np.stack([av[i * lda:i * lda + K] for i in range(M)])
    rows_b = N if trans_b else K
    cols_b = K if trans_b else N
    bvw = b.reshape(-1)[b_off:b_off + (rows_b - 1) * ldb + cols_b]
    B2 = np.stack([bvw[i * ldb:i * ldb + cols_b] for i in range(rows_b)])
    ref, pre = oracle.matmul(A2, B2, bias, dtype=dtype, trans_b=trans_b, alpha=alpha, epi=epi, want_preact=True)
    got = T.to_host_f64(out, out_dtype)[:M * ldc].reshape(M, ldc)[:, :N]
    return T.rel_err(got, ref, pre), kern


@pytest.mark.parametrize("dtype,out_dtype", [(BF16, BF16), (F16, F32)])
@pytest.mark.parametrize("trans_b", [0, 1])
@pytest.mark.parametrize("mnk_ld", [
    (300, 261, 1143, 1146, None, None),      # K = 1143 (the paper's example), N = 261, lda = K + 3
    (264, 264, 200, 203, None, 267),         # aligned sizes, leading dimensions that break the 16-byte pieces
    (130, 129, 70, None, None, None),
    (64, 520, 33, None, None, None),
    (1, 4099, 17, None, None, None),
    (4100, 5, 40, None, None, None),         # rows of a row-major B shorter than one 16-byte piece
])
def test_matmul_unaligned_on_matrix_units(dtype, out_dtype, trans_b, mnk_ld):
    M, N, K, lda, ldb, ldc = mnk_ld
    lda = lda or K
    ldb = ldb or ((K if trans_b else N) + 1)
    ldc = ldc or N
    a = wl.tensor((M, lda), dtype, 1, "normal")
    b = wl.tensor(((N if trans_b else K), ldb), dtype, 2, "normal", 1.0 / np.sqrt(K))
    a[:, K:] = 0x7FC0 if dtype == BF16 else 0x7E00          # NaN outside the views
    b[:, (K if trans_b else N):] = 0x7FC0 if dtype == BF16 else 0x7E00
    bias = wl.tensor((N,), F32, 3, "normal", 0.5)
    err, kern = run_views(a, b, bias, M, N, K, lda, ldb, ldc, dtype, out_dtype, trans_b, C.EPI_BIAS_GELU_TANH, alpha=0.75)
    print(f"gather {mnk_ld} trans_b={trans_b} kernel={kern} err={err:.3e}", flush=True)
    assert "gather" in kern
    assert err <= T.TIGHT[out_dtype], err


@pytest.mark.parametrize("a_off,b_off", [(1, 0), (0, 3), (5, 7)])
def test_matmul_unaligned_bases(a_off, b_off):
    """Aligned sizes whose base pointers are not 16-byte aligned (views that start inside a buffer)."""
    M, N, K = 200, 264, 136
    a = wl.tensor((M * K + 16,), BF16, 1, "normal")
    b = wl.tensor((K * N + 16,), BF16, 2, "normal", 1.0 / np.sqrt(K))
    err, kern = run_views(a, b, None, M, N, K, K, N, N, BF16, BF16, 0, C.EPI_RELU, a_off=a_off, b_off=b_off)
    assert "gather" in kern and err <= T.TIGHT[BF16], (kern, err)


def test_forced_matrix_unit_choice_takes_the_gather_kernel_for_unaligned_operands():
    a = wl.tensor((136, 75), BF16, 1, "normal"); b = wl.tensor((75, 131), BF16, 2, "normal", 0.1)
    for force in ("mfma", "mfma:6", "gather"):
        err, kern = run_views(a, b, None, 136, 131, 75, 75, 131, 131, BF16, BF16, 0, C.EPI_NONE, force=force)
        assert "gather" in kern and err <= T.TIGHT[BF16], (force, kern, err)
    err, kern = run_views(a, b, None, 136, 131, 75, 75, 131, 131, BF16, BF16, 0, C.EPI_NONE, force="generic")
    assert "generic" in kern and err <= T.TIGHT[BF16]


@pytest.mark.parametrize("trans_b", [0, 1])
@pytest.mark.parametrize("mnk", [(520, 9, 8), (131, 140, 9), (70, 3, 15), (9, 8, 1)])
def test_forced_gather_kernel_on_tiny_k_and_n(mnk, trans_b):
    """Sizes below the ones the dispatcher gives to this kernel: K of one piece or less, operands of a few
    elements (every load is then moved back inside its operand and the piece shifted)."""
    M, N, K = mnk
    lda, ldb = K, (K if trans_b else N)
    a = wl.tensor((M, lda), BF16, 1, "normal"); b = wl.tensor(((N if trans_b else K), ldb), BF16, 2, "normal", 0.3)
    err, kern = run_views(a, b, None, M, N, K, lda, ldb, N, BF16, F32, trans_b, C.EPI_NONE, force="gather")
    assert "gather" in kern and err <= T.TIGHT[F32], (kern, err)


def test_forced_gather_kernel_declines_operands_smaller_than_a_piece():
    import paper_2603_06731_amd as pbk
    a = T.to_device(wl.tensor((4, 1), BF16, 1, "normal")); b = T.to_device(wl.tensor((1, 4), BF16, 2, "normal"))
    out = T.device_empty(16, F32, fill=0)
    with T.forced_kernel("gather"):
        st = pbk.pbk_matmul(a, b, out, None, 4, 4, 1, 1, 4, 4, BF16, F32, 0, 1.0, C.EPI_NONE)
    assert st != 0 and "not supported" in pbk.pbk_status_string(st), pbk.pbk_status_string(st)
    st = pbk.pbk_matmul(a, b, out, None, 4, 4, 1, 1, 4, 4, BF16, F32, 0, 1.0, C.EPI_NONE)
    assert st == 0 and "generic" in pbk.pbk_last_kernel()


def check_workload(w, expect):
    import paper_2603_06731_amd as pbk
    host = wl.make_inputs(w)
    st, out = T.run_workload(w, T.upload(host))
    assert st == 0, pbk.pbk_status_string(st)
    kern = pbk.pbk_last_kernel()
    ref, pre = T.oracle_full(w, host)
    err = T.rel_err(T.to_host_f64(out, w.out_dtype).reshape(ref.shape), ref, pre)
    print(f"{w.name} kernel={kern} err={err:.3e}", flush=True)
    assert expect in kern, kern
    assert err <= T.TIGHT[w.out_dtype if w.in_dtype != F32 else F32], err


@pytest.mark.parametrize("case", [
    # n, H, W, Cin, Cout, KH, KW, stride, pad, dil
    (2, 44, 44, 127, 24, 3, 3, (2, 2), (0, 0), (1, 1)),      # the paper's first worked example, fewer images / outputs
    (1, 20, 19, 127, 136, 3, 3, (1, 1), (1, 1), (1, 1)),
    (2, 15, 17, 9, 40, 5, 3, (1, 2), (2, 1), (2, 1)),        # 9 channels: a tap is two pieces, one nearly empty
    (1, 30, 30, 3, 64, 7, 7, (2, 2), (3, 3), (1, 1)),        # 3 channels (an RGB stem): fewer than one piece
    (2, 10, 10, 5, 33, 3, 3, (1, 1), (1, 1), (1, 1)),
    (1, 12, 13, 20, 40, 3, 3, (1, 1), (1, 1), (1, 1)),       # 24 padded channels: a k-tile spans a tap and a third
    (1, 12, 12, 30, 261, 1, 1, (1, 1), (0, 0), (1, 1)),
    (6, 9, 11, 8, 12, 2, 2, (1, 1), (0, 1), (1, 1)),         # aligned channels, ragged Cout
])
@pytest.mark.parametrize("dtype,out_dtype", [(F16, F32), (BF16, BF16)])
def test_conv_unaligned_channels_on_matrix_units(case, dtype, out_dtype):
    n, H, W, Cin, Cout, KH, KW, stride, pad, dil = case
    w = wl.Workload("conv_gather", "conv", dtype, out_dtype, C.EPI_BIAS_RELU, n=n, H=H, W=W, Cin=Cin, Cout=Cout,
                    KH=KH, KW=KW, stride=stride, pad=pad, dil=dil,
                    dist_b=("normal", float(np.sqrt(2.0 / (KH * KW * Cin)))))
    check_workload(w, "gather")


def test_batched_unaligned_on_matrix_units():
    w = wl.Workload("bmm_gather", "batched", BF16, F32, C.EPI_NONE, alpha=0.5, batch=3, M=131, N=77, K=61,
                    dist_b=("normal", 0.1))
    check_workload(w, "gather")


def test_paper_example_full_size_against_an_aligned_twin():
    """The paper's first worked example in full (8 x 44 x 44 x 127 -> 512, 3 x 3, stride 2: M = 3528, K = 1143)
    on the matrix units, sampled against the oracle, and timed beside its 128-channel twin."""
    import torch
    import paper_2603_06731_amd as pbk
    times = {}
    for cin in (127, 128):
        w = wl.Workload(f"paper_conv_{cin}", "conv", F16, F32, C.EPI_NONE, n=8, H=44, W=44, Cin=cin, Cout=512,
                        KH=3, KW=3, stride=(2, 2), dist_b=("normal", 0.03))
        host = wl.make_inputs(w)
        dev = T.upload(host)
        st, out = T.run_workload(w, dev)
        assert st == 0
        kern = pbk.pbk_last_kernel()
        b, i, j = T.sample_coords(w, 1500)
        ref, pre = T.oracle_sampled(w, host, b, i, j)
        err = T.rel_err(T.gather_output(out, w, b, i, j), ref, pre)
        assert err <= T.TIGHT[F32], (cin, err)
        assert ("gather" in kern) == (cin == 127), kern
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        for _ in range(3):
            T.run_workload(w, dev, out=out)
        e0.record()
        for _ in range(20):
            T.run_workload(w, dev, out=out)
        e1.record(); torch.cuda.synchronize()
        times[cin] = e0.elapsed_time(e1) / 20 * 1e3
        print(f"paper conv Cin={cin}: kernel={kern} {times[cin]:.1f} us err={err:.2e}", flush=True)
    assert times[127] <= 2.0 * times[128], times


def test_matmul_k1143_beside_aligned_twin_and_generic_kernel():
    """3528 x 512 x 1143 (the matmul form of the paper's example, lda = K) on the gathering kernel, beside
    K = 1152 on the direct-to-LDS kernel and the generic kernel, both B layouts: timing table and the 2x bar."""
    import torch
    import paper_2603_06731_amd as pbk
    M, N = 3528, 512

    def timed(K, trans_b, force):
        a = T.to_device(wl.tensor((M, K), BF16, 1, "normal"))
        b = T.to_device(wl.tensor(((N, K) if trans_b else (K, N)), BF16, 2, "normal", 1.0 / np.sqrt(K)))
        out = T.device_empty(M * N, BF16)
        with T.forced_kernel(force):
            def call():
                return pbk.pbk_matmul(a, b, out, None, M, N, K, K, (K if trans_b else N), N, BF16, BF16, trans_b, 1.0,
                                      C.EPI_NONE)
            assert call() == 0
            kern = pbk.pbk_last_kernel()
            torch.cuda.synchronize()
            e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
            for _ in range(3):
                call()
            e0.record()
            for _ in range(20):
                call()
            e1.record(); torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / 20 * 1e3
        print(f"{M}x{N}x{K} trans_b={trans_b} {kern}: {us:.1f} us", flush=True)
        return us, kern
    for trans_b in (0, 1):
        g, kg = timed(1143, trans_b, None)
        al, ka = timed(1152, trans_b, None)
        timed(1152, trans_b, "gather")
        gen, _ = timed(1143, trans_b, "generic")
        assert "gather" in kg and "gather" not in ka and "mfma" in ka
        assert g <= 2.0 * al and g < gen, (g, al, gen)
