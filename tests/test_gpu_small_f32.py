"""Parity of the one-wave-per-tile fp32 kernel (small fp32 matmuls such as the 256^3 configuration) with
the CPU oracle, element by element, and its place in the dispatcher."""
import numpy as np
import pytest

import workloads as wl
from workloads import configs as C
import pbk_testlib as T

pytestmark = pytest.mark.gpu

F32 = wl.DTYPE_F32


def run(M, N, K, trans_b, epi, *, lda=None, ldb=None, ldc=None, alpha=1.0, force=None, residual=False, batch=1):
    import oracle
    import paper_2603_06731_amd as pbk
    lda = lda or K; ldb = ldb or (K if trans_b else N); ldc = ldc or N
    rows_b, cols_b = (N, K) if trans_b else (K, N)
    a = wl.tensor((batch, M, lda), F32, 1, "uniform", 1.0)
    b = wl.tensor((batch, rows_b, ldb), F32, 2, "uniform", 1.0)
    a[:, :, K:] = np.nan; b[:, :, cols_b:] = np.nan           # NaN outside the views
    bias = wl.tensor((N,), F32, 3, "uniform", 1.0) if epi in (C.EPI_BIAS, C.EPI_BIAS_RELU, C.EPI_BIAS_GELU_TANH) else None
    r = wl.tensor((batch, M, N), F32, 8, "uniform", 2.0) if residual else None
    out = T.device_empty(batch * M * ldc, F32, fill=0)
    da, db = T.to_device(a), T.to_device(b)
    dbias = None if bias is None else T.to_device(bias)
    with T.forced_kernel(force):
        if residual:
            assert batch == 1
            st = pbk.pbk_matmul_residual(da, db, out, dbias, T.to_device(r), M, N, K, lda, ldb, ldc, N, F32, F32,
                                         trans_b, alpha, 0.5, epi, None)
        elif batch == 1:
            st = pbk.pbk_matmul(da, db, out, dbias, M, N, K, lda, ldb, ldc, F32, F32, trans_b, alpha, epi)
        else:
            st = pbk.pbk_batched_matmul(da, db, out, dbias, batch, M, N, K, lda, ldb, ldc, M * lda, rows_b * ldb,
                                        M * ldc, F32, F32, trans_b, alpha, epi)
    assert st == 0, pbk.pbk_status_string(st)
    kern = pbk.pbk_last_kernel()
    got = T.to_host_f64(out, F32).reshape(batch, M, ldc)[:, :, :N]
    errs = []
    for i in range(batch):
        A2 = np.ascontiguousarray(a[i, :, :K]); B2 = np.ascontiguousarray(b[i, :, :cols_b])
        if residual:
            ref, pre = oracle.matmul_residual(A2, B2, bias, r[i], dtype=F32, r_dtype=F32, trans_b=trans_b, alpha=alpha,
                                              beta=0.5, epi=epi, want_preact=True)
        else:
            ref, pre = oracle.matmul(A2, B2, bias, dtype=F32, trans_b=trans_b, alpha=alpha, epi=epi, want_preact=True)
        errs.append(T.rel_err(got[i], ref, pre))
    return max(errs), kern


def test_the_256_cubed_configuration_takes_the_small_kernel():
    import paper_2603_06731_amd as pbk
    w = C.CONFIGS["cfg1_f32_256"]
    host = wl.make_inputs(w)
    st, out = T.run_workload(w, T.upload(host))
    assert st == 0
    assert "small_f32" in pbk.pbk_last_kernel(), pbk.pbk_last_kernel()
    ref, pre = T.oracle_full(w, host)
    err = T.rel_err(T.to_host_f64(out, F32).reshape(ref.shape), ref, pre)
    assert err <= T.TOL_F32, err


@pytest.mark.parametrize("trans_b", [0, 1])
@pytest.mark.parametrize("mnk_ld", [
    (256, 256, 256, None, None, None),
    (70, 45, 33, None, None, None),          # ragged in M, N and K
    (17, 130, 700, 703, None, 133),          # K beyond both register sets, odd leading dimensions
    (1, 1, 1, None, None, None),
    (100, 36, 129, 132, None, None),         # a k tail of one element, 16-byte loads allowed
    (48, 64, 260, None, None, None),
])
@pytest.mark.parametrize("epi", [C.EPI_NONE, C.EPI_BIAS_RELU, C.EPI_BIAS_GELU_TANH])
def test_small_f32_parity(trans_b, mnk_ld, epi):
    M, N, K, lda, ldb, ldc = mnk_ld
    err, kern = run(M, N, K, trans_b, epi, lda=lda, ldb=ldb, ldc=ldc, alpha=0.75, force="small")
    assert "small_f32" in kern, kern
    assert err <= T.TOL_F32, err


def test_small_f32_batched_and_residual():
    err, kern = run(40, 50, 90, 0, C.EPI_BIAS, batch=5, force="small")
    assert "small_f32" in kern and err <= T.TOL_F32, (kern, err)
    err, kern = run(70, 45, 33, 1, C.EPI_GELU_TANH, residual=True, force="small")
    assert "small_f32" in kern and err <= T.TOL_F32, (kern, err)


def test_dispatcher_keeps_larger_fp32_problems_off_the_small_kernel():
    err, kern = run(700, 600, 64, 0, C.EPI_NONE)               # 1672 tiles of 16 x 16
    assert "small_f32" not in kern and err <= T.TOL_F32, (kern, err)
    err, kern = run(70, 45, 33, 0, C.EPI_NONE, force="generic")
    assert "generic" in kern and err <= T.TOL_F32, (kern, err)


def test_small_choice_is_refused_for_other_dtypes():
    import paper_2603_06731_amd as pbk
    BF16 = wl.DTYPE_BF16
    a = T.to_device(wl.tensor((32, 32), BF16, 1, "normal")); b = T.to_device(wl.tensor((32, 32), BF16, 2, "normal"))
    out = T.device_empty(32 * 32, BF16, fill=0)
    with T.forced_kernel("small"):
        st = pbk.pbk_matmul(a, b, out, None, 32, 32, 32, 32, 32, 32, BF16, BF16, 0, 1.0, C.EPI_NONE)
    assert st != 0 and "not supported" in pbk.pbk_status_string(st)
