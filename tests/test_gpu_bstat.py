"""Parity of the B-stationary matrix-unit kernel (short contractions, K <= 256, over many rows: the
attention-score product and its relatives) with the CPU oracle, element by element."""
import numpy as np
import pytest

import workloads as wl
from workloads import configs as C
import pbk_testlib as T

pytestmark = pytest.mark.gpu

BF16, F16, F32 = wl.DTYPE_BF16, wl.DTYPE_F16, wl.DTYPE_F32
NAN16 = {BF16: 0x7FC0, F16: 0x7E00}


def run_case(batch, M, N, K, dtype, out_dtype, trans_b, epi, alpha=1.0, pad_ld=0, force="bstat", bias_on=True):
    """pbk_batched_matmul on views whose leading dimensions are pad_ld elements longer than the rows, with NaN
    in the padding; returns (max relative error, kernel name)."""
    import torch
    import oracle
    import paper_2603_06731_amd as pbk
    lda = K + pad_ld
    brows, bcols = (N, K) if trans_b else (K, N)
    ldb = bcols + pad_ld
    ldc = N + pad_ld
    a = wl.tensor((batch, M, lda), dtype, 1, "normal")
    b = wl.tensor((batch, brows, ldb), dtype, 2, "normal", 1.0 / np.sqrt(K))
    if pad_ld:
        a[:, :, K:] = NAN16[dtype]
        b[:, :, bcols:] = NAN16[dtype]
    bias = wl.tensor((N,), F32, 3, "normal", 0.5) if bias_on else None
    out = T.device_empty(batch * M * ldc, out_dtype, fill=0)
    with T.forced_kernel(force):
        st = pbk.pbk_batched_matmul(T.to_device(a.reshape(-1)), T.to_device(b.reshape(-1)), out,
                                    None if bias is None else T.to_device(bias), batch, M, N, K, lda, ldb, ldc,
                                    M * lda, brows * ldb, M * ldc, dtype, out_dtype, trans_b, alpha, epi)
    assert st == 0, pbk.pbk_status_string(st)
    torch.cuda.synchronize()
    kern = pbk.pbk_last_kernel()
    got = T.to_host_f64(out, out_dtype).reshape(batch, M, ldc)
    worst = 0.0
    for i in range(batch):
        ref, pre = oracle.matmul(np.ascontiguousarray(a[i, :, :K]), np.ascontiguousarray(b[i, :, :bcols]), bias,
                                 dtype=dtype, trans_b=trans_b, alpha=alpha, epi=epi, want_preact=True)
        worst = max(worst, T.rel_err(got[i, :, :N], ref, pre))
        if pad_ld:
            assert np.all(got[i, :, N:] == 0.0), "stores outside the view"
    return worst, kern


@pytest.mark.parametrize("trans_b", [0, 1])
@pytest.mark.parametrize("dtype,out_dtype", [(BF16, BF16), (F16, F16), (BF16, F32)])
@pytest.mark.parametrize("mnk", [
    (1024, 512, 128),        # whole steps, two column strips
    (1000, 264, 128),        # ragged last step (40 rows), ragged second strip (8 columns)
    (650, 256, 64),          # one 64-deep piece
    (77, 520, 96),           # K between the pieces: the second one half empty
    (200, 256, 40),          # K below one piece, not a multiple of 32
    (64, 8, 8),              # one step, one 16-byte piece of K, eight columns
    (700, 512, 256),         # four pieces, 32-row steps, a ragged last step
    (333, 264, 192),         # three pieces
    (96, 256, 136),          # just above two pieces
    (1000, 328, 232),        # four pieces, the last one ragged
])
def test_bstat_matches_oracle(mnk, dtype, out_dtype, trans_b):
    M, N, K = mnk
    err, kern = run_case(1, M, N, K, dtype, out_dtype, trans_b, C.EPI_BIAS_GELU_TANH, alpha=0.75)
    print(f"bstat {mnk} trans_b={trans_b} out={out_dtype} kernel={kern} err={err:.3e}", flush=True)
    assert "bstat" in kern
    assert err <= T.TIGHT[out_dtype], err


@pytest.mark.parametrize("trans_b", [0, 1])
@pytest.mark.parametrize("epi", [C.EPI_NONE, C.EPI_BIAS, C.EPI_RELU, C.EPI_BIAS_RELU, C.EPI_GELU_TANH])
def test_bstat_batched_views_and_epilogues(epi, trans_b):
    """Several batch entries, leading dimensions longer than the rows with NaN behind them, every epilogue;
    nothing may be stored outside the views."""
    for k in (128, 256):
        err, kern = run_case(3, 712, 328, k, BF16, BF16, trans_b, epi, alpha=1.0 / np.sqrt(128.0), pad_ld=8,
                             bias_on=epi in (C.EPI_BIAS, C.EPI_BIAS_RELU))
        assert "bstat" in kern and err <= T.TIGHT[BF16], (kern, err)


def test_bstat_is_the_dispatchers_choice_for_the_score_product_and_equals_the_tile_kernel():
    """A store-bound short contraction goes to this kernel by itself, and its result is that of the
    tile-per-workgroup configuration to within the output rounding."""
    err, kern = run_case(32, 2048, 1024, 128, BF16, BF16, 0, C.EPI_NONE, alpha=1.0 / np.sqrt(128.0), force=None, bias_on=False)
    assert "bstat" in kern and err <= T.TIGHT[BF16], (kern, err)
    err6, kern6 = run_case(32, 2048, 1024, 128, BF16, BF16, 0, C.EPI_NONE, alpha=1.0 / np.sqrt(128.0), force="mfma:6", bias_on=False)
    assert "128x256" in kern6 and err6 <= T.TIGHT[BF16], (kern6, err6)


def test_bstat_declines_long_contractions_and_convolutions():
    import paper_2603_06731_amd as pbk
    a = T.to_device(wl.tensor((64, 264), BF16, 1, "normal")); b = T.to_device(wl.tensor((264, 64), BF16, 2, "normal"))
    out = T.device_empty(64 * 64, BF16, fill=0)
    with T.forced_kernel("bstat"):
        st = pbk.pbk_matmul(a, b, out, None, 64, 64, 264, 264, 64, 64, BF16, BF16, 0, 1.0, C.EPI_NONE)
    assert st != 0 and "not supported" in pbk.pbk_status_string(st), pbk.pbk_status_string(st)
