"""Pins for the residual-add epilogue of the oracle.  None of these tests
touches the HIP library."""
import numpy as np
import pytest

import oracle
from oracle import F32, BF16, F16
import workloads as wl


def rng(seed):
    return np.random.default_rng(seed)


def sto(x, dtype):
    return wl.to_storage(np.asarray(x, dtype=np.float64), dtype)


def wide(x, dtype):
    s = sto(x, dtype)
    return s.astype(np.float64) if dtype == F32 else wl.widen(s, dtype)


@pytest.mark.parametrize("dtype,r_dtype", [(F32, F32), (BF16, BF16), (F16, F32), (BF16, F16)])
@pytest.mark.parametrize("trans_b", [0, 1])
def test_matches_numpy_float64(dtype, r_dtype, trans_b):
    r = rng(3)
    m, n, k = 9, 14, 21
    A = r.normal(size=(m, k)); B = r.normal(size=(n, k) if trans_b else (k, n)); R = r.normal(size=(m, n))
    bias = r.normal(size=n).astype(np.float32)
    got, pre = oracle.matmul_residual(sto(A, dtype), sto(B, dtype), bias, sto(R, r_dtype), dtype=dtype, r_dtype=r_dtype,
                                      trans_b=trans_b, alpha=0.75, beta=-1.5, epi=oracle.EPI_BIAS_RELU, want_preact=True)
    Bm = wide(B, dtype).T if trans_b else wide(B, dtype)
    want = np.float64(np.float32(0.75)) * (wide(A, dtype) @ Bm) + bias.astype(np.float64) + np.float64(np.float32(-1.5)) * wide(R, r_dtype)
    np.testing.assert_allclose(pre, want, rtol=1e-13, atol=1e-13)
    assert np.array_equal(got, np.maximum(pre, 0.0))


def test_special_cases_and_order():
    r = rng(4)
    A = sto(r.normal(size=(6, 8)), F32); B = sto(r.normal(size=(8, 5)), F32)
    R = sto(r.integers(-4, 5, size=(6, 5)), F32)
    plain = oracle.matmul(A, B, dtype=F32, alpha=0.5)
    # beta = 0 or R = 0: the plain operator
    assert np.array_equal(oracle.matmul_residual(A, B, None, R, dtype=F32, r_dtype=F32, alpha=0.5, beta=0.0), plain)
    assert np.array_equal(oracle.matmul_residual(A, B, None, np.zeros_like(R), dtype=F32, r_dtype=F32, alpha=0.5), plain)
    # A = 0: act(bias + beta R); R indexed [row][column], alpha does not touch it, the activation comes last
    bias = np.arange(5, dtype=np.float32)
    out = oracle.matmul_residual(np.zeros_like(A), B, bias, R, dtype=F32, r_dtype=F32, alpha=7.0, beta=2.0, epi=oracle.EPI_BIAS_RELU)
    assert np.array_equal(out, np.maximum(bias[None, :].astype(np.float64) + 2.0 * R.astype(np.float64), 0.0))
    # a transposed R would differ on a non-square output
    assert not np.array_equal(out[:5, :5], np.maximum(bias[None, :] + 2.0 * R.astype(np.float64)[:5, :5].T, 0.0))


def test_conv_residual_is_conv_plus_residual():
    r = rng(5)
    x = sto(r.normal(size=(2, 7, 6, 4)), BF16); w = sto(r.normal(size=(3, 3, 4, 5)), BF16)
    bias = r.normal(size=5).astype(np.float32)
    _, pre = oracle.conv2d_nhwc(x, w, bias, dtype=BF16, stride=(2, 1), pad=(1, 1), alpha=0.5, epi=oracle.EPI_BIAS, want_preact=True)
    res = sto(r.normal(size=pre.shape), BF16)
    got, gpre = oracle.conv2d_nhwc_residual(x, w, bias, res, dtype=BF16, r_dtype=BF16, stride=(2, 1), pad=(1, 1),
                                            alpha=0.5, beta=1.0, epi=oracle.EPI_BIAS_RELU, want_preact=True)
    np.testing.assert_allclose(gpre, pre + wl.widen(res, BF16), rtol=1e-15, atol=1e-15)
    assert np.array_equal(got, np.maximum(gpre, 0.0))
