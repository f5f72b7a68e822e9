"""Pins for the causal attention oracle: the explicitly masked form of the separately pinned attention
oracle, torch's float64 operators, special rows with a closed form, and plain Python loops.  None of these
tests touches the HIP library."""
import math

import numpy as np
import pytest
import torch

import oracle
from oracle import F32, BF16, F16
import workloads as wl


def rng(seed):
    return np.random.default_rng(seed)


def as_dtype(x, dtype):
    return wl.to_storage(np.asarray(x, dtype=np.float64), dtype)


def widened(x, dtype):
    s = as_dtype(x, dtype)
    return s.astype(np.float64) if dtype == F32 else wl.widen(s, dtype)


def visible(nq, nk):
    """visible[i][j]: key j <= i + (nk - nq)."""
    i = np.arange(nq)[:, None]; j = np.arange(nk)[None, :]
    return j <= i + (nk - nq)


@pytest.mark.parametrize("dtype", [F32, BF16, F16])
@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (2, 7, 7, 3), (3, 33, 70, 16), (1, 64, 64, 32), (2, 5, 9, 4)])
def test_equals_attention_with_minus_infinity_above_the_diagonal(dtype, shape):
    b, nq, nk, d = shape
    r = rng(300 + nq + nk)
    Q = as_dtype(r.normal(size=(b, nq, d)), dtype); K = as_dtype(r.normal(size=(b, nk, d)), dtype)
    V = as_dtype(r.normal(size=(b, nk, d)), dtype)
    alpha = float(np.float32(1.0 / math.sqrt(d)))
    got = oracle.attention_causal(Q, K, V, dtype=dtype, alpha=alpha)
    mask = np.where(visible(nq, nk), 0.0, -np.inf).astype(np.float32)
    want = oracle.attention(Q, K, V, mask, dtype=dtype, alpha=alpha)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("shape", [(2, 9, 9, 8), (1, 40, 40, 16)])
def test_against_torch_float64_is_causal(shape):
    b, n, _, d = shape
    r = rng(41)
    Q = r.normal(size=(b, n, d)); K = r.normal(size=(b, n, d)); V = r.normal(size=(b, n, d))
    alpha = float(np.float32(0.3))        # the oracle takes alpha as a binary32 value
    got = oracle.attention_causal(as_dtype(Q, BF16), as_dtype(K, BF16), as_dtype(V, BF16), dtype=BF16, alpha=alpha)
    q, k, v = (torch.from_numpy(widened(x, BF16)) for x in (Q, K, V))
    want = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True, scale=alpha)
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-11, atol=1e-12)
    s = alpha * (q @ k.transpose(-1, -2))
    s = s.masked_fill(torch.from_numpy(~visible(n, n)), -math.inf)
    np.testing.assert_allclose(got, (torch.softmax(s, dim=-1) @ v).numpy(), rtol=1e-12, atol=1e-13)


def test_first_row_is_the_first_value_and_last_row_sees_every_key():
    r = rng(5)
    Q = r.normal(size=(2, 6, 4)).astype(np.float32); K = r.normal(size=(2, 6, 4)).astype(np.float32)
    V = r.normal(size=(2, 6, 4)).astype(np.float32)
    got = oracle.attention_causal(Q, K, V, dtype=F32, alpha=0.9)
    assert np.array_equal(got[:, 0], V[:, 0].astype(np.float64))          # one key: weight 1
    full = oracle.attention(Q, K, V, None, dtype=F32, alpha=0.9)
    np.testing.assert_allclose(got[:, -1], full[:, -1], rtol=1e-14)


def test_fewer_queries_than_keys_are_the_last_positions():
    """Nq = 3, Nk = 8: row i sees keys 0 .. i + 5, i.e. rows 5, 6, 7 of the square problem."""
    r = rng(6)
    K = r.normal(size=(1, 8, 4)).astype(np.float32); V = r.normal(size=(1, 8, 4)).astype(np.float32)
    Qsq = r.normal(size=(1, 8, 4)).astype(np.float32)
    square = oracle.attention_causal(Qsq, K, V, dtype=F32, alpha=0.5)
    tail = oracle.attention_causal(np.ascontiguousarray(Qsq[:, 5:]), K, V, dtype=F32, alpha=0.5)
    np.testing.assert_allclose(tail, square[:, 5:], rtol=1e-14)


def test_more_queries_than_keys_leaves_rows_without_keys_undefined():
    Q = np.ones((1, 4, 2), np.float32); K = np.ones((1, 2, 2), np.float32); V = np.ones((1, 2, 2), np.float32)
    got = oracle.attention_causal(Q, K, V, dtype=F32, alpha=1.0)
    assert np.isnan(got[0, :2]).all() and np.isfinite(got[0, 2:]).all()


def test_against_plain_python_loops():
    r = rng(7)
    b, nq, nk, d = 2, 4, 6, 3
    Q = r.normal(size=(b, nq, d)).astype(np.float32); K = r.normal(size=(b, nk, d)).astype(np.float32)
    V = r.normal(size=(b, nk, d)).astype(np.float32)
    alpha = 0.75
    got = oracle.attention_causal(Q, K, V, dtype=F32, alpha=alpha)
    for bb in range(b):
        for i in range(nq):
            keys = [j for j in range(nk) if j <= i + nk - nq]
            e = [math.exp(alpha * sum(float(Q[bb, i, c]) * float(K[bb, j, c]) for c in range(d))) for j in keys]
            tot = math.fsum(e)
            for dd in range(d):
                want = math.fsum(w * float(V[bb, j, dd]) for w, j in zip(e, keys)) / tot
                assert got[bb, i, dd] == pytest.approx(want, rel=1e-13, abs=1e-15)


def test_rows_variant_matches_full():
    r = rng(8)
    Q = as_dtype(r.normal(size=(3, 20, 8)), F16); K = as_dtype(r.normal(size=(3, 31, 8)), F16)
    V = as_dtype(r.normal(size=(3, 31, 8)), F16)
    full = oracle.attention_causal(Q, K, V, dtype=F16, alpha=0.35)
    sb = np.array([0, 2, 1, 2, 0]); si = np.array([0, 19, 7, 3, 19])
    rows = oracle.attention_causal_rows(Q, K, V, sb, si, dtype=F16, alpha=0.35)
    assert np.array_equal(rows, full[sb, si])


def test_a_planted_mistake_would_be_seen():
    """Off-by-one in the visible range (j < i instead of j <= i) changes every row but the last."""
    r = rng(11)
    Q = r.normal(size=(1, 5, 4)).astype(np.float32); K = r.normal(size=(1, 5, 4)).astype(np.float32)
    V = r.normal(size=(1, 5, 4)).astype(np.float32)
    got = oracle.attention_causal(Q, K, V, dtype=F32, alpha=1.0)
    wrong_mask = np.where(np.arange(5)[None, :] < np.arange(5)[:, None] + 0, 0.0, -np.inf).astype(np.float32)
    wrong_mask[0, 0] = 0.0
    wrong = oracle.attention(Q, K, V, wrong_mask, dtype=F32, alpha=1.0)
    assert np.abs(got[0, 1:] - wrong[0, 1:]).max() > 1e-3
