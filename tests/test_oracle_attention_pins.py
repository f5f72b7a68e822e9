"""Pins for the attention oracle: closed forms of the softmax, special cases,
invariances, torch's float64 operators as the library routine, and a loop in
plain Python.  None of these tests touches the HIP library."""
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
    """What the oracle reads: the stored values as float64."""
    s = as_dtype(x, dtype)
    return s.astype(np.float64) if dtype == F32 else wl.widen(s, dtype)


ALL_DTYPES = [F32, BF16, F16]


# ------------------------------------------------------------- closed forms

@pytest.mark.parametrize("dtype", ALL_DTYPES)
def test_zero_queries_average_the_values(dtype):
    # all scores equal -> uniform weights -> every output row is the column mean of V
    r = rng(1)
    V = r.integers(-8, 9, size=(3, 11, 6)).astype(np.float64)
    K = r.integers(-4, 5, size=(3, 11, 6)).astype(np.float64)
    Q = np.zeros((3, 5, 6))
    out = oracle.attention(as_dtype(Q, dtype), as_dtype(K, dtype), as_dtype(V, dtype), dtype=dtype, alpha=0.7)
    want = np.broadcast_to(V.mean(axis=1, keepdims=True), out.shape)
    np.testing.assert_allclose(out, want, rtol=0, atol=1e-14)


@pytest.mark.parametrize("dtype", ALL_DTYPES)
def test_single_key_returns_its_value(dtype):
    r = rng(2)
    Q = r.normal(size=(2, 7, 4)); K = r.normal(size=(2, 1, 4)); V = r.integers(-9, 10, size=(2, 1, 4)).astype(np.float64)
    out = oracle.attention(as_dtype(Q, dtype), as_dtype(K, dtype), as_dtype(V, dtype), dtype=dtype, alpha=3.0)
    assert np.array_equal(out, np.broadcast_to(V, out.shape))


def test_two_keys_give_a_logistic_mix():
    # weights of two keys are sigmoid(+-(s0 - s1)); D = 1 makes the scores q*k
    q, k0, k1, v0, v1, alpha = 1.5, 2.0, -1.0, 10.0, -6.0, 0.5
    Q = np.array([[[q]]], dtype=np.float32)
    K = np.array([[[k0], [k1]]], dtype=np.float32)
    V = np.array([[[v0], [v1]]], dtype=np.float32)
    out = oracle.attention(Q, K, V, dtype=F32, alpha=alpha)
    w0 = 1.0 / (1.0 + math.exp(-(alpha * q * k0 - alpha * q * k1)))
    assert out[0, 0, 0] == pytest.approx(w0 * v0 + (1 - w0) * v1, rel=1e-15)
    # the weight must sit on the key with the LARGER score
    assert out[0, 0, 0] > 0.5 * (v0 + v1)


def test_alpha_scales_scores_not_bias():
    # alpha = 0 leaves softmax(bias): bias = log(1,2,3,...) gives weights j / sum
    n = 5
    bias = np.log(np.arange(1, n + 1, dtype=np.float64))[None, :].repeat(3, axis=0).astype(np.float32)
    r = rng(3)
    Q = r.normal(size=(1, 3, 4)).astype(np.float32); K = r.normal(size=(1, n, 4)).astype(np.float32)
    V = r.normal(size=(1, n, 4)).astype(np.float32)
    out = oracle.attention(Q, K, V, bias, dtype=F32, alpha=0.0)
    w = np.exp(bias[0].astype(np.float64)); w /= w.sum()
    np.testing.assert_allclose(out[0], w[None, :] @ V[0].astype(np.float64) * np.ones((3, 1)), rtol=1e-14)


def test_bias_is_indexed_query_then_key():
    # a bias that favours key (i + 1) mod n for query i picks row (i + 1) of V:
    # a transposed bias would pick (i - 1)
    n = 6
    bias = np.full((n, n), -1e4, dtype=np.float32)
    for i in range(n):
        bias[i, (i + 1) % n] = 0.0
    V = np.arange(n * 3, dtype=np.float32).reshape(1, n, 3)
    Z = np.zeros((1, n, 3), dtype=np.float32)
    out = oracle.attention(Z, Z, V, bias, dtype=F32)
    assert np.array_equal(out[0], np.roll(V[0], -1, axis=0))


def test_sharp_scores_select_the_matching_key():
    # orthogonal keys, queries equal to keys, large alpha: row i attends to key i only
    n = 8
    E = np.eye(n)
    V = rng(4).integers(-5, 6, size=(1, n, n)).astype(np.float64)
    out = oracle.attention(as_dtype(E[None], F32), as_dtype(E[None], F32), as_dtype(V, F32), dtype=F32, alpha=800.0)
    assert np.array_equal(out, V)            # exp(-800) underflows to exactly 0


# -------------------------------------------------------------- invariances

def test_row_shift_and_large_scores():
    r = rng(5)
    Q = r.normal(size=(2, 9, 16)).astype(np.float32); K = r.normal(size=(2, 13, 16)).astype(np.float32)
    V = r.normal(size=(2, 13, 16)).astype(np.float32)
    bias = r.normal(size=(2, 9, 13)).astype(np.float32)
    base = oracle.attention(Q, K, V, bias, dtype=F32, alpha=0.3)
    # adding a constant per query row changes nothing, even one that would overflow exp()
    shift = (r.integers(-3, 4, size=(2, 9, 1)) * 512.0).astype(np.float32)
    moved = oracle.attention(Q, K, V, bias + shift, dtype=F32, alpha=0.3)
    # bias + shift is rounded to float32: compare against the oracle fed the same rounded bias
    np.testing.assert_allclose(moved, oracle.attention(Q, K, V, ((bias + shift) - shift).astype(np.float32),
                                                       dtype=F32, alpha=0.3), rtol=1e-9, atol=1e-11)
    assert np.all(np.isfinite(moved))
    # (a score near 3e4 carries an absolute rounding error of about 4e-12 in double)
    big = oracle.attention(Q, K, V, np.full_like(bias, 3.0e4), dtype=F32, alpha=0.3)
    np.testing.assert_allclose(big, oracle.attention(Q, K, V, dtype=F32, alpha=0.3), rtol=1e-8, atol=1e-10)
    assert base.shape == (2, 9, 16)


def test_key_permutation_invariance():
    r = rng(6)
    Q = r.normal(size=(1, 5, 8)).astype(np.float32); K = r.normal(size=(1, 12, 8)).astype(np.float32)
    V = r.normal(size=(1, 12, 8)).astype(np.float32); bias = r.normal(size=(5, 12)).astype(np.float32)
    p = r.permutation(12)
    a = oracle.attention(Q, K, V, bias, dtype=F32, alpha=0.5)
    b = oracle.attention(Q, K[:, p].copy(), V[:, p].copy(), bias[:, p].copy(), dtype=F32, alpha=0.5)
    np.testing.assert_allclose(a, b, rtol=1e-13, atol=1e-14)


def test_minus_infinity_bias_removes_keys():
    r = rng(7)
    Q = r.normal(size=(1, 6, 8)).astype(np.float32); K = r.normal(size=(1, 10, 8)).astype(np.float32)
    V = r.normal(size=(1, 10, 8)).astype(np.float32)
    keep = np.array([0, 2, 3, 7, 9])
    bias = np.full((6, 10), -np.inf, dtype=np.float32)
    bias[:, keep] = 0.0
    a = oracle.attention(Q, K, V, bias, dtype=F32, alpha=0.4)
    b = oracle.attention(Q, K[:, keep].copy(), V[:, keep].copy(), dtype=F32, alpha=0.4)
    np.testing.assert_allclose(a, b, rtol=1e-14, atol=0)
    # causal mask: row i sees keys 0..i; row 0 returns V[0]
    causal = np.where(np.arange(10)[None, :] <= np.arange(6)[:, None], 0.0, -np.inf).astype(np.float32)
    c = oracle.attention(Q, K, V, causal, dtype=F32)
    np.testing.assert_allclose(c[0, 0], V[0, 0].astype(np.float64), rtol=0, atol=0)


def test_outputs_are_convex_combinations():
    r = rng(8)
    Q = r.normal(size=(2, 17, 8)).astype(np.float32) * 3; K = r.normal(size=(2, 29, 8)).astype(np.float32)
    V = r.normal(size=(2, 29, 8)).astype(np.float32)
    out = oracle.attention(Q, K, V, dtype=F32)
    lo = V.min(axis=1, keepdims=True).astype(np.float64); hi = V.max(axis=1, keepdims=True).astype(np.float64)
    assert np.all(out >= lo - 1e-12) and np.all(out <= hi + 1e-12)
    # with V = all ones the weights' sum is visible: exactly 1 up to rounding
    ones = oracle.attention(Q, K, np.ones_like(V), dtype=F32)
    np.testing.assert_allclose(ones, 1.0, rtol=1e-14)


# ------------------------------------------- library routine and brute force

@pytest.mark.parametrize("dtype", ALL_DTYPES)
@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (2, 7, 5, 3), (3, 33, 70, 16), (1, 64, 129, 32)])
@pytest.mark.parametrize("bias_kind", ["none", "shared", "per_batch"])
def test_against_torch_float64(dtype, shape, bias_kind):
    b, nq, nk, d = shape
    r = rng(100 + nq + nk)
    Q = r.normal(size=(b, nq, d)); K = r.normal(size=(b, nk, d)); V = r.normal(size=(b, nk, d))
    bias = {"none": None, "shared": r.normal(size=(nq, nk)), "per_batch": r.normal(size=(b, nq, nk))}[bias_kind]
    bias32 = None if bias is None else bias.astype(np.float32)
    alpha = float(np.float32(1.0 / math.sqrt(d)))
    got = oracle.attention(as_dtype(Q, dtype), as_dtype(K, dtype), as_dtype(V, dtype), bias32, dtype=dtype, alpha=alpha)
    q, k, v = (torch.from_numpy(widened(x, dtype)) for x in (Q, K, V))
    s = alpha * (q @ k.transpose(-1, -2))
    if bias32 is not None:
        s = s + torch.from_numpy(bias32.astype(np.float64))
    want = torch.softmax(s, dim=-1) @ v
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-12, atol=1e-13)
    # torch's fused operator as a second library routine
    mask = None if bias32 is None else torch.from_numpy(bias32.astype(np.float64)).expand(b, nq, nk)
    sdpa = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=mask, scale=alpha)
    np.testing.assert_allclose(got, sdpa.numpy(), rtol=1e-11, atol=1e-12)


def test_against_plain_python_loops():
    r = rng(9)
    b, nq, nk, d = 2, 4, 6, 3
    Q = r.normal(size=(b, nq, d)).astype(np.float32); K = r.normal(size=(b, nk, d)).astype(np.float32)
    V = r.normal(size=(b, nk, d)).astype(np.float32); bias = r.normal(size=(b, nq, nk)).astype(np.float32)
    alpha = 0.75
    got = oracle.attention(Q, K, V, bias, dtype=F32, alpha=alpha)
    for bb in range(b):
        for i in range(nq):
            e = []
            for j in range(nk):
                s = sum(float(Q[bb, i, c]) * float(K[bb, j, c]) for c in range(d))
                e.append(math.exp(alpha * s + float(bias[bb, i, j])))      # no max shift here
            tot = math.fsum(e)
            for dd in range(d):
                want = math.fsum(e[j] * float(V[bb, j, dd]) for j in range(nk)) / tot
                assert got[bb, i, dd] == pytest.approx(want, rel=1e-13, abs=1e-15)


def test_rows_variant_matches_full():
    r = rng(10)
    Q = as_dtype(r.normal(size=(3, 20, 8)), BF16); K = as_dtype(r.normal(size=(3, 31, 8)), BF16)
    V = as_dtype(r.normal(size=(3, 31, 8)), BF16); bias = r.normal(size=(20, 31)).astype(np.float32)
    full = oracle.attention(Q, K, V, bias, dtype=BF16, alpha=0.35)
    sb = np.array([0, 2, 1, 2, 0]); si = np.array([0, 19, 7, 3, 19])
    rows = oracle.attention_rows(Q, K, V, bias, sb, si, dtype=BF16, alpha=0.35)
    assert np.array_equal(rows, full[sb, si])


def test_rejects_bad_arguments():
    Q = np.zeros((1, 2, 4), np.float32)
    with pytest.raises(ValueError):
        oracle.attention(Q, np.zeros((1, 3, 5), np.float32), np.zeros((1, 3, 5), np.float32), dtype=F32)
    with pytest.raises(ValueError):
        oracle.attention(Q, Q, Q, np.zeros((3, 3), np.float32), dtype=F32)
    with pytest.raises(TypeError):
        oracle.attention(Q, Q, Q, dtype=BF16)
    with pytest.raises(ValueError):
        oracle.attention_rows(Q, Q, Q, None, [0], [2], dtype=F32)
