"""Pins for the int8 oracle: exact integer sums against numpy's integer
matmul and torch's integer convolution, the binary32 epilogue against numpy's
float32 element operations step by step, and hand-computed rounding,
saturation and ordering cases.  None of these tests touches the HIP library."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle


def rng(seed):
    return np.random.default_rng(seed)


def i8(r, shape):
    return r.integers(-128, 128, size=shape, dtype=np.int8)


def ref_epilogue(acc, scale, bias, mid_scale, mul, add, relu, out_scale, out_int8):
    """numpy float32, one rounded operation per line (numpy never contracts)."""
    f = np.float32
    t = acc.astype(np.float32)                     # int32 -> float32, round to nearest even
    t = t * scale[None, :]
    if bias is not None:
        t = t + bias[None, :]
    if mid_scale > 0:
        q = np.clip(np.rint(t / f(mid_scale)), f(-128), f(127))
        t = q * f(mid_scale)
    if mul is not None:
        t = t * mul[None, :]
    if add is not None:
        t = t + add[None, :]
    if relu:
        t = np.where(t > 0, t, f(0))
    if not out_int8:
        return t.astype(np.float32)
    return np.clip(np.rint(t / f(out_scale)), f(-128), f(127)).astype(np.int8)


# ------------------------------------------------------------- integer sums

@pytest.mark.parametrize("mnk", [(1, 1, 1), (5, 7, 3), (33, 20, 257), (8, 8, 4096)])
@pytest.mark.parametrize("trans_b", [0, 1])
def test_integer_sums_match_numpy_int64(mnk, trans_b):
    m, n, k = mnk
    r = rng(m + n + k)
    A = i8(r, (m, k)); B = i8(r, (n, k) if trans_b else (k, n))
    _, acc = oracle.matmul_int8(A, B, scale=np.ones(n, np.float32), trans_b=trans_b, want_acc=True)
    Bm = B.T if trans_b else B
    assert np.array_equal(acc, A.astype(np.int64) @ Bm.astype(np.int64))


def test_extreme_values_stay_exact():
    k = 4096
    A = np.full((2, k), -128, np.int8); B = np.full((k, 3), -128, np.int8)
    _, acc = oracle.matmul_int8(A, B, scale=np.ones(3, np.float32), want_acc=True)
    assert np.all(acc == k * 16384)
    B[:] = 127
    _, acc = oracle.matmul_int8(A, B, scale=np.ones(3, np.float32), want_acc=True)
    assert np.all(acc == -k * 128 * 127)


@pytest.mark.parametrize("geom", [((1, 1), (0, 0), (1, 1)), ((2, 2), (1, 1), (1, 1)), ((1, 2), (2, 0), (2, 1))])
def test_conv_integer_sums_match_torch(geom):
    stride, pad, dil = geom
    r = rng(5)
    x = i8(r, (2, 9, 8, 5)); w = i8(r, (3, 3, 5, 4))
    _, acc = oracle.conv2d_nhwc_int8(x, w, scale=np.ones(4, np.float32), stride=stride, pad=pad, dil=dil, want_acc=True)
    t = F.conv2d(torch.from_numpy(x.astype(np.int64)).permute(0, 3, 1, 2),
                 torch.from_numpy(w.astype(np.int64)).permute(3, 2, 0, 1), stride=stride, padding=pad, dilation=dil)
    assert np.array_equal(acc, t.permute(0, 2, 3, 1).numpy())


# ---------------------------------------------------------------- epilogue

def test_rounding_is_to_nearest_even_and_saturates():
    A = np.array([[1], [3], [5], [-1], [-3], [100], [-100]], np.int8); B = np.array([[1]], np.int8)
    out = oracle.matmul_int8(A, B, scale=np.ones(1, np.float32), out_scale=2.0)
    assert out[:, 0].tolist() == [0, 2, 2, 0, -2, 50, -50]               # .5 ties go to the even code
    out = oracle.matmul_int8(A, B, scale=np.full(1, 3.0, np.float32), out_scale=1.0)
    assert out[:, 0].tolist() == [3, 9, 15, -3, -9, 127, -128]           # clamp to [-128, 127]


def test_order_of_the_steps():
    one = np.ones(1, np.float32)
    A = np.array([[10]], np.int8); B = np.array([[1]], np.int8)
    # de-quantise, bias:  10 * 0.25 + 0.3 = 2.8
    f = oracle.matmul_int8(A, B, scale=one * 0.25, bias=one * 0.3, out_int8=False)
    assert f[0, 0] == np.float32(np.float32(10 * 0.25) + np.float32(0.3))
    # the middle quantise / de-quantise pair snaps 2.8 to the grid of step 1: 3
    f = oracle.matmul_int8(A, B, scale=one * 0.25, bias=one * 0.3, mid_scale=1.0, out_int8=False)
    assert f[0, 0] == 3.0
    # affine after the pair, ReLU after the affine:  3 * -2 + 1 = -5 -> 0 ;  3 * 2 - 1 = 5
    f = oracle.matmul_int8(A, B, scale=one * 0.25, bias=one * 0.3, mid_scale=1.0, mul=-2 * one, add=one, relu=True, out_int8=False)
    assert f[0, 0] == 0.0
    f = oracle.matmul_int8(A, B, scale=one * 0.25, bias=one * 0.3, mid_scale=1.0, mul=2 * one, add=-one, relu=True, out_int8=False)
    assert f[0, 0] == 5.0
    # ReLU before the output quantisation: -5 / 0.5 would be -10, ReLU makes it 0
    q = oracle.matmul_int8(A, B, scale=one * 0.25, bias=one * 0.3, mid_scale=1.0, mul=-2 * one, add=one, relu=True, out_scale=0.5)
    assert q[0, 0] == 0
    q = oracle.matmul_int8(A, B, scale=one * 0.25, bias=one * 0.3, mid_scale=1.0, mul=-2 * one, add=one, relu=False, out_scale=0.5)
    assert q[0, 0] == -10
    # per-channel parameters are indexed by the OUTPUT column
    A = np.array([[1, 1]], np.int8); B = np.array([[1, 2, 3], [0, 0, 0]], np.int8)
    f = oracle.matmul_int8(A, B, scale=np.array([1, 10, 100], np.float32), out_int8=False)
    assert f[0].tolist() == [1.0, 20.0, 300.0]


@pytest.mark.parametrize("variant", range(6))
def test_epilogue_matches_numpy_float32_step_by_step(variant):
    r = rng(100 + variant)
    m, n, k = 37, 29, 300
    A = i8(r, (m, k)); B = i8(r, (k, n))
    scale = (r.uniform(0.5, 2.0, n) * 1e-3).astype(np.float32)
    bias = r.normal(0, 0.5, n).astype(np.float32) if variant & 1 else None
    mid = [0.0, 0.05, 0.0, 0.031, 0.07, 0.0][variant]
    mul = r.uniform(0.5, 1.5, n).astype(np.float32) if variant in (2, 3, 4) else None
    add = r.normal(0, 0.3, n).astype(np.float32) if variant in (3, 4, 5) else None
    relu = variant in (1, 3, 4)
    out_scale = 0.043
    for out_int8 in (True, False):
        got, acc = oracle.matmul_int8(A, B, scale=scale, bias=bias, mid_scale=mid, mul=mul, add=add, relu=relu,
                                      out_scale=out_scale, out_int8=out_int8, want_acc=True)
        want = ref_epilogue(acc, scale, bias, mid, mul, add, relu, out_scale, out_int8)
        assert np.array_equal(got, want)
    codes = oracle.matmul_int8(A, B, scale=scale, bias=bias, mid_scale=mid, mul=mul, add=add, relu=relu, out_scale=out_scale)
    assert len(np.unique(codes)) > 20          # the case really exercises the quantiser


def test_large_sums_convert_to_float_with_one_rounding():
    # 2^24 + 1 is not a float: the conversion must round to even (2^24), not truncate or go through double math
    k = 1042
    A = np.full((1, k), 127, np.int8); B = np.full((k, 1), 127, np.int8)
    B[-1, 0] = 0; A[0, -1] = 0
    f, acc = oracle.matmul_int8(A, B, scale=np.ones(1, np.float32), out_int8=False, want_acc=True)
    assert acc[0, 0] == (k - 1) * 16129 and acc[0, 0] > 2 ** 24
    assert f[0, 0] == np.float32(acc[0, 0])


def test_conv_uses_the_same_epilogue():
    r = rng(9)
    x = i8(r, (1, 6, 6, 8)); w = i8(r, (1, 1, 8, 5))
    scale = np.full(5, 2e-3, np.float32); bias = r.normal(size=5).astype(np.float32)
    c = oracle.conv2d_nhwc_int8(x, w, scale=scale, bias=bias, mid_scale=0.1, relu=True, out_scale=0.05)
    m = oracle.matmul_int8(x.reshape(36, 8), w.reshape(8, 5), scale=scale, bias=bias, mid_scale=0.1, relu=True, out_scale=0.05)
    assert np.array_equal(c.reshape(36, 5), m)


def test_rejects_bad_arguments():
    A = np.zeros((2, 2), np.int8)
    with pytest.raises(ValueError):
        oracle.matmul_int8(A, A, scale=np.ones(2, np.float32), out_scale=0.0)
    with pytest.raises(TypeError):
        oracle.matmul_int8(A.astype(np.int16), A, scale=np.ones(2, np.float32))
    with pytest.raises(TypeError):
        oracle.matmul_int8(A, A, scale=np.ones(3, np.float32))
