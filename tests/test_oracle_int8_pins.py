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


# ------------------------------------------- unfolded batch norm (the figure's form)

def _f32(x):
    """Exact rational -> nearest binary32 (ties to even), as an exact rational again."""
    import struct
    from fractions import Fraction
    x = Fraction(x)
    if x == 0:
        return Fraction(0)
    # float() of a Fraction rounds correctly to binary64; binary64 -> binary32 could round twice, so the
    # two binary32 neighbours are compared with the exact value instead
    approx = struct.unpack("f", struct.pack("f", float(x)))[0]
    bits = struct.unpack("I", struct.pack("f", approx))[0]
    cands = []
    for d in (-1, 0, 1):
        b = bits + d
        v = struct.unpack("f", struct.pack("I", b))[0]
        cands.append((abs(Fraction(v) - x), b & 1, Fraction(v)))
    cands.sort(key=lambda c: (c[0], c[1]))          # nearest; on a tie the even significand
    return cands[0][2]


def _sqrt_f32(x):
    """Correctly rounded binary32 square root of an exact rational, by integer square roots."""
    from fractions import Fraction
    from math import isqrt
    x = Fraction(x)
    # sqrt(x) to 80 fractional bits: floor(sqrt(x * 4^80)) / 2^80, never a binary32 tie for these inputs
    n = isqrt((x.numerator << 160) // x.denominator)
    return _f32(Fraction(n, 1 << 80))


def exact_bn_epilogue(acc, scale, bias, mid, mean, var, eps, gamma, beta, relu, out_scale):
    """The figure's operations in exact rational arithmetic with one binary32 rounding after each."""
    from fractions import Fraction

    def F(v):                      # a binary32 (or Python) number as the exact rational it is
        return v if isinstance(v, Fraction) else Fraction(float(v))

    def q(t, step):
        v = _f32(t / F(step))
        fl = v.numerator // v.denominator
        frac = v - fl
        r = fl + (1 if frac > Fraction(1, 2) or (frac == Fraction(1, 2) and fl % 2 == 1) else 0)
        return Fraction(max(-128, min(127, r)))
    t = _f32(Fraction(int(acc)))
    t = _f32(t * F(scale))
    t = _f32(t + F(bias))
    t = _f32(q(t, mid) * F(mid))
    r = _f32(F(var) + F(eps))
    r = _sqrt_f32(r)
    r = _f32(1 / r)
    t = _f32(t - F(mean))
    t = _f32(t * r)
    t = _f32(t * F(gamma))
    t = _f32(t + F(beta))
    if relu and t <= 0:
        t = Fraction(0)
    return float(t), int(q(t, out_scale))


def test_unfolded_batch_norm_by_hand():
    one = np.ones(1, np.float32)
    A = np.array([[10]], np.int8); B = np.array([[1]], np.int8)
    # 10 * 0.25 + 0.3 = 2.8 -> grid of step 1: 3.  var + eps = 3.75 + 0.25 = 4, sqrt 2, r = 0.5 (all exact):
    # (3 - 1.5) * 0.5 * 3 - 0.25 = 2.0
    kw = dict(scale=one * 0.25, bias=one * 0.3, mid_scale=1.0, mean=one * 1.5, var=one * 3.75, eps=0.25,
              gamma=one * 3, beta=one * -0.25)
    assert oracle.matmul_int8_bn(A, B, out_int8=False, **kw)[0, 0] == 2.0
    assert oracle.matmul_int8_bn(A, B, out_scale=0.5, **kw)[0, 0] == 4
    # mean above the value: (3 - 5) * 0.5 * 3 - 0.25 = -3.25; the ReLU comes after the batch norm
    kw["mean"] = one * 5
    assert oracle.matmul_int8_bn(A, B, out_int8=False, **kw)[0, 0] == -3.25
    assert oracle.matmul_int8_bn(A, B, out_int8=False, relu=True, **kw)[0, 0] == 0.0
    assert oracle.matmul_int8_bn(A, B, out_scale=0.25, relu=False, **kw)[0, 0] == -13


@pytest.mark.parametrize("seed", range(4))
def test_unfolded_batch_norm_matches_exact_rational_evaluation(seed):
    """Every operation of the figure evaluated in exact rational arithmetic and rounded once to binary32
    (the square root through an integer square root): an evaluation that shares nothing with the C code."""
    r = rng(40 + seed)
    m, n, k = 6, 5, 40
    A = i8(r, (m, k)); B = i8(r, (k, n))
    scale = (r.uniform(0.5, 2.0, n) * 5e-5).astype(np.float32)
    bias = r.normal(0, 0.5, n).astype(np.float32)
    mean = r.normal(0, 0.5, n).astype(np.float32); var = r.uniform(0.3, 3.0, n).astype(np.float32)
    gamma = r.uniform(0.5, 1.5, n).astype(np.float32); beta = r.normal(0, 0.3, n).astype(np.float32)
    eps, mid, out_scale = float(np.float32(1e-5)), float(np.float32(0.05)), float(np.float32(0.043))
    relu = bool(seed & 1)
    kw = dict(scale=scale, bias=bias, mid_scale=mid, mean=mean, var=var, eps=eps, gamma=gamma, beta=beta, relu=relu)
    codes = oracle.matmul_int8_bn(A, B, out_scale=out_scale, **kw)
    vals = oracle.matmul_int8_bn(A, B, out_int8=False, **kw)
    acc = A.astype(np.int64) @ B.astype(np.int64)
    for i in range(m):
        for j in range(n):
            t, c = exact_bn_epilogue(int(acc[i, j]), scale[j], bias[j], mid, mean[j], var[j], eps, gamma[j], beta[j],
                                     relu, out_scale)
            assert vals[i, j] == np.float32(t), (i, j)
            assert codes[i, j] == c, (i, j)
    assert len(np.unique(codes)) > 8


def test_unfolded_form_is_not_the_folded_one_and_reduces_to_it():
    r = rng(77)
    m, n, k = 64, 48, 200
    A = i8(r, (m, k)); B = i8(r, (k, n))
    scale = (r.uniform(0.5, 2.0, n) * 1e-3).astype(np.float32)
    mean = r.normal(0, 0.5, n).astype(np.float32); var = r.uniform(0.3, 3.0, n).astype(np.float32)
    gamma = r.uniform(0.5, 1.5, n).astype(np.float32); beta = r.normal(0, 0.3, n).astype(np.float32)
    eps = 1e-5
    lit = oracle.matmul_int8_bn(A, B, scale=scale, mean=mean, var=var, eps=eps, gamma=gamma, beta=beta, out_int8=False)
    # the caller-folded multiplier and shift give values that differ in the last place somewhere: the
    # unfolded entry really evaluates the figure's sequence
    rr = (np.float32(1) / np.sqrt(var + np.float32(eps))).astype(np.float32)
    mul = (rr * gamma).astype(np.float32); add = (beta - mean * mul).astype(np.float32)
    fold = oracle.matmul_int8(A, B, scale=scale, mul=mul, add=add, out_int8=False)
    assert np.any(lit != fold) and np.allclose(lit, fold, rtol=1e-5, atol=1e-6)
    # mean 0, var + eps = 1: r is exactly 1 and the unfolded form IS t * gamma + beta, the folded path's arithmetic
    zero = np.zeros(n, np.float32); onev = np.ones(n, np.float32)
    a = oracle.matmul_int8_bn(A, B, scale=scale, mean=zero, var=onev, eps=0.0, gamma=gamma, beta=beta, relu=True, out_scale=0.02)
    b = oracle.matmul_int8(A, B, scale=scale, mul=gamma, add=beta, relu=True, out_scale=0.02)
    assert np.array_equal(a, b)


def test_relu_keeps_nan_like_the_unordered_compare():
    # a NaN scale makes t NaN; "greater than zero or unordered" selects t
    A = np.array([[1], [-1]], np.int8); B = np.array([[1]], np.int8)
    f = oracle.matmul_int8(A, B, scale=np.array([np.nan], np.float32), relu=True, out_int8=False)
    assert np.isnan(f).all()
    f = oracle.matmul_int8(A, B, scale=np.ones(1, np.float32), relu=True, out_int8=False)
    assert f[:, 0].tolist() == [1.0, 0.0]


def test_conv_unfolded_batch_norm_uses_the_same_epilogue():
    r = rng(19)
    x = i8(r, (1, 6, 6, 8)); w = i8(r, (1, 1, 8, 5))
    kw = dict(scale=np.full(5, 2e-3, np.float32), bias=r.normal(size=5).astype(np.float32), mid_scale=0.1,
              mean=r.normal(size=5).astype(np.float32), var=r.uniform(0.5, 2, 5).astype(np.float32), eps=1e-5,
              gamma=r.uniform(0.5, 2, 5).astype(np.float32), beta=r.normal(size=5).astype(np.float32), relu=True, out_scale=0.05)
    c = oracle.conv2d_nhwc_int8_bn(x, w, **kw)
    m = oracle.matmul_int8_bn(x.reshape(36, 8), w.reshape(8, 5), **kw)
    assert np.array_equal(c.reshape(36, 5), m)
