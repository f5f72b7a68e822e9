"""Pins for the oracle's convolution variants: four-sided padding and the
transposed convolution.  Library routines (torch float64), the adjoint
identity against the already pinned convolution oracle, closed forms and a
plain Python loop.  None of these tests touches the HIP library."""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

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


# --------------------------------------------------------- four-sided padding

@pytest.mark.parametrize("pad", [(0, 1, 0, 1), (2, 0, 1, 3), (1, 1, 1, 1), (0, 0, 2, 0)])
@pytest.mark.parametrize("stride,dil", [((1, 1), (1, 1)), ((2, 2), (1, 1)), ((2, 1), (1, 2))])
def test_pad4_equals_convolution_of_explicitly_padded_image(pad, stride, dil):
    r = rng(sum(pad) + stride[0])
    x = r.integers(-4, 5, size=(2, 7, 8, 3)).astype(np.float64)
    w = r.integers(-3, 4, size=(3, 2, 3, 4)).astype(np.float64)
    got = oracle.conv2d_nhwc_pad4(as_dtype(x, F32), as_dtype(w, F32), dtype=F32, stride=stride, pad=pad, dil=dil)
    xp = np.pad(x, ((0, 0), (pad[0], pad[1]), (pad[2], pad[3]), (0, 0)))
    want = oracle.conv2d_nhwc(as_dtype(xp, F32), as_dtype(w, F32), dtype=F32, stride=stride, pad=(0, 0), dil=dil)
    assert got.shape == want.shape and np.array_equal(got, want)
    # and torch on the padded image
    t = F.conv2d(torch.from_numpy(xp).permute(0, 3, 1, 2), torch.from_numpy(w).permute(3, 2, 0, 1),
                 stride=stride, dilation=dil).permute(0, 2, 3, 1).numpy()
    assert np.array_equal(got, t)


def test_pad4_same_padding_of_a_stride_2_layer():
    # the "same" rule of the frameworks for H = 8, K = 3, stride 2: total padding 1, all of it at the far side
    x = np.ones((1, 8, 8, 1)); w = np.ones((3, 3, 1, 1))
    got = oracle.conv2d_nhwc_pad4(as_dtype(x, F32), as_dtype(w, F32), dtype=F32, stride=(2, 2), pad=(0, 1, 0, 1))
    assert got.shape == (1, 4, 4, 1)
    assert got[0, 0, 0, 0] == 9 and got[0, 3, 3, 0] == 4 and got[0, 3, 0, 0] == 6 and got[0, 0, 3, 0] == 6


def test_pad4_symmetric_is_the_plain_entry():
    r = rng(4)
    x = as_dtype(r.normal(size=(1, 6, 5, 4)), BF16); w = as_dtype(r.normal(size=(3, 3, 4, 2)), BF16)
    b = r.normal(size=2).astype(np.float32)
    a = oracle.conv2d_nhwc_pad4(x, w, b, dtype=BF16, stride=(2, 1), pad=(1, 1, 2, 2), dil=(1, 1), alpha=0.5, epi=3)
    c = oracle.conv2d_nhwc(x, w, b, dtype=BF16, stride=(2, 1), pad=(1, 2), dil=(1, 1), alpha=0.5, epi=3)
    assert np.array_equal(a, c)


# ------------------------------------------------------ transposed convolution

GEOMS = [  # (H, W, KH, KW, stride, pad, out_pad, dil)
    (5, 6, 3, 3, (1, 1), (0, 0), (0, 0), (1, 1)),
    (5, 6, 3, 3, (2, 2), (1, 1), (1, 1), (1, 1)),
    (4, 7, 2, 4, (3, 2), (0, 1), (2, 0), (1, 1)),
    (6, 5, 3, 2, (2, 1), (2, 0), (0, 0), (2, 3)),
    (3, 3, 1, 1, (2, 2), (0, 0), (1, 1), (1, 1)),
    (7, 4, 4, 4, (2, 2), (1, 1), (0, 0), (1, 1)),
]


@pytest.mark.parametrize("dtype", [F32, BF16, F16])
@pytest.mark.parametrize("geom", GEOMS)
def test_transpose_against_torch_float64(dtype, geom):
    H, W, KH, KW, stride, pad, out_pad, dil = geom
    r = rng(H * 10 + KW)
    x = r.normal(size=(2, H, W, 3)); w = r.normal(size=(KH, KW, 3, 5))
    got = oracle.conv2d_transpose_nhwc(as_dtype(x, dtype), as_dtype(w, dtype), dtype=dtype, stride=stride,
                                       pad=pad, out_pad=out_pad, dil=dil)
    tx = torch.from_numpy(widened(x, dtype)).permute(0, 3, 1, 2)
    tw = torch.from_numpy(widened(w, dtype)).permute(2, 3, 0, 1)          # [Cin][Cout][KH][KW]
    want = F.conv_transpose2d(tx, tw, stride=stride, padding=pad, output_padding=out_pad,
                              dilation=dil).permute(0, 2, 3, 1).numpy()
    assert got.shape == want.shape
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("geom", GEOMS)
def test_transpose_is_the_adjoint_of_the_pinned_convolution(geom):
    """<conv(u, w), y> == <u, conv_transpose(y, w')> with w' = w with its channel axes
    swapped: ties the scatter definition to the convolution oracle pinned elsewhere."""
    H, W, KH, KW, stride, pad, out_pad, dil = geom
    r = rng(7)
    cy, cu = 3, 4
    y = r.integers(-3, 4, size=(1, H, W, cy)).astype(np.float64)
    w = r.integers(-2, 3, size=(KH, KW, cy, cu)).astype(np.float64)       # transposed conv: cy -> cu
    t = oracle.conv2d_transpose_nhwc(as_dtype(y, F32), as_dtype(w, F32), dtype=F32, stride=stride, pad=pad,
                                     out_pad=out_pad, dil=dil)
    u = r.integers(-3, 4, size=t.shape).astype(np.float64)
    wf = np.ascontiguousarray(w.transpose(0, 1, 3, 2))                      # forward conv: cu -> cy
    fwd = oracle.conv2d_nhwc(as_dtype(u, F32), as_dtype(wf, F32), dtype=F32, stride=stride, pad=pad, dil=dil)
    # the forward convolution of an image of the transposed output's size gives back (at least) H x W
    assert fwd.shape[1] >= H and fwd.shape[2] >= W
    lhs = float((fwd[:, :H, :W, :] * y).sum())
    rhs = float((u * t).sum())
    assert lhs == rhs                                                       # small integers: exact


def test_transpose_closed_forms():
    # a single input pixel paints the filter into the output at (ih*s - p, iw*s - p)
    w = rng(1).integers(1, 9, size=(3, 3, 1, 2)).astype(np.float64)
    x = np.zeros((1, 4, 4, 1)); x[0, 1, 2, 0] = 2.0
    out = oracle.conv2d_transpose_nhwc(as_dtype(x, F32), as_dtype(w, F32), dtype=F32, stride=(2, 2))
    assert out.shape == (1, 9, 9, 2)
    want = np.zeros_like(out); want[0, 2:5, 4:7, :] = 2.0 * w[:, :, 0, :]
    assert np.array_equal(out, want)
    # stride 1, no padding: the full correlation = convolution with the filter rotated by 180 degrees
    r = rng(2)
    x = r.integers(-3, 4, size=(1, 5, 5, 2)).astype(np.float64)
    w = r.integers(-3, 4, size=(3, 3, 2, 2)).astype(np.float64)
    t = oracle.conv2d_transpose_nhwc(as_dtype(x, F32), as_dtype(w, F32), dtype=F32)
    wrot = np.ascontiguousarray(w[::-1, ::-1])
    c = oracle.conv2d_nhwc(as_dtype(x, F32), as_dtype(wrot, F32), dtype=F32, pad=(2, 2))
    assert np.array_equal(t, c)
    # 1x1 filter, stride 2: the input lands on the even grid, zeros elsewhere (out_pad adds an empty row/column)
    x = r.integers(1, 5, size=(1, 3, 3, 1)).astype(np.float64)
    t = oracle.conv2d_transpose_nhwc(as_dtype(x, F32), as_dtype(np.ones((1, 1, 1, 1)), F32), dtype=F32,
                                     stride=(2, 2), out_pad=(1, 1))
    assert t.shape == (1, 6, 6, 1)
    assert np.array_equal(t[0, ::2, ::2, 0], x[0, :, :, 0]) and t[0, 1::2].sum() == 0 and t[0, :, 1::2].sum() == 0


def test_transpose_epilogue_and_sampled_variant():
    r = rng(3)
    x = as_dtype(r.normal(size=(2, 5, 4, 3)), BF16); w = as_dtype(r.normal(size=(3, 2, 3, 4)), BF16)
    b = r.normal(size=4).astype(np.float32)
    kw = dict(dtype=BF16, stride=(2, 3), pad=(1, 0), out_pad=(1, 2), dil=(1, 2), alpha=0.5, epi=3)
    full, pre = oracle.conv2d_transpose_nhwc(x, w, b, want_preact=True, **kw)
    plain = oracle.conv2d_transpose_nhwc(x, w, dtype=BF16, stride=(2, 3), pad=(1, 0), out_pad=(1, 2), dil=(1, 2))
    np.testing.assert_allclose(pre, 0.5 * plain + b.astype(np.float64), rtol=1e-15, atol=1e-15)
    assert np.array_equal(full, np.maximum(pre, 0.0))
    idx = list(itertools.product(range(2), range(full.shape[1]), range(full.shape[2]), range(4)))
    sn, soh, sow, sco = (np.array(c) for c in zip(*idx))
    at, at_pre = oracle.conv2d_transpose_nhwc_at(x, w, b, sn, soh, sow, sco, **kw)
    np.testing.assert_allclose(at.reshape(full.shape), full, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(at_pre.reshape(full.shape), pre, rtol=1e-13, atol=1e-14)


def test_transpose_output_size_rule():
    assert oracle.conv_transpose_out_dim(5, 3, 2, 1, 1, 1) == 10
    assert oracle.conv_transpose_out_dim(4, 4, 2, 1, 0, 1) == 8
    assert oracle.conv_transpose_out_dim(1, 1, 1, 0, 0, 1) == 1
    assert oracle.conv_transpose_out_dim(5, 3, 2, 1, 2, 1) == -1      # out_pad must stay below stride or dilation
    assert oracle.conv_transpose_out_dim(1, 1, 1, 1, 0, 1) == -1      # empty
    # inverse of the convolution's size rule: conv_out(transpose_out(n)) == n
    for n, k, s, p, d in [(5, 3, 2, 1, 1), (7, 4, 3, 2, 1), (4, 3, 1, 0, 2)]:
        o = oracle.conv_transpose_out_dim(n, k, s, p, 0, d)
        assert oracle.conv_out_dim(o, k, s, p, d) == n
