"""Parity of the int8 path (through the C ABI) with the CPU oracle: integer
codes and fp32 outputs must be bit-exact."""
import numpy as np
import pytest

import workloads as wl
import pbk_testlib as T

pytestmark = pytest.mark.gpu

INT8, F32 = 5, 0


def params(n, variant, seed=0):
    """Epilogue parameter sets: 0 scale only; 1 +bias, ReLU; 2 +mul; 3 everything incl. the
    middle quantise/de-quantise pair (the paper's fused nest); 4 pair, no affine; 5 add only."""
    r = np.random.default_rng(1000 + seed + variant)
    scale = (r.uniform(0.5, 2.0, n) * 2e-4).astype(np.float32)
    bias = r.normal(0, 0.5, n).astype(np.float32) if variant in (1, 3) else None
    mid = {0: 0.0, 1: 0.0, 2: 0.0, 3: 0.031, 4: 0.07, 5: 0.0}[variant]
    mul = r.uniform(0.5, 1.5, n).astype(np.float32) if variant in (2, 3) else None
    add = r.normal(0, 0.3, n).astype(np.float32) if variant in (3, 5) else None
    relu = variant in (1, 3)
    return dict(scale=scale, bias=bias, mid_scale=mid, mul=mul, add=add, relu=relu, out_scale=0.043)


def dev_or_none(a):
    return None if a is None else T.to_device(a)


def run_matmul(A, B, q, trans_b, out_int8, force=None, lda=None, ldb=None):
    import torch
    import paper_2603_06731_amd as pbk
    m, k = A.shape
    n = B.shape[0] if trans_b else B.shape[1]
    dA = torch.from_numpy(A).cuda(); dB = torch.from_numpy(B).cuda()
    out = torch.empty(m * n, dtype=torch.int8 if out_int8 else torch.float32, device="cuda")
    d = {k2: dev_or_none(v) if isinstance(v, np.ndarray) else v for k2, v in q.items()}
    with T.forced_kernel(force):
        st = pbk.pbk_matmul_int8(dA, dB, out, m, n, k, lda or k, ldb or B.shape[1], n, trans_b, d["scale"], d["bias"],
                                 q["mid_scale"], d["mul"], d["add"], q["relu"], q["out_scale"],
                                 INT8 if out_int8 else F32, None)
    assert st == 0, pbk.pbk_status_string(st)
    return out.cpu().numpy().reshape(m, n), pbk.pbk_last_kernel()


SHAPES = [(300, 264, 208), (256, 256, 64), (520, 136, 80), (33, 520, 144), (64, 8, 16), (130, 260, 4096)]


@pytest.mark.parametrize("cfg", [None, 0, 1, 4, 8, 9, "generic"])
@pytest.mark.parametrize("mnk", SHAPES)
def test_matmul_int8_kmajor(cfg, mnk):
    import oracle
    m, n, k = mnk
    A = wl.int8_tensor((m, k), 1); B = wl.int8_tensor((n, k), 2)
    q = params(n, 3)
    force = None if cfg is None else ("generic" if cfg == "generic" else f"mfma:{cfg}")
    got, kern = run_matmul(A, B, q, 1, True, force)
    want = oracle.matmul_int8(A, B, trans_b=1, **q)
    print(f"int8 {mnk} force={force} kernel={kern} codes={len(np.unique(want))}", flush=True)
    assert ("generic" in kern) == (cfg == "generic")
    assert np.array_equal(got, want)


@pytest.mark.parametrize("k", [16, 64, 80, 128, 144, 192, 256, 272, 320, 400, 448, 528, 656, 2192])
def test_matmul_int8_pair_pipeline_k_sweep(k):
    """Both operands staged 128 values deep, one barrier per pair of 64-value k-tiles: prologue only, drain
    only, odd and even tile counts, ragged last tiles, the paired steady state."""
    import oracle
    m, n = 300, 517
    A = wl.int8_tensor((m, k), 1); B = wl.int8_tensor((n, k), 2)
    q = params(n, 3)
    got, kern = run_matmul(A, B, q, 1, True, "mfma:9")
    assert "pair" in kern, kern
    assert np.array_equal(got, oracle.matmul_int8(A, B, trans_b=1, **q))


@pytest.mark.parametrize("variant", range(6))
@pytest.mark.parametrize("out_int8", [True, False])
@pytest.mark.parametrize("force", [None, "generic"])
def test_matmul_int8_epilogue_variants(variant, out_int8, force):
    import oracle
    m, n, k = 200, 264, 304
    A = wl.int8_tensor((m, k), 1, "normal", 40.0); B = wl.int8_tensor((n, k), 2, "normal", 30.0)
    q = params(n, variant)
    got, kern = run_matmul(A, B, q, 1, out_int8, force)
    want = oracle.matmul_int8(A, B, trans_b=1, out_int8=out_int8, **q)
    assert got.dtype == want.dtype
    assert np.array_equal(got.view(np.uint8 if out_int8 else np.uint32), want.view(np.uint8 if out_int8 else np.uint32)), kern


def test_matmul_int8_row_major_b_runs_generic():
    import oracle
    m, n, k = 70, 50, 90
    A = wl.int8_tensor((m, k), 1); B = wl.int8_tensor((k, n), 2)
    q = params(n, 1)
    got, kern = run_matmul(A, B, q, 0, True)
    assert "generic" in kern
    assert np.array_equal(got, oracle.matmul_int8(A, B, trans_b=0, **q))


@pytest.mark.parametrize("cfg", [None, 0, 1, 4, 8, 9])
@pytest.mark.parametrize("mnk", [(300, 272, 208), (256, 512, 128), (33, 144, 4096)])
def test_matmul_int8_row_major_b_on_mfma(cfg, mnk):
    """Row-major B: the n-major byte tile is read with the 8-bit transposing LDS read."""
    import oracle
    m, n, k = mnk
    A = wl.int8_tensor((m, k), 1); B = wl.int8_tensor((k, n), 2)
    q = params(n, 3)
    got, kern = run_matmul(A, B, q, 0, True, None if cfg is None else f"mfma:{cfg}")
    assert "mfma" in kern
    assert np.array_equal(got, oracle.matmul_int8(A, B, trans_b=0, **q))


@pytest.mark.parametrize("cfg", [None, 0, 1, 4])
@pytest.mark.parametrize("geom", [((1, 1), (1, 1), (1, 1)), ((2, 2), (1, 1), (1, 1)), ((1, 2), (2, 0), (2, 1))])
def test_conv_int8_on_mfma(cfg, geom):
    """The paper's quantised example is a convolution: channels multiples of 16 run on the matrix units."""
    import torch
    import oracle
    import paper_2603_06731_amd as pbk
    stride, pad, dil = geom
    n, H, W, Cin, Cout, KH, KW = 2, 15, 14, 32, 48, 3, 3
    x = wl.int8_tensor((n, H, W, Cin), 1, "normal", 40.0); w = wl.int8_tensor((KH, KW, Cin, Cout), 2, "normal", 30.0)
    q = params(Cout, 3)
    want = oracle.conv2d_nhwc_int8(x, w, stride=stride, pad=pad, dil=dil, **q)
    out = torch.empty(want.size, dtype=torch.int8, device="cuda")
    d = {k2: dev_or_none(v) if isinstance(v, np.ndarray) else v for k2, v in q.items()}
    with T.forced_kernel(None if cfg is None else f"mfma:{cfg}"):
        st = pbk.pbk_conv2d_nhwc_int8(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), out, n, H, W, Cin, Cout,
                                      KH, KW, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1], d["scale"], d["bias"],
                                      q["mid_scale"], d["mul"], d["add"], q["relu"], q["out_scale"], INT8, None)
    assert st == 0, pbk.pbk_status_string(st)
    assert "mfma" in pbk.pbk_last_kernel()
    assert np.array_equal(out.cpu().numpy().reshape(want.shape), want)


def test_matmul_int8_extreme_values_and_saturation():
    import oracle
    m, n, k = 128, 256, 8192
    A = np.full((m, k), -128, np.int8); B = np.full((n, k), -128, np.int8)
    B[::2] = 127
    q = dict(scale=np.full(n, 1e-6, np.float32), bias=None, mid_scale=0.0, mul=None, add=None, relu=False, out_scale=0.5)
    got, kern = run_matmul(A, B, q, 1, True)
    want, acc = oracle.matmul_int8(A, B, trans_b=1, want_acc=True, **q)
    assert acc.max() == k * 16384 and "mfma" in kern
    assert np.array_equal(got, want) and got.max() == 127 and got.min() == -128
    gotf, _ = run_matmul(A, B, q, 1, False)
    assert np.array_equal(gotf, oracle.matmul_int8(A, B, trans_b=1, out_int8=False, **q))


def test_matmul_int8_views():
    """Leading dimensions larger than K: bytes outside the views must not matter."""
    import oracle
    m, n, k, ld = 140, 136, 96, 128
    r = np.random.default_rng(3)
    Ap = r.integers(-128, 128, size=(m, ld), dtype=np.int8); Bp = r.integers(-128, 128, size=(n, ld), dtype=np.int8)
    q = params(n, 3)
    import torch
    import paper_2603_06731_amd as pbk
    dA = torch.from_numpy(Ap).cuda(); dB = torch.from_numpy(Bp).cuda()
    out = torch.empty(m * n, dtype=torch.int8, device="cuda")
    d = {k2: dev_or_none(v) if isinstance(v, np.ndarray) else v for k2, v in q.items()}
    st = pbk.pbk_matmul_int8(dA, dB, out, m, n, k, ld, ld, n, 1, d["scale"], d["bias"], q["mid_scale"], d["mul"],
                             d["add"], q["relu"], q["out_scale"], INT8, None)
    assert st == 0 and "mfma" in pbk.pbk_last_kernel()
    want = oracle.matmul_int8(np.ascontiguousarray(Ap[:, :k]), np.ascontiguousarray(Bp[:, :k]), trans_b=1, **q)
    assert np.array_equal(out.cpu().numpy().reshape(m, n), want)


@pytest.mark.parametrize("geom", [((1, 1), (1, 1), (1, 1)), ((2, 2), (1, 1), (1, 1)), ((1, 2), (2, 0), (2, 1))])
@pytest.mark.parametrize("out_int8", [True, False])
def test_conv_int8(geom, out_int8):
    import torch
    import oracle
    import paper_2603_06731_amd as pbk
    stride, pad, dil = geom
    n, H, W, Cin, Cout, KH, KW = 2, 14, 13, 16, 24, 3, 3
    x = wl.int8_tensor((n, H, W, Cin), 1, "normal", 40.0); w = wl.int8_tensor((KH, KW, Cin, Cout), 2, "normal", 30.0)
    q = params(Cout, 3)
    want = oracle.conv2d_nhwc_int8(x, w, stride=stride, pad=pad, dil=dil, out_int8=out_int8, **q)
    out = torch.empty(want.size, dtype=torch.int8 if out_int8 else torch.float32, device="cuda")
    d = {k2: dev_or_none(v) if isinstance(v, np.ndarray) else v for k2, v in q.items()}
    st = pbk.pbk_conv2d_nhwc_int8(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), out, n, H, W, Cin, Cout,
                                  KH, KW, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1], d["scale"], d["bias"],
                                  q["mid_scale"], d["mul"], d["add"], q["relu"], q["out_scale"],
                                  INT8 if out_int8 else F32, None)
    assert st == 0, pbk.pbk_status_string(st)
    got = out.cpu().numpy().reshape(want.shape)
    assert np.array_equal(got, want)


def test_matmul_int8_full_size_sampled_rows():
    """8192^3 in the bench's configuration; whole rows of the output against the oracle."""
    import oracle
    m = n = k = 8192
    A = wl.int8_tensor((m, k), 1, "normal", 40.0); B = wl.int8_tensor((n, k), 2, "normal", 30.0)
    q = params(n, 3)
    q["scale"] = (q["scale"] * 0.05).astype(np.float32)
    got, kern = run_matmul(A, B, q, 1, True)
    rows = np.array([0, 1, 127, 128, 4095, 4096, 8191, 777, 2301, 6000])
    want = oracle.matmul_int8(np.ascontiguousarray(A[rows]), B, trans_b=1, **q)
    print(f"int8 8192^3 kernel={kern} codes={len(np.unique(want))}", flush=True)
    assert "256x256" in kern
    assert np.array_equal(got[rows], want) and len(np.unique(want)) > 50


# ------------------------------------------- the batch-norm step unfolded, as in the paper's figure

def bn_params(n, seed=0, relu=True, mid=0.031):
    r = np.random.default_rng(2000 + seed)
    return dict(scale=(r.uniform(0.5, 2.0, n) * 2e-4).astype(np.float32), bias=r.normal(0, 0.5, n).astype(np.float32),
                mid_scale=mid, mean=r.normal(0, 0.5, n).astype(np.float32), var=r.uniform(0.3, 3.0, n).astype(np.float32),
                eps=1e-5, gamma=r.uniform(0.5, 1.5, n).astype(np.float32), beta=r.normal(0, 0.3, n).astype(np.float32),
                relu=relu, out_scale=0.043)


@pytest.mark.parametrize("force", [None, "mfma:1", "mfma:4", "mfma:8", "generic"])
@pytest.mark.parametrize("out_int8", [True, False])
@pytest.mark.parametrize("mnk", [(300, 264, 208), (130, 272, 4096)])
def test_matmul_int8_unfolded_batch_norm_is_bit_exact(force, out_int8, mnk):
    import torch
    import oracle
    import paper_2603_06731_amd as pbk
    m, n, k = mnk
    A = wl.int8_tensor((m, k), 1, "normal", 40.0); B = wl.int8_tensor((n, k), 2, "normal", 30.0)
    q = bn_params(n, seed=m)
    d = {k2: dev_or_none(v) if isinstance(v, np.ndarray) else v for k2, v in q.items()}
    out = torch.empty(m * n, dtype=torch.int8 if out_int8 else torch.float32, device="cuda")
    with T.forced_kernel(force):
        st = pbk.pbk_matmul_int8_bn(torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda(), out, m, n, k, k, k, n, 1,
                                    d["scale"], d["bias"], q["mid_scale"], d["mean"], d["var"], q["eps"], d["gamma"], d["beta"],
                                    q["relu"], q["out_scale"], INT8 if out_int8 else F32, None)
    assert st == 0, pbk.pbk_status_string(st)
    want = oracle.matmul_int8_bn(A, B, trans_b=1, out_int8=out_int8, **q)
    got = out.cpu().numpy().reshape(m, n)
    view = np.uint8 if out_int8 else np.uint32
    assert np.array_equal(got.view(view), want.view(view)), pbk.pbk_last_kernel()
    if out_int8:
        assert len(np.unique(want)) > 40
    # and it is not the folded form: the caller-folded parameters give other bits somewhere
    if not out_int8:
        rr = (np.float32(1) / np.sqrt(q["var"] + np.float32(q["eps"]))).astype(np.float32)
        mul = (rr * q["gamma"]).astype(np.float32); add = (q["beta"] - q["mean"] * mul).astype(np.float32)
        folded = oracle.matmul_int8(A, B, trans_b=1, out_int8=False, scale=q["scale"], bias=q["bias"],
                                    mid_scale=q["mid_scale"], mul=mul, add=add, relu=q["relu"])
        assert np.any(folded != want)


@pytest.mark.parametrize("force", [None, "generic"])
def test_conv_int8_unfolded_batch_norm_is_bit_exact(force):
    import torch
    import oracle
    import paper_2603_06731_amd as pbk
    n, H, W, Cin, Cout = 2, 14, 13, 32, 48
    x = wl.int8_tensor((n, H, W, Cin), 1, "normal", 40.0); w = wl.int8_tensor((3, 3, Cin, Cout), 2, "normal", 30.0)
    q = bn_params(Cout, seed=5)
    d = {k2: dev_or_none(v) if isinstance(v, np.ndarray) else v for k2, v in q.items()}
    out = torch.empty(n * H * W * Cout, dtype=torch.int8, device="cuda")
    with T.forced_kernel(force):
        st = pbk.pbk_conv2d_nhwc_int8_bn(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), out, n, H, W, Cin, Cout,
                                         3, 3, 1, 1, 1, 1, 1, 1, d["scale"], d["bias"], q["mid_scale"], d["mean"], d["var"],
                                         q["eps"], d["gamma"], d["beta"], q["relu"], q["out_scale"], INT8, None)
    assert st == 0, pbk.pbk_status_string(st)
    want = oracle.conv2d_nhwc_int8_bn(x, w, pad=(1, 1), **q)
    assert np.array_equal(out.cpu().numpy().reshape(want.shape), want), pbk.pbk_last_kernel()


@pytest.mark.parametrize("force", [None, "generic"])
def test_int8_relu_keeps_nan(force):
    """A NaN de-quantisation scale makes a column NaN; the ReLU (greater or unordered) keeps it."""
    import torch
    import oracle
    import paper_2603_06731_amd as pbk
    m, n, k = 64, 32, 64
    A = wl.int8_tensor((m, k), 1); B = wl.int8_tensor((n, k), 2)
    scale = np.full(n, 1e-3, np.float32); scale[5] = np.nan
    out = torch.empty(m * n, dtype=torch.float32, device="cuda")
    with T.forced_kernel(force):
        st = pbk.pbk_matmul_int8(torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda(), out, m, n, k, k, k, n, 1,
                                 T.to_device(scale), None, 0.0, None, None, 1, 1.0, F32, None)
    assert st == 0
    got = out.cpu().numpy().reshape(m, n)
    want = oracle.matmul_int8(A, B, trans_b=1, scale=scale, relu=True, out_int8=False)
    assert np.isnan(got[:, 5]).all() and np.isnan(want[:, 5]).all()
    keep = np.ones(n, bool); keep[5] = False
    assert np.array_equal(got[:, keep], want[:, keep])


@pytest.mark.parametrize("chan", [(32, 48), (64, 272), (24, 20)])
@pytest.mark.parametrize("out_int8", [True, False])
def test_pointwise_conv_int8_runs_as_the_plain_matmul(chan, out_int8):
    """A 1x1 filter at stride 1 without padding goes to the plain-matrix int8 kernels (channel counts that are
    multiples of 16: the matrix units; others: the generic kernel) and stays bit-exact with the convolution oracle."""
    import torch
    import oracle
    import paper_2603_06731_amd as pbk
    Cin, Cout = chan
    n, H, W = 3, 11, 13
    x = wl.int8_tensor((n, H, W, Cin), 1, "normal", 40.0); w = wl.int8_tensor((1, 1, Cin, Cout), 2, "normal", 30.0)
    q = params(Cout, 3)
    want = oracle.conv2d_nhwc_int8(x, w, stride=(1, 1), pad=(0, 0), dil=(1, 1), out_int8=out_int8, **q)
    out = torch.empty(want.size, dtype=torch.int8 if out_int8 else torch.float32, device="cuda")
    d = {k2: dev_or_none(v) if isinstance(v, np.ndarray) else v for k2, v in q.items()}
    st = pbk.pbk_conv2d_nhwc_int8(torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda(), out, n, H, W, Cin, Cout,
                                  1, 1, 1, 1, 0, 0, 1, 1, d["scale"], d["bias"], q["mid_scale"], d["mul"], d["add"],
                                  q["relu"], q["out_scale"], INT8 if out_int8 else F32, None)
    assert st == 0, pbk.pbk_status_string(st)
    assert ("mfma" in pbk.pbk_last_kernel()) == (Cin % 16 == 0 and Cout % 16 == 0), pbk.pbk_last_kernel()
    assert np.array_equal(out.cpu().numpy().reshape(want.shape), want)
