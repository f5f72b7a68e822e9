"""Parity of the fused attention kernels (through the C ABI) with the CPU
oracle.  Small cases are compared element by element; the paper-sized shapes
on sampled rows the oracle computes one by one."""
import numpy as np
import pytest

import workloads as wl
import pbk_testlib as T

pytestmark = pytest.mark.gpu

BF16, F16, F32 = wl.DTYPE_BF16, wl.DTYPE_F16, wl.DTYPE_F32

# 16-bit path: the weights are rounded to the 16-bit type before they multiply V
# (relative 2^-9 for bf16, 2^-12 for fp16, averaging out over the keys) and the
# output is rounded once (2^-9 / 2^-12 of its magnitude, which can be a few times
# the RMS the error is measured against): bound asserted besides the contract's 2e-2.
ATT_TIGHT = {BF16: 1.2e-2, F16: 2e-3, F32: 1e-5}


def tol_for(dtype):
    return T.TOL_F32 if dtype == F32 else T.TOL_16BIT


def check_attention(w, force=None, expect_kernel=None):
    import paper_2603_06731_amd as pbk
    host = wl.make_attention_inputs(w)
    dev = T.upload(host)
    with T.forced_kernel(force):
        st, out = T.run_attention(w, dev)
    assert st == 0, pbk.pbk_status_string(st)
    if expect_kernel:
        assert expect_kernel in pbk.pbk_last_kernel(), pbk.pbk_last_kernel()
    ref = T.oracle_attention_full(w, host)
    got = T.to_host_f64(out, w.dtype).reshape(ref.shape)
    err = T.rel_err(got, ref, ref)
    print(f"{w.name} force={force} kernel={pbk.pbk_last_kernel()} err={err:.3e}", flush=True)
    assert err <= tol_for(w.dtype), (w.name, force, err)
    assert err <= ATT_TIGHT[w.dtype], (w.name, force, err)
    return err


def scale(d):
    return float(np.float32(1.0 / np.sqrt(d)))


# (batch, Nq, Nk, D): several query tiles and key tiles, ragged tails in both, tiny cases
SMALL = [
    (2, 128, 64, 64),
    (3, 200, 300, 64),
    (1, 577, 577, 64),
    (2, 10, 10, 64),
    (1, 1, 1, 32),
    (2, 130, 129, 128),
    (1, 256, 63, 128),
    (2, 297, 65, 32),
    (1, 33, 500, 32),
]


@pytest.mark.parametrize("dtype", [BF16, F16])
@pytest.mark.parametrize("shape", SMALL)
def test_attention_mfma_small(dtype, shape):
    b, nq, nk, d = shape
    w = wl.AttentionWorkload(f"att_{b}x{nq}x{nk}x{d}", dtype, b, nq, nk, d, alpha=scale(d))
    check_attention(w, expect_kernel="attn_mfma")


@pytest.mark.parametrize("bias", ["shared", "per_batch"])
@pytest.mark.parametrize("shape", [(2, 200, 300, 64), (2, 130, 129, 128), (3, 70, 37, 32)])
def test_attention_mfma_bias(bias, shape):
    b, nq, nk, d = shape
    w = wl.AttentionWorkload(f"att_bias_{bias}", BF16, b, nq, nk, d, alpha=scale(d), bias=bias)
    check_attention(w, expect_kernel="attn_mfma")


@pytest.mark.parametrize("dtype", [F32, BF16, F16])
@pytest.mark.parametrize("shape", [(2, 50, 300, 64), (1, 17, 513, 40), (2, 9, 5, 3), (1, 3, 70, 200)])
@pytest.mark.parametrize("bias", ["none", "per_batch"])
def test_attention_generic(dtype, shape, bias):
    b, nq, nk, d = shape
    w = wl.AttentionWorkload("att_generic", dtype, b, nq, nk, d, alpha=scale(d), bias=bias)
    check_attention(w, force="generic", expect_kernel="attn_generic")


@pytest.mark.parametrize("alpha", [0.0, -0.3])
def test_attention_mfma_nonpositive_scale(alpha):
    """alpha <= 0 takes the kernel variant that scales the scores before the row maximum."""
    w = wl.AttentionWorkload("att_alpha", BF16, 2, 150, 200, 64, alpha=alpha)
    check_attention(w, expect_kernel="attn_mfma")


def test_attention_odd_head_size_falls_back():
    w = wl.AttentionWorkload("att_d40", BF16, 2, 100, 90, 40, alpha=scale(40))
    check_attention(w, expect_kernel="attn_generic")


def test_attention_large_scores_are_stable():
    # scores of a few hundred: exp() of them would overflow fp32 without the running maximum
    w = wl.AttentionWorkload("att_sharp", BF16, 2, 150, 260, 64, alpha=4.0,
                             dist_q=("normal", 3.0), dist_k=("normal", 3.0))
    check_attention(w, expect_kernel="attn_mfma")
    check_attention(w, force="generic")


@pytest.mark.parametrize("force", [None, "generic"])
def test_attention_causal_mask_through_bias(force):
    import paper_2603_06731_amd as pbk
    import oracle
    b, n, d = 2, 200, 64
    w = wl.AttentionWorkload("att_causal", BF16, b, n, n, d, alpha=scale(d), bias="shared")
    host = wl.make_attention_inputs(w)
    host["bias"] = np.where(np.arange(n)[None, :] <= np.arange(n)[:, None], 0.0, -np.inf).astype(np.float32)
    dev = T.upload(host)
    with T.forced_kernel(force):
        st, out = T.run_attention(w, dev)
    assert st == 0, pbk.pbk_status_string(st)
    ref = oracle.attention(host["q"], host["k"], host["v"], host["bias"], dtype=BF16, alpha=w.alpha)
    got = T.to_host_f64(out, BF16).reshape(ref.shape)
    err = T.rel_err(got, ref, ref)
    print(f"causal force={force} kernel={pbk.pbk_last_kernel()} err={err:.3e}", flush=True)
    assert err <= ATT_TIGHT[BF16]
    # row 0 sees key 0 only: exactly V[0] (already a bf16 value)
    v0 = wl.widen(host["v"][:, 0, :], BF16)
    assert np.array_equal(got[:, 0, :], v0)


# (batch, Nq, Nk, D) with Nk >= Nq: every row sees at least one key
CAUSAL_SHAPES = [
    (2, 128, 128, 64),
    (3, 200, 300, 64),
    (1, 577, 577, 64),
    (2, 10, 10, 64),
    (1, 1, 1, 32),
    (2, 130, 131, 128),
    (1, 256, 256, 128),
    (2, 297, 400, 32),
    (1, 33, 500, 32),
    (1, 1, 700, 64),         # one query at the end of a long context: sees every key
]


@pytest.mark.parametrize("dtype", [BF16, F16])
@pytest.mark.parametrize("shape", CAUSAL_SHAPES)
def test_attention_causal_mfma(dtype, shape):
    b, nq, nk, d = shape
    w = wl.AttentionWorkload(f"att_causal_{b}x{nq}x{nk}x{d}", dtype, b, nq, nk, d, alpha=scale(d), causal=True)
    check_attention(w, expect_kernel="causal")


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("nk", [159, 160, 161, 223, 224, 225, 287, 288, 289, 352])
def test_attention_interior_loop_boundaries(nk, causal):
    """The kernel walks its leading 64-key tiles in a loop body without range tests and the rest in the
    general one; the first tile that needs a test depends on Nk (the next tile's loads must lie inside) and,
    for the causal form, on the wave's first query.  Key counts on both sides of every such boundary."""
    w = wl.AttentionWorkload(f"att_edge_{nk}", BF16, 2, 150, nk, 64, alpha=scale(64), causal=causal)
    check_attention(w, expect_kernel="causal" if causal else "attn_mfma")


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("shape", [(2, 50, 300, 64), (1, 17, 513, 40), (2, 9, 9, 3), (1, 70, 70, 200)])
def test_attention_causal_generic(dtype, shape):
    b, nq, nk, d = shape
    w = wl.AttentionWorkload("att_causal_generic", dtype, b, nq, nk, d, alpha=scale(d), causal=True)
    check_attention(w, force="generic", expect_kernel="attn_generic")


def test_attention_causal_first_row_is_the_first_value_and_equals_the_masked_bias_form():
    import torch
    import paper_2603_06731_amd as pbk
    b, n, d = 2, 333, 64
    w = wl.AttentionWorkload("att_causal_row0", BF16, b, n, n, d, alpha=scale(d), causal=True)
    host = wl.make_attention_inputs(w)
    dev = T.upload(host)
    st, out = T.run_attention(w, dev)
    assert st == 0 and "causal" in pbk.pbk_last_kernel()
    got = T.to_host_f64(out, BF16).reshape(b, n, d)
    assert np.array_equal(got[:, 0, :], wl.widen(host["v"][:, 0, :], BF16))
    # the same mask given as a bias of -inf: the two kernels agree to the rounding of the output
    wb = wl.AttentionWorkload("att_causal_bias", BF16, b, n, n, d, alpha=scale(d), bias="shared")
    hb = dict(host)
    hb["bias"] = np.where(np.arange(n)[None, :] <= np.arange(n)[:, None], 0.0, -np.inf).astype(np.float32)
    st, outb = T.run_attention(wb, T.upload(hb))
    assert st == 0
    gotb = T.to_host_f64(outb, BF16).reshape(b, n, d)
    assert T.rel_err(got, gotb, gotb) <= ATT_TIGHT[BF16]


@pytest.mark.parametrize("force", [None, "generic"])
def test_attention_causal_more_queries_than_keys(force):
    """Nq > Nk: the first Nq - Nk rows see no key (0/0: NaN on both sides), the others are defined."""
    import paper_2603_06731_amd as pbk
    b, nq, nk, d = 2, 200, 130, 64
    w = wl.AttentionWorkload("att_causal_tall", BF16, b, nq, nk, d, alpha=scale(d), causal=True)
    host = wl.make_attention_inputs(w)
    with T.forced_kernel(force):
        st, out = T.run_attention(w, T.upload(host))
    assert st == 0, pbk.pbk_status_string(st)
    ref = T.oracle_attention_full(w, host)
    got = T.to_host_f64(out, BF16).reshape(ref.shape)
    empty = nq - nk
    assert np.isnan(ref[:, :empty]).all() and np.isnan(got[:, :empty]).all()
    assert T.rel_err(got[:, empty:], ref[:, empty:], ref[:, empty:]) <= ATT_TIGHT[BF16]


def test_attention_causal_nonpositive_scale_takes_the_generic_kernel():
    w = wl.AttentionWorkload("att_causal_alpha0", BF16, 2, 150, 150, 64, alpha=0.0, causal=True)
    check_attention(w, expect_kernel="attn_generic")


@pytest.mark.parametrize("force", [None, "generic"])
def test_attention_views_strides_and_guard_bands(force):
    """Row strides larger than D with NaN planted in the gaps, K and V shared by
    all batch entries (stride 0), and untouched output outside the O view."""
    import torch
    import paper_2603_06731_amd as pbk
    import oracle
    b, nq, nk, d, ld = 3, 140, 101, 64, 80
    r = np.random.default_rng(5)
    q = wl.to_storage(r.normal(size=(b, nq, d)), BF16)
    k = wl.to_storage(r.normal(size=(1, nk, d)), BF16)
    v = wl.to_storage(r.normal(size=(1, nk, d)), BF16)
    nan = np.uint16(0x7FC0)

    def padded(x):
        p = np.full(x.shape[:2] + (ld,), nan, dtype=np.uint16)
        p[:, :, :d] = x
        return p
    dq, dk, dv = (T.to_device(padded(x)) for x in (q, k, v))
    sentinel = 0x1234
    out = torch.full((b * nq * ld + 64,), sentinel, dtype=torch.int16, device="cuda")
    with T.forced_kernel(force):
        st = pbk.pbk_attention(dq, dk, dv, None, out, b, nq, nk, d, ld, ld, ld, ld,
                               nq * ld, 0, 0, nq * ld, 0, 0, BF16, 0.125, None)
    assert st == 0, pbk.pbk_status_string(st)
    ref = oracle.attention(q, np.repeat(k, b, axis=0), np.repeat(v, b, axis=0), dtype=BF16, alpha=0.125)
    raw = out.cpu().numpy().view(np.uint16)
    body = raw[:b * nq * ld].reshape(b, nq, ld)
    got = wl.widen(np.ascontiguousarray(body[:, :, :d]), BF16)
    err = T.rel_err(got, ref, ref)
    print(f"views force={force} kernel={pbk.pbk_last_kernel()} err={err:.3e}", flush=True)
    assert err <= ATT_TIGHT[BF16]
    assert np.all(body[:, :, d:] == sentinel) and np.all(raw[b * nq * ld:] == sentinel)


def test_attention_is_deterministic():
    import torch
    w = wl.AttentionWorkload("att_det", BF16, 4, 300, 700, 128, alpha=scale(128))
    dev = T.upload(wl.make_attention_inputs(w))
    _, a = T.run_attention(w, dev)
    _, b = T.run_attention(w, dev)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


PAPER_SHAPES = ["attn_h16_n512_d64", "attn_h16_n2048_d64", "attn_h16_n8192_d64", "attn_h16_n512_d128",
                "attn_h16_n2048_d128", "attn_h16_n8192_d128", "attn_h16_n577_d64", "attn_h12_n10_d64",
                "attn_h6_n297_d64", "attn_h8_n500_d32", "attn_h32_n1024_d128",
                "attn_h16_n2048_d64_causal", "attn_h16_n8192_d64_causal", "attn_h16_n8192_d128_causal"]


@pytest.mark.parametrize("name", PAPER_SHAPES)
def test_attention_paper_shapes_sampled_rows(name):
    """The shapes of the paper's attention table, in the launch configuration the
    bench times; rows sampled over every query tile position and the tile edges."""
    import paper_2603_06731_amd as pbk
    w = wl.ATTENTION_CONFIGS[name]
    host = wl.make_attention_inputs(w)
    dev = T.upload(host)
    st, out = T.run_attention(w, dev)
    assert st == 0, pbk.pbk_status_string(st)
    r = np.random.default_rng(11)
    edge = np.array([0, 1, 31, 32, 63, 64, 127, 128], dtype=np.int64)
    si = np.unique(np.concatenate([edge[edge < w.Nq], w.Nq - 1 - edge[edge < w.Nq],
                                   r.integers(0, w.Nq, size=48)]))
    sb = r.integers(0, w.batch, size=si.size)
    sb[:2] = [0, w.batch - 1]
    ref = T.oracle_attention_rows(w, host, sb, si)
    got = T.to_host_f64(out, w.dtype).reshape(w.batch, w.Nq, w.D)[sb, si]
    err = T.rel_err(got, ref, ref)
    print(f"{name} kernel={pbk.pbk_last_kernel()} rows={si.size} err={err:.3e}", flush=True)
    assert "attn_mfma" in pbk.pbk_last_kernel()
    assert err <= ATT_TIGHT[w.dtype], (name, err)
