"""Parity of the HIP path (through the C ABI) with the CPU oracle on seeded
inputs.  Small cases are compared element by element; the full-size workloads
are compared on sampled outputs the oracle computes one by one."""
import numpy as np
import pytest

import workloads as wl
from workloads import configs as C
import pbk_testlib as T

pytestmark = pytest.mark.gpu

BF16, F16, F32 = wl.DTYPE_BF16, wl.DTYPE_F16, wl.DTYPE_F32
MFMA_CONFIGS = [0, 1, 5, 6, 7, 9]       # the configurations built for the 16-bit types


def tol_for(w):
    return T.TOL_F32 if w.in_dtype == F32 else T.TOL_16BIT


def tight_for(w):
    if w.in_dtype == F32:
        return T.TOL_F32
    if w.in_dtype in (wl.DTYPE_FP8_E4M3, wl.DTYPE_FP8_E5M2) and w.out_dtype == F32:
        # the FP8 matrix instructions do not add the (exact) products in full binary32: every block shape of
        # v_mfma_*_f8f6f4 gives the same result, 1.0e-4 .. 1.9e-4 away from the oracle on these shapes (about 13
        # bits below the largest term), where the FMA kernel is 6e-8 away; the bar for an fp32 output follows that
        return 4e-4
    return T.TIGHT[w.out_dtype]


def check_full(w, force=None, expect_kernel=None):
    import paper_2603_06731_amd as pbk
    host = wl.make_inputs(w)
    dev = T.upload(host)
    with T.forced_kernel(force):
        st, out = T.run_workload(w, dev)
    assert st == 0, pbk.pbk_status_string(st)
    if expect_kernel:
        assert expect_kernel in pbk.pbk_last_kernel(), pbk.pbk_last_kernel()
    ref, pre = T.oracle_full(w, host)
    got = T.to_host_f64(out, w.out_dtype).reshape(ref.shape)
    err = T.rel_err(got, ref, pre)
    print(f"{w.name} force={force} kernel={pbk.pbk_last_kernel()} err={err:.3e}", flush=True)
    assert err <= tol_for(w), (w.name, force, err)
    assert err <= tight_for(w), (w.name, force, err)
    return err


# --------------------------------------------------------------- matmul, small

SMALL_MM = [
    # M, N, K  (several tiles, ragged tails in M and N, K not a multiple of the k-tile)
    (300, 264, 200),
    (256, 256, 64),
    (520, 136, 72),
    (33, 520, 136),
    (64, 8, 8),
]


@pytest.mark.parametrize("cfg", MFMA_CONFIGS)
@pytest.mark.parametrize("mnk", SMALL_MM)
def test_matmul_bf16_mfma_configs(cfg, mnk):
    m, n, k = mnk
    w = wl.Workload(f"mm_{m}x{n}x{k}", "matmul", BF16, BF16, C.EPI_BIAS_RELU, M=m, N=n, K=k,
                    dist_b=("normal", 1.0 / np.sqrt(k)), dist_bias=("normal", 0.5))
    check_full(w, force=f"mfma:{cfg}", expect_kernel="mfma")


@pytest.mark.parametrize("cfg", [7, 9])
@pytest.mark.parametrize("dtype", [BF16, F16])
@pytest.mark.parametrize("k", [8, 40, 64, 72, 96, 128, 136, 160, 168, 192, 200, 224, 232, 264, 328, 392, 1096])
def test_matmul_a_staged_64_deep_k_sweep(cfg, dtype, k):
    """Configurations 7 and 9 stage A every other k-tile (9 with six B stages and one barrier per pair of
    k-tiles): prologue only, drain only, odd and even numbers of k-tiles (1 to 13 and 35), a ragged
    last tile, and enough tiles for the paired steady state."""
    w = wl.Workload(f"mm_a64_k{k}", "matmul", dtype, dtype, C.EPI_BIAS, M=300, N=520, K=k,
                    dist_b=("normal", 1.0 / np.sqrt(k)), dist_bias=("normal", 0.5))
    check_full(w, force=f"mfma:{cfg}", expect_kernel="a64")


@pytest.mark.parametrize("dtype", [BF16, F16])
@pytest.mark.parametrize("k", [8, 40, 64, 72, 96, 128, 136, 160, 168, 192, 200, 224, 232, 264, 328, 392, 1096])
def test_matmul_pair_pipeline_k_major_b_k_sweep(dtype, k):
    """Configuration 9 with a k-major B stages both operands 64 deep: the same sweep over the number of k-tiles,
    with a ragged N and M."""
    w = wl.Workload(f"mm_pair_tb_k{k}", "matmul", dtype, dtype, C.EPI_BIAS, M=300, N=517, K=k, trans_b=1,
                    dist_b=("normal", 1.0 / np.sqrt(k)), dist_bias=("normal", 0.5))
    check_full(w, force="mfma:9", expect_kernel="pair")


@pytest.mark.parametrize("cfg", [7, 9])
def test_batched_on_a_staged_64_deep(cfg):
    w = wl.Workload("bmm_a64", "batched", BF16, F32, C.EPI_NONE, alpha=0.5, batch=3, M=264, N=256, K=392,
                    dist_b=("normal", 0.05))
    check_full(w, force=f"mfma:{cfg}", expect_kernel="a64")


@pytest.mark.parametrize("dtype", [BF16, F16])
@pytest.mark.parametrize("out_dtype", ["same", "f32"])
@pytest.mark.parametrize("epi", [C.EPI_NONE, C.EPI_BIAS, C.EPI_RELU, C.EPI_BIAS_RELU,
                                 C.EPI_BIAS_GELU_TANH, C.EPI_GELU_TANH])
def test_matmul_epilogues_and_dtypes(dtype, out_dtype, epi):
    od = dtype if out_dtype == "same" else F32
    w = wl.Workload("mm_epi", "matmul", dtype, od, epi, alpha=0.75, M=200, N=264, K=136,
                    dist_b=("normal", 1.0 / np.sqrt(136)), dist_bias=("normal", 0.5))
    check_full(w, expect_kernel="mfma")


@pytest.mark.parametrize("cfg", MFMA_CONFIGS)
@pytest.mark.parametrize("dtype", [BF16, F16])
def test_matmul_trans_b(cfg, dtype):
    w = wl.Workload("mm_tb", "matmul", dtype, dtype, C.EPI_BIAS, M=264, N=301, K=200, trans_b=1,
                    dist_b=("normal", 1.0 / np.sqrt(200)))
    check_full(w, force=f"mfma:{cfg}", expect_kernel="mfma")


@pytest.mark.parametrize("dtype", [F32, BF16, F16])
@pytest.mark.parametrize("mnk", [(67, 45, 33), (1, 1, 1), (130, 129, 70), (5, 300, 7)])
@pytest.mark.parametrize("trans_b", [0, 1])
def test_matmul_generic_odd_shapes(dtype, mnk, trans_b):
    m, n, k = mnk
    w = wl.Workload("mm_odd", "matmul", dtype, dtype, C.EPI_BIAS_GELU_TANH, alpha=0.5, M=m, N=n, K=k,
                    trans_b=trans_b, dist_b=("normal", 1.0 / np.sqrt(k)))
    # 16-bit operands with enough work (M N >= 4096, K >= 16) take the gathering matrix-unit kernel
    gather = dtype != F32 and m * n >= 4096 and k >= 16
    # small fp32 problems take the one-wave-per-tile kernel
    check_full(w, expect_kernel="small_f32" if dtype == F32 else "gather" if gather else "generic")
    check_full(w, force="generic", expect_kernel="generic")


def test_cfg1_fp32_256():
    check_full(wl.CONFIGS["cfg1_f32_256"])


# ------------------------------------------------------------------- batched

@pytest.mark.parametrize("trans_b", [0, 1])
def test_batched_small(trans_b):
    w = wl.Workload("bmm", "batched", BF16, BF16, C.EPI_NONE, alpha=float(np.float32(1 / np.sqrt(128))),
                    batch=5, M=264, N=200, K=128, trans_b=trans_b)
    check_full(w, expect_kernel="mfma")


def test_batched_broadcast_b():
    import paper_2603_06731_amd as pbk
    import oracle
    batch, m, n, k = 3, 136, 264, 72
    a = wl.tensor((batch, m, k), BF16, 1, "normal")
    b = wl.tensor((k, n), BF16, 2, "normal", 0.1)
    da, db = T.to_device(a), T.to_device(b)
    out = T.device_empty(batch * m * n, BF16)
    st = pbk.pbk_batched_matmul(da, db, out, None, batch, m, n, k, k, n, n, m * k, 0, m * n,
                                BF16, BF16, 0, 1.0, C.EPI_NONE)
    assert st == 0
    ref, pre = oracle.batched_matmul(a, b, None, dtype=BF16, batch=batch, stride_b=0, want_preact=True)
    err = T.rel_err(T.to_host_f64(out, BF16).reshape(ref.shape), ref, pre)
    assert err <= T.TIGHT[BF16], err


# ---------------------------------------------------------------------- conv

CONV_SMALL = [
    # n, H, W, Cin, Cout, KH, KW, stride, pad, dil
    (2, 14, 14, 32, 64, 3, 3, (1, 1), (1, 1), (1, 1)),
    (1, 23, 21, 16, 136, 3, 3, (2, 2), (0, 0), (1, 1)),
    (2, 17, 19, 8, 264, 5, 3, (1, 2), (2, 1), (2, 1)),
    (3, 9, 9, 64, 8, 1, 1, (1, 1), (0, 0), (1, 1)),
]


@pytest.mark.parametrize("case", CONV_SMALL)
@pytest.mark.parametrize("cfg", [None] + MFMA_CONFIGS)
def test_conv_small_mfma(case, cfg):
    n, H, W, Cin, Cout, KH, KW, stride, pad, dil = case
    w = wl.Workload("conv_s", "conv", BF16, BF16, C.EPI_BIAS_RELU, n=n, H=H, W=W, Cin=Cin, Cout=Cout,
                    KH=KH, KW=KW, stride=stride, pad=pad, dil=dil,
                    dist_b=("normal", float(np.sqrt(2.0 / (KH * KW * Cin)))))
    check_full(w, force=None if cfg is None else f"mfma:{cfg}", expect_kernel="mfma")


@pytest.mark.parametrize("dtype", [BF16, F16])
@pytest.mark.parametrize("case", [
    # n, H, W, Cin, Cout, KH, KW, stride, pad, dil: channel counts that are multiples of 64, so that the pair
    # pipeline stages the image 64 deep; 2 to 50 k-tiles (prologue only, drain only, the steady state), padding
    # on every side, stride, dilation, ragged M and Cout
    (3, 9, 9, 64, 8, 1, 1, (1, 1), (0, 0), (1, 1)),
    (2, 14, 13, 64, 264, 3, 3, (1, 1), (1, 1), (1, 1)),
    (1, 23, 21, 128, 136, 3, 3, (2, 2), (0, 0), (1, 1)),
    (2, 17, 19, 64, 72, 5, 3, (1, 2), (2, 1), (2, 1)),
    (1, 20, 20, 192, 256, 1, 3, (1, 1), (0, 1), (1, 1)),
    (1, 12, 12, 320, 40, 2, 2, (1, 1), (1, 0), (1, 1)),
])
def test_conv_pair_pipeline(case, dtype):
    n, H, W, Cin, Cout, KH, KW, stride, pad, dil = case
    w = wl.Workload("conv_pair", "conv", dtype, dtype, C.EPI_BIAS_RELU, n=n, H=H, W=W, Cin=Cin, Cout=Cout,
                    KH=KH, KW=KW, stride=stride, pad=pad, dil=dil,
                    dist_b=("normal", float(np.sqrt(2.0 / (KH * KW * Cin)))))
    check_full(w, force="mfma:9", expect_kernel="pair")


@pytest.mark.parametrize("dtype,out_dtype", [(F16, F32), (F32, F32), (BF16, BF16)])
def test_conv_generic_tiny_channels(dtype, out_dtype):
    # Cin = 3, Cout = 3, 5x5 filter: the shape family of the paper's second worked example
    w = wl.Workload("conv_c3", "conv", dtype, out_dtype, C.EPI_BIAS, n=1, H=40, W=36, Cin=3, Cout=3,
                    KH=5, KW=5, dist_b=("normal", 0.2))
    check_full(w, expect_kernel="generic")


def test_conv_paper_example_shape_reduced():
    # stride-2 3x3 over 127 channels (paper's first worked example, fewer images/outputs)
    w = wl.Workload("conv_p1", "conv", F16, F32, C.EPI_NONE, n=2, H=44, W=44, Cin=127, Cout=24,
                    KH=3, KW=3, stride=(2, 2), dist_b=("normal", 0.03))
    check_full(w, expect_kernel="mfma")           # 127 channels: the gathering matrix-unit kernel
    check_full(w, force="generic", expect_kernel="generic")


# ---------------------------------------------------- full-size, sampled outputs

@pytest.mark.parametrize("name", ["cfg2_bf16_8192", "cfg3_bf16_attn_scores", "cfg4_bf16_mlp",
                                  "cfg5_bf16_conv3x3"])
def test_full_size_sampled(name):
    import paper_2603_06731_amd as pbk
    w = wl.CONFIGS[name]
    host = wl.make_inputs(w)
    dev = T.upload(host)
    st, out = T.run_workload(w, dev)
    assert st == 0
    kern = pbk.pbk_last_kernel()
    b, i, j = T.sample_coords(w, 3000)
    ref, pre = T.oracle_sampled(w, host, b, i, j)
    got = T.gather_output(out, w, b, i, j)
    err = T.rel_err(got, ref, pre)
    print(f"{name} kernel={kern} samples={len(i)} err={err:.3e}", flush=True)
    assert "mfma" in kern
    assert err <= T.TOL_16BIT and err <= T.TIGHT[w.out_dtype], err
    # every workgroup tile: one complete row per 128 rows and one complete column per 128 columns
    rows, cols = T.tile_lines(w)
    ro, rp, co, cp = T.oracle_tile_lines(w, host, rows, cols)
    gr, gc = T.gather_tile_lines(out, w, rows, cols)
    floor_pre = np.concatenate([rp.reshape(-1), cp.reshape(-1)])
    err_r = T.rel_err(gr, ro, floor_pre)
    err_c = T.rel_err(gc, co, floor_pre)
    print(f"{name} complete rows {len(rows)} x batch {w.batch}: err={err_r:.3e}; complete columns {len(cols)}: "
          f"err={err_c:.3e}", flush=True)
    assert max(err_r, err_c) <= T.TIGHT[w.out_dtype], (err_r, err_c)
    if name == "cfg2_bf16_8192":
        # bias dominates that output; also check the bare contraction
        w2 = wl.Workload("cfg2_noepi", "matmul", BF16, BF16, C.EPI_NONE, M=w.M, N=w.N, K=w.K,
                         dist_a=w.dist_a, dist_b=w.dist_b)
        st, out2 = T.run_workload(w2, {"a": dev["a"], "b": dev["b"], "bias": None})
        assert st == 0
        ref2, pre2 = T.oracle_sampled(w2, {"a": host["a"], "b": host["b"], "bias": None}, b, i, j)
        err2 = T.rel_err(T.gather_output(out2, w2, b, i, j), ref2, pre2)
        print(f"cfg2 without epilogue err={err2:.3e}", flush=True)
        assert err2 <= T.TIGHT[BF16], err2


# ------------------------------------------------------------------ edge cases

def test_views_ignore_nan_outside_and_guard_band_survives():
    import paper_2603_06731_amd as pbk
    import oracle
    M, N, K, lda, ldb, ldc = 136, 264, 72, 96, 280, 272
    a = wl.tensor((M, lda), BF16, 1, "normal")
    b = wl.tensor((K, ldb), BF16, 2, "normal", 0.1)
    a[:, K:] = 0x7FC0            # NaN beyond K
    b[:, N:] = 0x7FC0            # NaN beyond N
    da, db = T.to_device(a), T.to_device(b)
    sentinel = 0x5A5A
    out = T.device_empty(M * ldc + 64, BF16, fill=np.array(sentinel, dtype=np.uint16).view(np.int16).item())
    for force in ("mfma:0", "mfma:1", "mfma:5", "mfma:7", "mfma:9", "generic"):
        with T.forced_kernel(force):
            st = pbk.pbk_matmul(da, db, out, None, M, N, K, lda, ldb, ldc, BF16, BF16, 0, 1.0, C.EPI_NONE)
        assert st == 0
        raw = out.cpu().numpy().view(np.uint16)
        body = raw[:M * ldc].reshape(M, ldc)
        assert np.all(body[:, N:] == sentinel) and np.all(raw[M * ldc:] == sentinel)
        ref, pre = oracle.matmul(a, b, None, dtype=BF16, M=M, N=N, K=K, lda=lda, ldb=ldb, want_preact=True)
        got = wl.widen(np.ascontiguousarray(body[:, :N]), BF16)
        assert T.rel_err(got, ref, pre) <= T.TIGHT[BF16], force


def test_run_to_run_bit_exact():
    w = wl.Workload("det", "matmul", BF16, BF16, C.EPI_BIAS_GELU_TANH, M=520, N=520, K=520,
                    dist_b=("normal", 0.05))
    dev = T.upload(wl.make_inputs(w))
    outs = []
    for _ in range(3):
        st, out = T.run_workload(w, dev)
        assert st == 0
        outs.append(out.cpu().numpy().copy())
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


_det_big_cache = {}


def _det_big_oracle(w, host):
    """The oracle's full result for the long many-tile case, computed once per session."""
    if "ref" not in _det_big_cache:
        _det_big_cache["ref"] = T.oracle_full(w, host)
    return _det_big_cache["ref"]


@pytest.mark.parametrize("cfg", [5, 6, 7, 9])
def test_large_run_to_run_bit_exact_and_equal_across_configurations(cfg):
    """The pipelines reuse LDS stages under explicit wait counts and one barrier per k-tile: a race
    would show as run-to-run differences on a long contraction.  All 16x16 configurations add the
    products of an output element in the same order (k ascending inside the MFMA chain), so their
    results are also bit-identical to each other."""
    import torch
    w = wl.Workload("det_big", "matmul", BF16, BF16, C.EPI_BIAS, M=1024, N=1536, K=8192,
                    dist_b=("normal", 1.0 / np.sqrt(8192)))
    host = wl.make_inputs(w)
    dev = T.upload(host)
    with T.forced_kernel("mfma:5"):
        st, ref = T.run_workload(w, dev)
    assert st == 0
    ref = ref.clone()
    # the whole tensor of this configuration against the oracle, element by element
    with T.forced_kernel(f"mfma:{cfg}"):
        st, out = T.run_workload(w, dev)
    assert st == 0
    want, pre = _det_big_oracle(w, host)
    err = T.rel_err(T.to_host_f64(out, w.out_dtype).reshape(want.shape), want, pre)
    print(f"det_big cfg={cfg} full oracle comparison err={err:.3e}", flush=True)
    assert err <= T.TIGHT[BF16], (cfg, err)
    for _ in range(4):
        with T.forced_kernel(f"mfma:{cfg}"):
            st, out = T.run_workload(w, dev)
        assert st == 0
        torch.cuda.synchronize()
        assert torch.equal(out, ref), cfg


def test_zero_sizes_and_k_zero():
    import paper_2603_06731_amd as pbk
    out = T.device_empty(16, F32, fill=7.0)
    assert pbk.pbk_matmul(None, None, out, None, 0, 4, 4, 4, 4, 4, F32, F32, 0, 1.0, 0) == 0
    assert pbk.pbk_matmul(None, None, out, None, 4, 0, 4, 4, 4, 4, F32, F32, 0, 1.0, 0) == 0
    assert np.all(out.cpu().numpy() == 7.0)
    bias = T.to_device(np.array([1.0, -2.0, 3.0, -4.0], dtype=np.float32))
    assert pbk.pbk_matmul(None, None, out, bias, 4, 4, 0, 4, 4, 4, F32, F32, 0, 1.0, C.EPI_BIAS_RELU) == 0
    assert np.array_equal(out.cpu().numpy().reshape(4, 4), np.tile([1.0, 0.0, 3.0, 0.0], (4, 1)))


def test_non_default_stream():
    import torch
    w = wl.Workload("stream", "matmul", F16, F16, C.EPI_RELU, M=264, N=264, K=264, dist_b=("normal", 0.06))
    host = wl.make_inputs(w)
    dev = T.upload(host)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        st, out = T.run_workload(w, dev, stream=s)
    s.synchronize()
    assert st == 0
    ref, pre = T.oracle_full(w, host)
    assert T.rel_err(T.to_host_f64(out, F16).reshape(ref.shape), ref, pre) <= T.TIGHT[F16]


# ------------------------------------------------------------------------ FP8

FP8_TYPES = [wl.DTYPE_FP8_E4M3, wl.DTYPE_FP8_E5M2]


@pytest.mark.parametrize("dtype", FP8_TYPES)
@pytest.mark.parametrize("out_dtype", [BF16, F16, F32])
@pytest.mark.parametrize("cfg", [None, 1, 4, 9])
def test_fp8_matmul_kmajor_operands(dtype, out_dtype, cfg):
    # both operands k-major (trans_b): MFMA path; several tiles, ragged M and N, K not a multiple of 128
    w = wl.Workload("fp8_nt", "matmul", dtype, out_dtype, C.EPI_BIAS_GELU_TANH, alpha=0.5, M=300, N=261, K=208,
                    trans_b=1, dist_b=("normal", 1.0 / np.sqrt(208)), dist_bias=("normal", 0.5))
    check_full(w, force=None if cfg is None else f"mfma:{cfg}", expect_kernel="mfma")


@pytest.mark.parametrize("dtype", FP8_TYPES)
@pytest.mark.parametrize("k", [16, 64, 80, 128, 144, 192, 256, 272, 320, 400, 448, 528, 656, 2192])
def test_fp8_pair_pipeline_k_sweep(dtype, k):
    """Both operands staged 128 values deep, one v_mfma_f32_16x16x128 k-step and one barrier per pair of
    64-value k-tiles: prologue only, drain only, odd and even tile counts, ragged last pieces, the steady state."""
    w = wl.Workload(f"fp8_pair_k{k}", "matmul", dtype, F32, C.EPI_BIAS, M=300, N=517, K=k, trans_b=1,
                    dist_b=("normal", 1.0 / np.sqrt(k)), dist_bias=("normal", 0.5))
    check_full(w, force="mfma:9", expect_kernel="pair")


@pytest.mark.parametrize("dtype", FP8_TYPES)
@pytest.mark.parametrize("mnk,trans_b", [((136, 264, 72), 0), ((67, 45, 33), 1), ((130, 129, 70), 0)])
def test_fp8_matmul_other_layouts_take_generic_kernel(dtype, mnk, trans_b):
    m, n, k = mnk
    w = wl.Workload("fp8_gen", "matmul", dtype, BF16, C.EPI_BIAS_RELU, M=m, N=n, K=k, trans_b=trans_b,
                    dist_b=("normal", 1.0 / np.sqrt(k)))
    check_full(w, expect_kernel="generic")


@pytest.mark.parametrize("dtype", FP8_TYPES)
@pytest.mark.parametrize("cfg", [None, 1, 4])
@pytest.mark.parametrize("mnk", [(300, 272, 208), (256, 512, 128), (33, 144, 4096)])
def test_fp8_matmul_row_major_b_on_mfma(dtype, cfg, mnk):
    """Row-major B: the n-major byte tile is read with the 8-bit transposing LDS read."""
    m, n, k = mnk
    w = wl.Workload("fp8_nn", "matmul", dtype, BF16, C.EPI_BIAS_RELU, M=m, N=n, K=k,
                    dist_b=("normal", 1.0 / np.sqrt(k)), dist_bias=("normal", 0.5))
    check_full(w, force=None if cfg is None else f"mfma:{cfg}", expect_kernel="mfma")


@pytest.mark.parametrize("dtype", FP8_TYPES)
@pytest.mark.parametrize("cfg", [None, 1, 4])
@pytest.mark.parametrize("case", [(2, 14, 13, 32, 48, 3, 3, (1, 1), (1, 1), (1, 1)),
                                  (1, 17, 16, 128, 64, 3, 3, (2, 2), (1, 1), (1, 1)),
                                  (2, 12, 12, 48, 80, 2, 3, (1, 2), (0, 2), (2, 1))])
def test_fp8_conv_on_mfma(dtype, cfg, case):
    n, H, W, Cin, Cout, KH, KW, stride, pad, dil = case
    w = wl.Workload("fp8_conv_mfma", "conv", dtype, BF16, C.EPI_BIAS_RELU, n=n, H=H, W=W, Cin=Cin, Cout=Cout,
                    KH=KH, KW=KW, stride=stride, pad=pad, dil=dil,
                    dist_b=("normal", float(np.sqrt(2.0 / (KH * KW * Cin)))))
    check_full(w, force=None if cfg is None else f"mfma:{cfg}", expect_kernel="mfma")


def test_fp8_batched_and_conv_generic():
    w = wl.Workload("fp8_bmm", "batched", wl.DTYPE_FP8_E4M3, F16, C.EPI_NONE, alpha=0.25, batch=3, M=136, N=200,
                    K=128, trans_b=1)
    check_full(w, expect_kernel="mfma")
    w = wl.Workload("fp8_conv", "conv", wl.DTYPE_FP8_E4M3, F32, C.EPI_BIAS_RELU, n=1, H=9, W=10, Cin=16, Cout=24,
                    KH=3, KW=3, pad=(1, 1), dist_b=("normal", 0.1))
    check_full(w, expect_kernel="generic")


def test_fp8_full_size_sampled():
    import paper_2603_06731_amd as pbk
    w = wl.EXTRA_CONFIGS["fp8_e4m3_8192_nt"]
    host = wl.make_inputs(w)
    st, out = T.run_workload(w, T.upload(host))
    assert st == 0 and "mfma" in pbk.pbk_last_kernel()
    b, i, j = T.sample_coords(w, 3000)
    ref, pre = T.oracle_sampled(w, host, b, i, j)
    err = T.rel_err(T.gather_output(out, w, b, i, j), ref, pre)
    print(f"fp8 8192^3 kernel={pbk.pbk_last_kernel()} err={err:.3e}", flush=True)
    assert err <= T.TIGHT[BF16], err


# ----------------------------------------------------------------- fp32 on MFMA

@pytest.mark.parametrize("cfg", [None, 0, 1])
@pytest.mark.parametrize("mnk,trans_b", [((520, 264, 200), 0), ((256, 512, 64), 1), ((1100, 1032, 132), 0),
                                         ((300, 260, 36), 1)])
def test_fp32_matmul_on_mfma(cfg, mnk, trans_b):
    """fp32 operands on v_mfma_f32_32x32x2_f32: true fp32 arithmetic, the 1e-5 bar."""
    m, n, k = mnk
    w = wl.Workload("f32_mfma", "matmul", F32, F32, C.EPI_BIAS_GELU_TANH, alpha=0.75, M=m, N=n, K=k, trans_b=trans_b,
                    dist_a=("uniform", 1.0), dist_b=("uniform", 1.0), dist_bias=("uniform", 1.0))
    if cfg is None and m * n < 1024 * 1024:
        # too little work for 128-wide tiles: the one-wave-per-tile kernel up to 1024 tiles of 16 x 16, else the generic one
        small = ((m + 15) // 16) * ((n + 15) // 16) <= 1024
        check_full(w, expect_kernel="small_f32" if small else "generic")
    else:
        check_full(w, force=None if cfg is None else f"mfma:{cfg}", expect_kernel="mfma_f32")


@pytest.mark.parametrize("cfg", [0, 1])
def test_fp32_batched_and_conv_on_mfma(cfg):
    w = wl.Workload("f32_bmm", "batched", F32, F32, C.EPI_NONE, alpha=0.5, batch=3, M=264, N=200, K=96,
                    dist_a=("uniform", 1.0), dist_b=("uniform", 1.0))
    check_full(w, force=f"mfma:{cfg}", expect_kernel="mfma_f32")
    w = wl.Workload("f32_conv", "conv", F32, F32, C.EPI_BIAS_RELU, n=2, H=14, W=13, Cin=20, Cout=36, KH=3, KW=3,
                    stride=(2, 1), pad=(1, 2), dil=(1, 2), dist_a=("uniform", 1.0), dist_b=("uniform", 0.2),
                    dist_bias=("uniform", 0.5))
    check_full(w, force=f"mfma:{cfg}", expect_kernel="mfma_f32")


def test_fp32_large_matmul_takes_mfma_and_is_sampled():
    import paper_2603_06731_amd as pbk
    w = wl.Workload("f32_2048", "matmul", F32, F32, C.EPI_BIAS_RELU, M=2048, N=2048, K=1024,
                    dist_a=("uniform", 1.0), dist_b=("uniform", 1.0), dist_bias=("uniform", 1.0))
    host = wl.make_inputs(w)
    st, out = T.run_workload(w, T.upload(host))
    assert st == 0 and "mfma_f32" in pbk.pbk_last_kernel()
    b, i, j = T.sample_coords(w, 2000)
    ref, pre = T.oracle_sampled(w, host, b, i, j)
    err = T.rel_err(T.gather_output(out, w, b, i, j), ref, pre)
    print(f"f32 2048x2048x1024 kernel={pbk.pbk_last_kernel()} err={err:.3e}", flush=True)
    assert err <= T.TOL_F32, err


@pytest.mark.parametrize("force", [None, "mfma:1", "mfma:6", "generic"])
def test_relu_keeps_nan(force):
    """ReLU(NaN) is NaN on both sides (the oracle's definition; the paper's nest compares 'unordered or
    greater'): a NaN in one row of A makes that output row NaN, every other row stays as the oracle has it."""
    import paper_2603_06731_amd as pbk
    w = wl.Workload("relu_nan", "matmul", BF16, BF16, C.EPI_BIAS_RELU, M=264, N=264, K=136, dist_b=("normal", 0.1))
    host = wl.make_inputs(w)
    host["a"][7, 3] = 0x7FC0                     # a bf16 NaN
    with T.forced_kernel(force):
        st, out = T.run_workload(w, T.upload(host))
    assert st == 0
    got = T.to_host_f64(out, BF16).reshape(w.M, w.N)
    ref, pre = T.oracle_full(w, host)
    ref, pre = ref.reshape(w.M, w.N), pre.reshape(w.M, w.N)
    assert np.isnan(ref[7]).all() and np.isnan(got[7]).all(), pbk.pbk_last_kernel()
    rows = np.arange(w.M) != 7
    assert np.isfinite(got[rows]).all()
    assert T.rel_err(got[rows], ref[rows], pre[rows]) <= T.TIGHT[BF16]
