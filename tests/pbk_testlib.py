"""Helpers shared by the GPU parity tests, the smoke check and the bench:
device upload/download through torch (memory and streams only), calls through
the C ABI binding, and the error metric."""
from __future__ import annotations

import contextlib
import os

import numpy as np

import workloads as wl

TOL_16BIT = 2e-2      # max relative error, bf16/fp16 inputs with fp32 accumulation
TOL_F32 = 1e-5        # fp32

# tighter expectations derived from the arithmetic: one rounding to the output
# type (half an ulp: 2^-9 of the leading power for bf16 -> <= 2^-8 relative,
# 2^-11 for fp16) plus fp32 accumulation noise
TIGHT = {wl.DTYPE_BF16: 5e-3, wl.DTYPE_F16: 8e-4, wl.DTYPE_F32: 1e-4}


def torch_mod():
    import torch
    return torch


def to_device(a: np.ndarray):
    """numpy (float32 or uint16 bits) -> torch device tensor (float32 / int16 bits)."""
    torch = torch_mod()
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    if a.dtype == np.uint8:
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def device_empty(nelem: int, dtype: int, fill=None):
    torch = torch_mod()
    td = torch.float32 if dtype == wl.DTYPE_F32 else torch.int16
    if fill is None:
        return torch.empty(nelem, dtype=td, device="cuda")
    return torch.full((nelem,), fill, dtype=td, device="cuda")


def to_host_f64(t, dtype: int) -> np.ndarray:
    """device tensor -> float64 numpy, widening stored bits exactly."""
    a = t.cpu().numpy()
    if dtype == wl.DTYPE_F32:
        return a.astype(np.float64)
    return wl.widen(a.view(np.uint16), dtype)


def rel_err(got: np.ndarray, ref: np.ndarray, preact: np.ndarray) -> float:
    """max |g - r| / max(|r|, RMS(pre-activation oracle value))."""
    if ref.size == 0:
        return 0.0
    floor = float(np.sqrt(np.mean(np.square(preact))))
    if floor == 0.0:
        floor = 1.0
    d = np.abs(got - ref) / np.maximum(np.abs(ref), floor)
    if not np.all(np.isfinite(got)):
        return float("inf")
    return float(d.max())


_forced = [None]


@contextlib.contextmanager
def forced_kernel(choice: str | None):
    """Force the dispatcher ("generic", "mfma", "mfma:<id>") for the calls inside (this thread)."""
    import paper_2603_06731_amd as pbk
    old = _forced[0]
    pbk.check(pbk.pbk_force_kernel(choice), f"pbk_force_kernel({choice!r})")
    _forced[0] = choice
    try:
        yield
    finally:
        pbk.pbk_force_kernel(old)
        _forced[0] = old


def run_workload(w: wl.Workload, dev: dict, out=None, stream=None):
    """Enqueue the workload's call on device tensors dev = {"a","b","bias"}.
    Returns (status, out tensor)."""
    import paper_2603_06731_amd as pbk
    m, n, k = w.gemm_mnk
    if out is None:
        out = device_empty(w.batch * m * n, w.out_dtype)
    if w.kind == "conv" and w.transposed:
        st = pbk.pbk_conv2d_transpose_nhwc(dev["a"], dev["b"], out, dev["bias"], w.n, w.H, w.W, w.Cin, w.Cout,
                                           w.KH, w.KW, w.stride[0], w.stride[1], w.pad[0], w.pad[1],
                                           w.out_pad[0], w.out_pad[1], w.dil[0], w.dil[1],
                                           w.in_dtype, w.out_dtype, w.alpha, w.epi, stream)
    elif w.kind == "conv" and w.pad4:
        st = pbk.pbk_conv2d_nhwc_pad4(dev["a"], dev["b"], out, dev["bias"], w.n, w.H, w.W, w.Cin, w.Cout,
                                      w.KH, w.KW, w.stride[0], w.stride[1], *w.pad4, w.dil[0], w.dil[1],
                                      w.in_dtype, w.out_dtype, w.alpha, w.epi, stream)
    elif w.kind == "conv":
        st = pbk.pbk_conv2d_nhwc(dev["a"], dev["b"], out, dev["bias"], w.n, w.H, w.W, w.Cin, w.Cout,
                                 w.KH, w.KW, w.stride[0], w.stride[1], w.pad[0], w.pad[1],
                                 w.dil[0], w.dil[1], w.in_dtype, w.out_dtype, w.alpha, w.epi, stream)
    elif w.kind == "batched":
        ldb = k if w.trans_b else n
        st = pbk.pbk_batched_matmul(dev["a"], dev["b"], out, dev["bias"], w.batch, m, n, k,
                                    k, ldb, n, m * k, k * n, m * n, w.in_dtype, w.out_dtype,
                                    w.trans_b, w.alpha, w.epi, stream)
    else:
        ldb = k if w.trans_b else n
        st = pbk.pbk_matmul(dev["a"], dev["b"], out, dev["bias"], m, n, k, k, ldb, n,
                            w.in_dtype, w.out_dtype, w.trans_b, w.alpha, w.epi, stream)
    return st, out


def upload(host: dict) -> dict:
    return {k: (None if v is None else to_device(v)) for k, v in host.items()}


def oracle_full(w: wl.Workload, host: dict):
    """(out, preact) float64 from the CPU oracle, full tensor."""
    import oracle
    if w.kind == "conv" and w.transposed:
        return oracle.conv2d_transpose_nhwc(host["a"], host["b"], host["bias"], dtype=w.in_dtype,
                                            stride=w.stride, pad=w.pad, out_pad=w.out_pad, dil=w.dil,
                                            alpha=w.alpha, epi=w.epi, want_preact=True)
    if w.kind == "conv" and w.pad4:
        return oracle.conv2d_nhwc_pad4(host["a"], host["b"], host["bias"], dtype=w.in_dtype,
                                       stride=w.stride, pad=w.pad4, dil=w.dil, alpha=w.alpha,
                                       epi=w.epi, want_preact=True)
    if w.kind == "conv":
        return oracle.conv2d_nhwc(host["a"], host["b"], host["bias"], dtype=w.in_dtype,
                                  stride=w.stride, pad=w.pad, dil=w.dil, alpha=w.alpha,
                                  epi=w.epi, want_preact=True)
    return oracle.batched_matmul(host["a"], host["b"], host["bias"], dtype=w.in_dtype,
                                 trans_b=w.trans_b, alpha=w.alpha, epi=w.epi,
                                 batch=w.batch, M=w.M, N=w.N, K=w.K,
                                 stride_a=w.M * w.K, stride_b=w.K * w.N, want_preact=True)


def sample_coords(w: wl.Workload, count: int, seed: int = 1):
    """Output coordinates for sampled checks: tile corners/edges of every
    256-tile residue class plus uniformly random points.  Returns (b, i, j)
    in GEMM coordinates."""
    m, n, _ = w.gemm_mnk
    r = np.random.default_rng(seed)
    edge = np.array([0, 1, 31, 32, 63, 64, 127, 128, 255], dtype=np.int64)
    si = np.concatenate([edge[edge < m], m - 1 - edge[edge < m]])
    sj = np.concatenate([edge[edge < n], n - 1 - edge[edge < n]])
    gi, gj = np.meshgrid(si, sj, indexing="ij")
    gi, gj = gi.reshape(-1), gj.reshape(-1)
    ri = r.integers(0, m, size=count)
    rj = r.integers(0, n, size=count)
    i = np.concatenate([gi, ri])
    j = np.concatenate([gj, rj])
    b = r.integers(0, w.batch, size=i.size)
    b[:gi.size] = np.where(np.arange(gi.size) % 2 == 0, 0, w.batch - 1)
    return b.astype(np.int64), i.astype(np.int64), j.astype(np.int64)


def oracle_sampled(w: wl.Workload, host: dict, b, i, j):
    """(out, preact) float64 at GEMM coordinates (b, i, j)."""
    import oracle
    if w.kind == "conv":
        pix = w.OH * w.OW
        sn, rem = i // pix, i % pix
        if w.transposed:
            return oracle.conv2d_transpose_nhwc_at(host["a"], host["b"], host["bias"], sn, rem // w.OW, rem % w.OW, j,
                                                   dtype=w.in_dtype, stride=w.stride, pad=w.pad, out_pad=w.out_pad,
                                                   dil=w.dil, alpha=w.alpha, epi=w.epi)
        return oracle.conv2d_nhwc_at(host["a"], host["b"], host["bias"], sn, rem // w.OW, rem % w.OW, j,
                                     dtype=w.in_dtype, stride=w.stride, pad=w.pad, dil=w.dil,
                                     alpha=w.alpha, epi=w.epi)
    return oracle.batched_matmul_at(host["a"], host["b"], host["bias"], b, i, j, dtype=w.in_dtype,
                                    trans_b=w.trans_b, alpha=w.alpha, epi=w.epi,
                                    batch=w.batch, M=w.M, N=w.N, K=w.K)


def tile_lines(w: wl.Workload, block: int = 128, seed: int = 2):
    """One complete output row in every `block` rows and one complete output column in every `block`
    columns, of every batch entry, at seeded offsets inside the blocks: with block = 128 every
    workgroup tile of every configuration (128 or 256 on a side) is crossed by at least one full
    row and one full column.  Returns (rows, cols): row and column indices in GEMM coordinates."""
    m, n, _ = w.gemm_mnk
    r = np.random.default_rng(seed)
    rows = np.array([min(m - 1, q * block + int(r.integers(0, block))) for q in range((m + block - 1) // block)], dtype=np.int64)
    cols = np.array([min(n - 1, q * block + int(r.integers(0, block))) for q in range((n + block - 1) // block)], dtype=np.int64)
    return rows, cols


def oracle_tile_lines(w: wl.Workload, host: dict, rows, cols):
    """The oracle on the complete rows `rows` and the complete columns `cols` of every batch entry:
    (row_ref [batch][len(rows)][N], row_pre, col_ref [batch][M][len(cols)], col_pre), float64."""
    import oracle
    m, n, k = w.gemm_mnk
    if w.kind == "conv":
        assert not w.transposed and not w.pad4
        pix = w.OH * w.OW

        def at(i, j):
            sn, rem = i // pix, i % pix
            return oracle.conv2d_nhwc_at(host["a"], host["b"], host["bias"], sn, rem // w.OW, rem % w.OW, j,
                                         dtype=w.in_dtype, stride=w.stride, pad=w.pad, dil=w.dil,
                                         alpha=w.alpha, epi=w.epi)
        ri, rj = np.meshgrid(rows, np.arange(n, dtype=np.int64), indexing="ij")
        ro, rp = at(ri.reshape(-1), rj.reshape(-1))
        ci, cj = np.meshgrid(np.arange(m, dtype=np.int64), cols, indexing="ij")
        co, cp = at(ci.reshape(-1), cj.reshape(-1))
        return (ro.reshape(1, len(rows), n), rp.reshape(1, len(rows), n),
                co.reshape(1, m, len(cols)), cp.reshape(1, m, len(cols)))
    a = host["a"].reshape(w.batch, m, k)
    b = host["b"].reshape(w.batch, n, k) if w.trans_b else host["b"].reshape(w.batch, k, n)
    bias = host["bias"]
    ro = np.empty((w.batch, len(rows), n)); rp = np.empty_like(ro)
    co = np.empty((w.batch, m, len(cols))); cp = np.empty_like(co)
    for e in range(w.batch):
        ro[e], rp[e] = oracle.matmul(np.ascontiguousarray(a[e][rows]), b[e], bias, dtype=w.in_dtype,
                                     trans_b=w.trans_b, alpha=w.alpha, epi=w.epi, want_preact=True)
        bsub = np.ascontiguousarray(b[e][cols] if w.trans_b else b[e][:, cols])
        co[e], cp[e] = oracle.matmul(a[e], bsub, None if bias is None else np.ascontiguousarray(bias[cols]),
                                     dtype=w.in_dtype, trans_b=w.trans_b, alpha=w.alpha, epi=w.epi, want_preact=True)
    return ro, rp, co, cp


def gather_tile_lines(out_t, w: wl.Workload, rows, cols):
    """The same rows and columns of the device output (flat [batch][M][N]) as float64."""
    torch = torch_mod()
    m, n, _ = w.gemm_mnk
    o = out_t.view(w.batch, m, n)
    r = o[:, torch.from_numpy(rows).cuda(), :].contiguous()
    c = o[:, :, torch.from_numpy(cols).cuda()].contiguous()
    return (to_host_f64(r.view(-1), w.out_dtype).reshape(w.batch, len(rows), n),
            to_host_f64(c.view(-1), w.out_dtype).reshape(w.batch, m, len(cols)))


def gather_output(out_t, w: wl.Workload, b, i, j) -> np.ndarray:
    """Pick sampled outputs from the device tensor (flat [batch][M][N]) as float64."""
    torch = torch_mod()
    m, n, _ = w.gemm_mnk
    flat = torch.from_numpy((b * m + i) * n + j).cuda()
    return to_host_f64(out_t[flat], w.out_dtype)


# ------------------------------------------------------------------ attention

def run_attention(w: wl.AttentionWorkload, dev: dict, out=None, stream=None):
    """Enqueue the attention call on device tensors dev = {"q","k","v","bias"}
    (dense [batch][N][D] layouts).  Returns (status, out tensor)."""
    import paper_2603_06731_amd as pbk
    if out is None:
        out = device_empty(w.batch * w.Nq * w.D, w.dtype)
    if w.causal:
        st = pbk.pbk_attention_causal(dev["q"], dev["k"], dev["v"], out, w.batch, w.Nq, w.Nk, w.D,
                                      w.D, w.D, w.D, w.D, w.Nq * w.D, w.Nk * w.D, w.Nk * w.D, w.Nq * w.D,
                                      w.dtype, w.alpha, stream)
        return st, out
    ld_bias = w.Nk if w.bias != "none" else 0
    stride_bias = w.Nq * w.Nk if w.bias == "per_batch" else 0
    st = pbk.pbk_attention(dev["q"], dev["k"], dev["v"], dev["bias"], out, w.batch, w.Nq, w.Nk, w.D,
                           w.D, w.D, w.D, w.D, w.Nq * w.D, w.Nk * w.D, w.Nk * w.D, w.Nq * w.D,
                           ld_bias, stride_bias, w.dtype, w.alpha, stream)
    return st, out


def oracle_attention_full(w: wl.AttentionWorkload, host: dict) -> np.ndarray:
    import oracle
    if w.causal:
        return oracle.attention_causal(host["q"], host["k"], host["v"], dtype=w.dtype, alpha=w.alpha)
    return oracle.attention(host["q"], host["k"], host["v"], host["bias"], dtype=w.dtype, alpha=w.alpha)


def oracle_attention_rows(w: wl.AttentionWorkload, host: dict, sb, si) -> np.ndarray:
    import oracle
    if w.causal:
        return oracle.attention_causal_rows(host["q"], host["k"], host["v"], sb, si, dtype=w.dtype, alpha=w.alpha)
    return oracle.attention_rows(host["q"], host["k"], host["v"], host["bias"], sb, si,
                                 dtype=w.dtype, alpha=w.alpha)
