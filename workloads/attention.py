"""Synthetic attention-layer workloads: shapes of the paper's attention study
(batch x heads, sequence length, head size) with seeded normal tensors.
No arithmetic of the method lives here."""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

from . import gen


@dataclass(frozen=True)
class AttentionWorkload:
    name: str
    dtype: int                   # of Q, K, V and the output
    batch: int                   # batch x heads, flattened
    Nq: int
    Nk: int
    D: int
    alpha: float = 1.0           # score scale (an fp32 value)
    bias: str = "none"           # "none" | "shared" ([Nq][Nk]) | "per_batch" ([batch][Nq][Nk])
    causal: bool = False         # row i attends to keys j <= i + (Nk - Nq) only (no bias then)
    dist_q: tuple = ("normal", 1.0)
    dist_k: tuple = ("normal", 1.0)
    dist_v: tuple = ("normal", 1.0)
    dist_bias: tuple = ("normal", 1.0)
    seed: int = gen.MASTER_SEED
    note: str = field(default="", compare=False)

    @property
    def flops(self) -> int:
        """Both contractions: 2*D per (query, visible key) pair each."""
        pairs = self.Nq * self.Nk
        if self.causal:
            off = self.Nk - self.Nq
            pairs = sum(min(self.Nk, max(0, i + off + 1)) for i in range(self.Nq))
        return 4 * self.batch * pairs * self.D

    @property
    def algorithmic_bytes(self) -> int:
        """Q, K, V and the bias read once, O written once."""
        esz = 4 if self.dtype == gen.DTYPE_F32 else 2
        nb = {"none": 0, "shared": 1, "per_batch": self.batch}[self.bias]
        return esz * self.batch * (2 * self.Nq * self.D + 2 * self.Nk * self.D) + 4 * nb * self.Nq * self.Nk


def _scale(d: int) -> float:
    return float(np.float32(1.0 / math.sqrt(d)))


def _paper_shape(name, heads, n, d, dtype=gen.DTYPE_BF16, causal=False):
    return AttentionWorkload(name, dtype, heads, n, n, d, alpha=_scale(d), causal=causal)


# (batch = 1) x heads, sequence length, head size: the rows of the paper's attention table
ATTENTION_CONFIGS = {w.name: w for w in [
    _paper_shape("attn_h16_n512_d64", 16, 512, 64),
    _paper_shape("attn_h16_n2048_d64", 16, 2048, 64),
    _paper_shape("attn_h16_n8192_d64", 16, 8192, 64),
    _paper_shape("attn_h16_n512_d128", 16, 512, 128),
    _paper_shape("attn_h16_n2048_d128", 16, 2048, 128),
    _paper_shape("attn_h16_n8192_d128", 16, 8192, 128),
    _paper_shape("attn_h16_n577_d64", 16, 577, 64),
    _paper_shape("attn_h12_n10_d64", 12, 10, 64),
    _paper_shape("attn_h6_n297_d64", 6, 297, 64),
    _paper_shape("attn_h8_n500_d32", 8, 500, 32),
    _paper_shape("attn_h32_n1024_d128", 32, 1024, 128),
    # the long rows again with the decoder mask
    _paper_shape("attn_h16_n2048_d64_causal", 16, 2048, 64, causal=True),
    _paper_shape("attn_h16_n8192_d64_causal", 16, 8192, 64, causal=True),
    _paper_shape("attn_h16_n8192_d128_causal", 16, 8192, 128, causal=True),
]}


def make_attention_inputs(w: AttentionWorkload) -> dict:
    """Keys "q", "k", "v" (storage dtype) and "bias" (float32 or None).
    tensor ids: q=1, k=2, bias=3, v=4."""
    q = gen.tensor((w.batch, w.Nq, w.D), w.dtype, 1, w.dist_q[0], w.dist_q[1], w.seed)
    k = gen.tensor((w.batch, w.Nk, w.D), w.dtype, 2, w.dist_k[0], w.dist_k[1], w.seed)
    v = gen.tensor((w.batch, w.Nk, w.D), w.dtype, 4, w.dist_v[0], w.dist_v[1], w.seed)
    bias = None
    if w.bias == "shared":
        bias = gen.tensor((w.Nq, w.Nk), gen.DTYPE_F32, 3, w.dist_bias[0], w.dist_bias[1], w.seed)
    elif w.bias == "per_batch":
        bias = gen.tensor((w.batch, w.Nq, w.Nk), gen.DTYPE_F32, 3, w.dist_bias[0], w.dist_bias[1], w.seed)
    return {"q": q, "k": k, "v": v, "bias": bias}


@dataclass(frozen=True)
class Int8Workload:
    """int8 matmul C = quant_epilogue(A . B^T), both operands k-major, int8 codes out."""
    name: str
    M: int
    N: int
    K: int
    seed: int = gen.MASTER_SEED

    @property
    def flops(self) -> int:
        return 2 * self.M * self.N * self.K

    @property
    def algorithmic_bytes(self) -> int:
        return self.M * self.K + self.N * self.K + self.M * self.N + 4 * 4 * self.N


INT8_CONFIGS = {"int8_8192_nt": Int8Workload("int8_8192_nt", 8192, 8192, 8192)}


def make_int8_inputs(w: Int8Workload) -> dict:
    """Quantised activations / weights (rounded normals) and the per-channel epilogue
    parameters of the paper's fused nest: de-quantisation scale, bias, the middle
    quantise/de-quantise pair, folded batch-norm affine, ReLU, output step."""
    a = gen.int8_tensor((w.M, w.K), 1, "normal", 40.0, w.seed)
    b = gen.int8_tensor((w.N, w.K), 2, "normal", 30.0, w.seed)
    u = gen.uniform_f64(w.seed, 5, 0, w.N, 0.5, 2.0)
    scale = (u * (3.0 / (40.0 * 30.0 * math.sqrt(w.K)))).astype(np.float32)
    bias = gen.tensor((w.N,), gen.DTYPE_F32, 3, "normal", 0.5, w.seed)
    mul = gen.uniform_f64(w.seed, 6, 0, w.N, 0.5, 1.5).astype(np.float32)
    add = gen.tensor((w.N,), gen.DTYPE_F32, 7, "normal", 0.3, w.seed)
    return {"a": a, "b": b, "scale": scale, "bias": bias, "mid_scale": 0.05, "mul": mul, "add": add,
            "relu": True, "out_scale": 0.06}
