"""The five synthetic workloads and reduced-size relatives used by tests.

Shapes, dtypes, value distributions and the fused epilogue of each workload
are fixed here; tensors are drawn with workloads.gen.  Integer codes for
dtypes and epilogues are the ones both C interfaces use.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

from . import gen

# epilogue codes (out = act(alpha * acc + bias[n]))
EPI_NONE = 0
EPI_BIAS = 1
EPI_RELU = 2
EPI_BIAS_RELU = 3
EPI_BIAS_GELU_TANH = 4
EPI_GELU_TANH = 5

EPI_HAS_BIAS = {EPI_BIAS, EPI_BIAS_RELU, EPI_BIAS_GELU_TANH}


@dataclass(frozen=True)
class Workload:
    name: str
    kind: str                    # "matmul" | "batched" | "conv"
    in_dtype: int
    out_dtype: int
    epi: int
    alpha: float = 1.0
    # matmul / batched
    batch: int = 1
    M: int = 0
    N: int = 0
    K: int = 0
    trans_b: int = 0
    # conv (NHWC image, HWIO weights)
    n: int = 0
    H: int = 0
    W: int = 0
    Cin: int = 0
    Cout: int = 0
    KH: int = 1
    KW: int = 1
    stride: tuple = (1, 1)
    pad: tuple = (0, 0)
    dil: tuple = (1, 1)
    pad4: tuple = None           # (top, bottom, left, right) instead of `pad`
    transposed: int = 0          # transposed convolution (uses pad, out_pad)
    out_pad: tuple = (0, 0)
    # distributions: (dist, scale) per tensor
    dist_a: tuple = ("normal", 1.0)
    dist_b: tuple = ("normal", 1.0)
    dist_bias: tuple = ("normal", 0.1)
    seed: int = gen.MASTER_SEED
    note: str = field(default="", compare=False)

    # ---- derived sizes -------------------------------------------------
    @property
    def OH(self) -> int:
        if self.transposed:
            return (self.H - 1) * self.stride[0] - 2 * self.pad[0] + self.dil[0] * (self.KH - 1) + self.out_pad[0] + 1
        both = self.pad4[0] + self.pad4[1] if self.pad4 else 2 * self.pad[0]
        return (self.H + both - self.dil[0] * (self.KH - 1) - 1) // self.stride[0] + 1

    @property
    def OW(self) -> int:
        if self.transposed:
            return (self.W - 1) * self.stride[1] - 2 * self.pad[1] + self.dil[1] * (self.KW - 1) + self.out_pad[1] + 1
        both = self.pad4[2] + self.pad4[3] if self.pad4 else 2 * self.pad[1]
        return (self.W + both - self.dil[1] * (self.KW - 1) - 1) // self.stride[1] + 1

    @property
    def gemm_mnk(self):
        """(M, N, K) of the contraction, per batch entry."""
        if self.kind == "conv":
            return (self.n * self.OH * self.OW, self.Cout, self.KH * self.KW * self.Cin)
        return (self.M, self.N, self.K)

    @property
    def flops(self) -> int:
        m, n, k = self.gemm_mnk
        return 2 * m * n * k * self.batch

    @property
    def algorithmic_bytes(self) -> int:
        """Each operand read once, bias read once, output written once."""
        esz_in = {gen.DTYPE_F32: 4, gen.DTYPE_BF16: 2, gen.DTYPE_F16: 2}.get(self.in_dtype, 1)
        esz_out = 4 if self.out_dtype == gen.DTYPE_F32 else 2
        m, n, k = self.gemm_mnk
        if self.kind == "conv":
            a = self.n * self.H * self.W * self.Cin
            b = k * n
        else:
            a = self.batch * m * k
            b = self.batch * k * n
        bias = 4 * n if self.epi in EPI_HAS_BIAS else 0
        return esz_in * (a + b) + bias + esz_out * self.batch * m * n


_F32, _BF16, _F16 = gen.DTYPE_F32, gen.DTYPE_BF16, gen.DTYPE_F16

CONFIGS = {
    "cfg1_f32_256": Workload(
        "cfg1_f32_256", "matmul", _F32, _F32, EPI_BIAS_RELU, M=256, N=256, K=256,
        dist_a=("uniform", 1.0), dist_b=("uniform", 1.0), dist_bias=("uniform", 1.0)),
    "cfg2_bf16_8192": Workload(
        "cfg2_bf16_8192", "matmul", _BF16, _BF16, EPI_BIAS_RELU, M=8192, N=8192, K=8192,
        dist_a=("normal", 1.0 / math.sqrt(8192)), dist_b=("normal", 1.0 / math.sqrt(8192)),
        dist_bias=("normal", 0.1)),
    "cfg3_bf16_attn_scores": Workload(
        "cfg3_bf16_attn_scores", "batched", _BF16, _BF16, EPI_NONE,
        alpha=float(np.float32(1.0 / math.sqrt(128.0))), batch=64, M=2048, N=2048, K=128),
    "cfg4_bf16_mlp": Workload(
        "cfg4_bf16_mlp", "matmul", _BF16, _BF16, EPI_BIAS_GELU_TANH, M=8192, N=14336, K=4096,
        dist_a=("normal", 1.0), dist_b=("normal", 1.0 / 64.0), dist_bias=("normal", 0.1)),
    "cfg5_bf16_conv3x3": Workload(
        "cfg5_bf16_conv3x3", "conv", _BF16, _BF16, EPI_BIAS_RELU, n=32, H=56, W=56,
        Cin=256, Cout=256, KH=3, KW=3, stride=(1, 1), pad=(1, 1),
        dist_a=("normal", 1.0), dist_b=("normal", math.sqrt(2.0 / 2304.0)),
        dist_bias=("normal", 0.1)),
}


# Further workloads beyond the five headline ones (widening per the scope table's "next" rows).
EXTRA_CONFIGS = {
    "fp8_e4m3_8192_nt": Workload(
        "fp8_e4m3_8192_nt", "matmul", gen.DTYPE_FP8_E4M3, _BF16, EPI_BIAS_RELU, M=8192, N=8192, K=8192,
        trans_b=1, dist_a=("normal", 1.0), dist_b=("normal", 1.0 / math.sqrt(8192)),
        dist_bias=("normal", 0.1)),
    # score product with a head dimension of 256 (the shape of cfg3 with twice the contraction)
    "bf16_attn_scores_d256": Workload(
        "bf16_attn_scores_d256", "batched", _BF16, _BF16, EPI_NONE,
        alpha=float(np.float32(1.0 / math.sqrt(256.0))), batch=64, M=2048, N=2048, K=256),
    # pointwise convolution of a bottleneck block (64 -> 256 channels at 56 x 56): the matmul [N H W][64] x [64][256]
    "bf16_conv1x1_64_256": Workload(
        "bf16_conv1x1_64_256", "conv", _BF16, _BF16, EPI_BIAS_RELU, n=128, H=56, W=56,
        Cin=64, Cout=256, KH=1, KW=1, stride=(1, 1), pad=(0, 0),
        dist_a=("normal", 1.0), dist_b=("normal", math.sqrt(2.0 / 64.0)), dist_bias=("normal", 0.1)),
}


def make_inputs(w: Workload) -> dict:
    """Draw the workload's tensors (storage dtype, numpy, host memory).

    Keys: "a" (A or image), "b" (B or weights), "bias" (float32 or None).
    tensor ids: a=1, b=2, bias=3.
    """
    m, n, k = w.gemm_mnk
    if w.kind == "conv":
        a_shape = (w.n, w.H, w.W, w.Cin)
        b_shape = (w.KH, w.KW, w.Cin, w.Cout)
    elif w.kind == "batched":
        a_shape = (w.batch, m, k)
        b_shape = (w.batch, n, k) if w.trans_b else (w.batch, k, n)
    else:
        a_shape = (m, k)
        b_shape = (n, k) if w.trans_b else (k, n)
    a = gen.tensor(a_shape, w.in_dtype, 1, w.dist_a[0], w.dist_a[1], w.seed)
    b = gen.tensor(b_shape, w.in_dtype, 2, w.dist_b[0], w.dist_b[1], w.seed)
    bias = None
    if w.epi in EPI_HAS_BIAS:
        bias = gen.tensor((n,), gen.DTYPE_F32, 3, w.dist_bias[0], w.dist_bias[1], w.seed)
    return {"a": a, "b": b, "bias": bias}
