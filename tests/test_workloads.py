"""Input generator and workload table: determinism, published hash vectors,
distribution moments, byte/flop counts."""
import importlib.util
import json
import math
import os

import numpy as np

import workloads as wl
from workloads import gen


def test_splitmix64_published_vectors():
    # first three outputs of SplitMix64 seeded with 0 (reference vectors of the
    # public-domain generator): the state advances by the golden-ratio constant.
    g = 0x9E3779B97F4A7C15
    x = np.array([0, g, (2 * g) & (2 ** 64 - 1)], dtype=np.uint64)
    got = [int(v) for v in gen._splitmix64(x)]
    assert got == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_element_addressable_and_seeded():
    full = gen.normal_f64(7, 3, 0, 1000)
    part = gen.normal_f64(7, 3, 400, 50)
    assert np.array_equal(full[400:450], part)
    assert not np.array_equal(full, gen.normal_f64(8, 3, 0, 1000))
    assert not np.array_equal(full, gen.normal_f64(7, 4, 0, 1000))
    t1 = wl.tensor((5, 1 << 20), wl.DTYPE_BF16, 1, "normal")      # spans chunks
    t2 = wl.tensor((5, 1 << 20), wl.DTYPE_BF16, 1, "normal")
    assert np.array_equal(t1, t2)
    assert np.array_equal(t1.reshape(-1)[(1 << 22) - 3:(1 << 22) + 3],
                          wl.to_storage(gen.normal_f64(wl.MASTER_SEED, 1, (1 << 22) - 3, 6), wl.DTYPE_BF16))


def test_moments():
    v = gen.normal_f64(1, 1, 0, 1 << 20, std=2.0)
    assert abs(v.mean()) < 0.01 and abs(v.std() - 2.0) < 0.01
    assert abs(((v / 2.0) ** 4).mean() - 3.0) < 0.05                 # normal kurtosis
    u = gen.uniform_f64(1, 2, 0, 1 << 20)
    assert u.min() > -1 and u.max() < 1 and abs(u.mean()) < 0.005
    assert abs(u.std() - 1 / math.sqrt(3)) < 0.005


def test_storage_round_trip():
    x = np.array([1.0, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -0.3333, 65504.0, 1e-30])
    b = wl.to_storage(x, wl.DTYPE_BF16)
    assert list(b[:3]) == [0x3F80, 0x3F80, 0x3F82]
    assert np.array_equal(wl.to_storage(wl.widen(b, wl.DTYPE_BF16), wl.DTYPE_BF16), b)
    h = wl.to_storage(x[:5], wl.DTYPE_F16)
    assert np.array_equal(wl.widen(h, wl.DTYPE_F16), x[:5].astype(np.float16).astype(np.float64))


def test_fingerprint_regression(golden_dir):
    spec = importlib.util.spec_from_file_location(
        "mkfp", os.path.join(golden_dir, "make_generator_fingerprint.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    with open(os.path.join(golden_dir, "generator_fingerprint.json")) as f:
        want = json.load(f)
    assert mod.fingerprint() == want


def test_workload_counts():
    c = wl.CONFIGS
    assert c["cfg1_f32_256"].flops == 33_554_432 and c["cfg1_f32_256"].algorithmic_bytes == 787_456
    assert c["cfg2_bf16_8192"].flops == 1_099_511_627_776
    assert c["cfg2_bf16_8192"].algorithmic_bytes == 402_685_952
    assert c["cfg3_bf16_attn_scores"].flops == 68_719_476_736
    assert c["cfg3_bf16_attn_scores"].algorithmic_bytes == 603_979_776
    assert c["cfg4_bf16_mlp"].flops == 962_072_674_304
    assert c["cfg4_bf16_mlp"].algorithmic_bytes == 419_487_744
    assert c["cfg5_bf16_conv3x3"].gemm_mnk == (100352, 256, 2304)
    assert c["cfg5_bf16_conv3x3"].flops == 118_380_036_096
    assert c["cfg5_bf16_conv3x3"].algorithmic_bytes == 103_941_120


def test_make_inputs_shapes():
    w = wl.CONFIGS["cfg1_f32_256"]
    t = wl.make_inputs(w)
    assert t["a"].shape == (256, 256) and t["a"].dtype == np.float32 and t["bias"].shape == (256,)
    assert np.abs(t["a"]).max() <= 1.0
    small = wl.Workload("s", "conv", wl.DTYPE_BF16, wl.DTYPE_BF16, 3, n=2, H=5, W=6, Cin=8, Cout=4,
                        KH=3, KW=3, pad=(1, 1))
    t = wl.make_inputs(small)
    assert t["a"].shape == (2, 5, 6, 8) and t["b"].shape == (3, 3, 8, 4) and t["a"].dtype == np.uint16
