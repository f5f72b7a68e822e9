"""Counter-based, element-addressable random tensors.

Every element is a pure function of (seed, tensor_id, flat index), so any
slice of any tensor can be regenerated anywhere with identical bits and no
generator state.  The hash is SplitMix64 (Steele, Lea & Flood 2014, the
finaliser used by java.util.SplittableRandom) applied to key + index.

Storage dtypes are numpy arrays: float32 for F32, uint16 bit patterns for
BF16 / F16 (numpy has no bfloat16), uint8 codes for the OCP FP8 formats.  Rounding to storage happens once, here.
"""
from __future__ import annotations

import numpy as np

MASTER_SEED = 20260306

DTYPE_F32 = 0
DTYPE_BF16 = 1
DTYPE_F16 = 2
DTYPE_FP8_E4M3 = 3      # OCP FP8, stored as uint8
DTYPE_FP8_E5M2 = 4

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_SECOND_STREAM = np.uint64(1 << 62)
_CHUNK = 1 << 22


def _splitmix64(x: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = x + _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def _key(seed: int, tensor_id: int) -> np.uint64:
    return np.uint64((seed ^ ((tensor_id * 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF))
                     & 0xFFFFFFFFFFFFFFFF)


def _unit(h: np.ndarray) -> np.ndarray:
    """53 random bits mapped to the open interval (0, 1)."""
    return ((h >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def uniform_f64(seed: int, tensor_id: int, start: int, count: int,
                lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    """`count` uniform doubles in (lo, hi) for flat indices start..start+count-1."""
    idx = np.arange(start, start + count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        h = _splitmix64(_key(seed, tensor_id) + idx)
    return lo + (hi - lo) * _unit(h)


def normal_f64(seed: int, tensor_id: int, start: int, count: int,
               std: float = 1.0) -> np.ndarray:
    """`count` N(0, std^2) doubles (Box-Muller on two hash streams)."""
    idx = np.arange(start, start + count, dtype=np.uint64)
    k = _key(seed, tensor_id)
    with np.errstate(over="ignore"):
        u1 = _unit(_splitmix64(k + idx))
        u2 = _unit(_splitmix64(k + idx + _SECOND_STREAM))
    return std * np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def _fp8_tables(dtype: int):
    """(sorted finite non-negative values, their codes) of an OCP FP8 format."""
    if dtype == DTYPE_FP8_E4M3:
        ebits, mbits, bias, top = 4, 3, 7, 0x7E          # 0x7F is NaN
    else:
        ebits, mbits, bias, top = 5, 2, 15, 0x7B         # 0x7C.. are inf / NaN
    codes = np.arange(0, top + 1, dtype=np.int64)
    e = codes >> mbits
    m = codes & ((1 << mbits) - 1)
    vals = np.where(e == 0, m * 2.0 ** (1 - bias - mbits), (m + (1 << mbits)) * 2.0 ** (e - bias - mbits))
    return vals, codes


def _to_fp8(x: np.ndarray, dtype: int) -> np.ndarray:
    """Round to nearest representable value, ties to the even code, saturating at
    the largest finite value (the generator never produces NaN or infinity)."""
    vals, codes = _fp8_tables(dtype)
    a = np.abs(x)
    hi = np.clip(np.searchsorted(vals, a, side="left"), 1, len(vals) - 1)
    lo = hi - 1
    dlo, dhi = a - vals[lo], vals[hi] - a
    pick_hi = (dhi < dlo) | ((dhi == dlo) & (codes[hi] % 2 == 0))
    code = np.where(pick_hi, codes[hi], codes[lo])
    code = np.where(a >= vals[-1], codes[-1], code)
    return (code | (np.signbit(x).astype(np.int64) << 7)).astype(np.uint8)


def to_storage(x: np.ndarray, dtype: int) -> np.ndarray:
    """Round doubles once to the storage dtype (round-to-nearest-even)."""
    if dtype in (DTYPE_FP8_E4M3, DTYPE_FP8_E5M2):
        return _to_fp8(x, dtype)
    if dtype == DTYPE_F32:
        return x.astype(np.float32)
    if dtype == DTYPE_F16:
        return x.astype(np.float16).view(np.uint16)
    if dtype == DTYPE_BF16:
        b = x.astype(np.float32).view(np.uint32)
        r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
        return r.astype(np.uint16)
    raise ValueError(f"unknown dtype {dtype}")


def widen(a: np.ndarray, dtype: int) -> np.ndarray:
    """Stored bits -> float64, exactly."""
    if dtype in (DTYPE_FP8_E4M3, DTYPE_FP8_E5M2):
        vals, codes = _fp8_tables(dtype)
        table = np.full(128, np.nan)
        table[codes] = vals
        if dtype == DTYPE_FP8_E5M2:
            table[0x7C] = np.inf
        mag = table[a & 0x7F]
        return np.where(a & 0x80, -mag, mag)
    if dtype == DTYPE_F32:
        return a.astype(np.float64)
    if dtype == DTYPE_F16:
        return a.view(np.float16).astype(np.float64)
    if dtype == DTYPE_BF16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype}")


def tensor(shape, dtype: int, tensor_id: int, dist: str, scale: float = 1.0,
           seed: int = MASTER_SEED) -> np.ndarray:
    """A whole tensor in storage dtype.

    dist = "normal": N(0, scale^2);  dist = "uniform": U(-scale, scale).
    Generated in chunks so the float64 temporaries stay small.
    """
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32 if dtype == DTYPE_F32 else
                   np.uint16 if dtype in (DTYPE_BF16, DTYPE_F16) else np.uint8)
    for s in range(0, n, _CHUNK):
        c = min(_CHUNK, n - s)
        if dist == "normal":
            v = normal_f64(seed, tensor_id, s, c, scale)
        elif dist == "uniform":
            v = uniform_f64(seed, tensor_id, s, c, -scale, scale)
        else:
            raise ValueError(dist)
        out[s:s + c] = to_storage(v, dtype)
    return out.reshape(shape)


def int8_tensor(shape, tensor_id: int, dist: str = "uniform", scale: float = 127.0,
                seed: int = MASTER_SEED) -> np.ndarray:
    """int8 codes: "uniform" draws every code in [-128, 127] equally often;
    "normal" rounds N(0, scale^2) to the nearest integer and saturates (the
    bell shape of quantised activations and weights)."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.int8)
    for s in range(0, n, _CHUNK):
        c = min(_CHUNK, n - s)
        if dist == "uniform":
            v = np.floor(uniform_f64(seed, tensor_id, s, c, -128.0, 128.0))
        elif dist == "normal":
            v = np.rint(normal_f64(seed, tensor_id, s, c, scale))
        else:
            raise ValueError(dist)
        out[s:s + c] = np.clip(v, -128, 127).astype(np.int8)
    return out.reshape(shape)
