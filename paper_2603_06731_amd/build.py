"""Builds libpbk.so with hipcc for gfx950 (in-tree, next to the sources)."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpbk.so")
# (source, object stem, extra defines).  The 16-bit kernels compile once per element type and group of
# tile configurations (csrc/gemm_mfma_launch.h: kGroupMask16), in parallel.
N_GROUPS_16 = 5
# (the units that take longest to compile come first: the pool starts them first)
SOURCES = [("gemm_mfma_fp8_tu.hip", f"gemm_mfma_fp8_{name}_{out}",
            [f"-DPBK_FP8_TYPE=fp8_{name}_t", f"-DPBK_FP8_NAME={name}", f"-DPBK_FP8_OUT={out}_t", f"-DPBK_FP8_OUTNAME={out}"])
           for name in ("e4m3", "e5m2") for out in ("bf16", "f16")]
SOURCES += [("gemm_mfma_int8.hip", "gemm_mfma_int8", [])]
SOURCES += [("gemm_mfma_16bit.hip", f"gemm_mfma_{name}_g{g}",
             [f"-DPBK_16BIT_TYPE={name}_t", f"-DPBK_16BIT_NAME={name}", f"-DPBK_GROUP={g}"])
            for g in reversed(range(N_GROUPS_16)) for name in ("bf16", "f16")]
SOURCES += [(f, f[:-4], []) for f in ("gemm_mfma_bstat.hip", "gemm_mfma_gather.hip", "gemm_mfma_f32.hip", "attention_mfma.hip", "gemm_mfma_fp8.hip",
                                      "gemm_mfma.hip", "pbk_api.hip", "gemm_generic.hip", "gemm_small_f32.hip",
                                      "attention_generic.hip")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument",
         # M0 is on the clobber list of the direct-to-LDS load statements; the compiler notes that it is a reserved register
         "-Wno-inline-asm"]


def _headers():
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hs.append(os.path.join(os.path.dirname(HERE), "include", "pbk.h"))
    return hs


def _extra_flags(stem: str):
    """Development aid: PBK_BUILD_CFGS="6,9" compiles only those tile configurations of the 16-bit
    types, and with PBK_BUILD_TYPES="bf16" only that type; the default builds everything."""
    only = os.environ.get("PBK_BUILD_CFGS")
    if not only or "_g" not in stem:
        return []
    mask = 0
    types = os.environ.get("PBK_BUILD_TYPES", "bf16,f16").split(",")
    if any(f"_{t}_" in stem for t in types):
        for c in only.split(","):
            mask |= 1 << int(c)
    return [f"-DPBK_DEV_MASK={mask}u"]


def _compile(src, force: bool) -> str:
    name, stem, defines = src
    obj = os.path.join(CSRC, stem + ".o")
    path = os.path.join(CSRC, name)
    newest = max([os.path.getmtime(path)] + [os.path.getmtime(h) for h in _headers()])
    cmd = [HIPCC, *FLAGS, *defines, *_extra_flags(stem), "-c", path, "-o", obj]
    stamp = obj + ".cmd"                     # the command line the object was built with
    same_cmd = os.path.exists(stamp) and open(stamp).read() == " ".join(cmd)
    if force or not same_cmd or not os.path.exists(obj) or os.path.getmtime(obj) < newest:
        subprocess.check_call(cmd, stderr=subprocess.DEVNULL if os.environ.get("PBK_BUILD_QUIET") else None)
        with open(stamp, "w") as f:
            f.write(" ".join(cmd))
    return obj


def build(force: bool = False, jobs: int = 8) -> str:
    """Compile every HIP source for gfx950 and link libpbk.so.  `force`
    recompiles even if objects look current."""
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < max(os.path.getmtime(o) for o in objs):
        tmp = LIB + f".tmp{os.getpid()}"
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(force="--force" in sys.argv))
