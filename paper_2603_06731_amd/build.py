"""Builds libpbk.so with hipcc for gfx950 (in-tree, next to the sources)."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpbk.so")
SOURCES = ["pbk_api.hip", "gemm_generic.hip", "gemm_mfma.hip", "gemm_mfma_bf16.hip", "gemm_mfma_f16.hip",
           "gemm_mfma_fp8.hip", "gemm_mfma_fp8_e5m2.hip", "gemm_mfma_int8.hip", "gemm_mfma_f32.hip", "attention_generic.hip", "attention_mfma.hip"]
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


def _extra_flags(src: str):
    """Development aid: PBK_BUILD_CFGS="1,8" compiles only those MFMA tile
    configurations (bf16 only); the default builds everything."""
    only = os.environ.get("PBK_BUILD_CFGS")
    if not only or "gemm_mfma_" not in src:
        return []
    mask = 0
    if "bf16" in src:
        for c in only.split(","):
            mask |= 1 << int(c)
    return [f"-DPBK_CFG_MASK={mask}u"]


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    path = os.path.join(CSRC, src)
    newest = max([os.path.getmtime(path)] + [os.path.getmtime(h) for h in _headers()])
    cmd = [HIPCC, *FLAGS, *_extra_flags(src), "-c", path, "-o", obj]
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
