"""Builds ``libla_verify.so`` (HIP, gfx950 only) next to this file.

Every translation unit under ``csrc/`` is compiled with hipcc for gfx950 and
linked into one shared library that exports only the ``la_*`` C symbols.
Packed-fp32 instruction selection is switched off for all device code.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

HERE = Path(__file__).resolve().parent
ROOT = HERE.parent
CSRC = HERE / "csrc"
OBJ = HERE / "_build"
LIB = HERE / "libla_verify.so"

SOURCES = ["api.hip", "attn_mfma.hip", "attn_merge.hip", "attn_f32.hip", "accept.hip", "accept_static.hip", "kv_commit.hip",
           "controller.hip", "calibrate.hip"]
# -fno-honor-nans: no NaN can arise in these kernels (masked scores are -inf, handled explicitly); without it
# every fmaxf is preceded by a canonicalising v_max(x, x).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-fno-honor-nans", "-Wall",
         "-Wextra",
         "-Wno-unused-parameter", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         f"-I{ROOT / 'include'}", f"-I{CSRC}"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or Path(cand).exists()):
            return cand
    return "hipcc"


def build(verbose: bool = False, extra_flags=(), lib: Path = LIB) -> Path:
    LIB_OUT = lib
    OBJ.mkdir(exist_ok=True)
    hipcc = _hipcc()

    def compile_one(src: str) -> Path:
        obj = OBJ / (src + ".o")
        cmd = [hipcc, *FLAGS, *extra_flags, "-c", str(CSRC / src), "-o", str(obj)]
        r = subprocess.run(cmd, capture_output=True, text=True)
        # the host pass does not know the device-only target feature; that warning is expected
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    tmp = LIB_OUT.with_suffix(".so.tmp%d" % os.getpid())
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp), *map(str, objs)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    os.replace(tmp, LIB_OUT)
    return LIB_OUT


if __name__ == "__main__":
    print(build(verbose=True))
