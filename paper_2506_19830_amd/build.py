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

SOURCES = ["api.hip", "attn_mfma.hip", "attn_stream.hip", "attn_merge.hip", "attn_f32.hip", "accept.hip",
           "accept_static.hip", "kv_commit.hip", "controller.hip"]
# benchmark aids (per-kernel event timing, calibration kernels, a self-test hook): only in libla_verify_bench.so,
# which is the product library's objects linked together with these
BENCH_SOURCES = ["bench_aids.hip", "calibrate.hip"]
BENCH_LIB = HERE / "libla_verify_bench.so"
# -fno-honor-nans: no NaN can arise in these kernels (masked scores are -inf, handled explicitly); without it
# every fmaxf is preceded by a canonicalising v_max(x, x).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-fno-honor-nans", "-Wall",
         "-Wextra",
         "-Wno-unused-parameter", "-Wno-inline-asm", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         f"-I{ROOT / 'include'}", f"-I{CSRC}"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or Path(cand).exists()):
            return cand
    return "hipcc"


def build(verbose: bool = False, extra_flags=(), lib: Path = LIB, bench_lib: Path = BENCH_LIB) -> Path:
    """Compile every translation unit once and link the product library and the benchmark library from them."""
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

    all_sources = SOURCES + BENCH_SOURCES
    with ThreadPoolExecutor(max_workers=min(8, len(all_sources))) as pool:
        objs = list(pool.map(compile_one, all_sources))

    def link(out: Path, objects) -> None:
        tmp = out.with_suffix(".so.tmp%d" % os.getpid())
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp), *map(str, objects)]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stderr}")
        os.replace(tmp, out)

    link(lib, objs[:len(SOURCES)])
    link(bench_lib, objs)
    return lib


# Host-side translation units: argument validation, planning, the step-level controller, the scratch look-up of
# la_spec_accept_static.  build_host_sanitized() recompiles these with the host sanitizers (device code is compiled
# as always) and links them with the other, unchanged objects into a library for the CPU test that exercises
# every host path under AddressSanitizer and UndefinedBehaviorSanitizer.
HOST_SOURCES = ["api.hip", "controller.hip", "accept_static.hip"]


def asan_runtime() -> Path:
    """The shared AddressSanitizer runtime of hipcc's clang (to be preloaded into the process that loads the library)."""
    hipcc = _hipcc()
    r = subprocess.run([hipcc, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    cand = Path(r.stdout.strip())
    if cand.is_file():
        return cand
    for cand in Path("/opt/rocm/lib/llvm/lib/clang").glob("*/lib/linux/libclang_rt.asan-x86_64.so"):
        return cand
    raise FileNotFoundError("libclang_rt.asan-x86_64.so")


def build_host_sanitized(out: Path) -> Path:
    """``out``: the library with its host-only translation units built with -fsanitize=address,undefined."""
    if not all((OBJ / (src + ".o")).exists() for src in SOURCES):
        build()
    hipcc = _hipcc()
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined", "-g"]
    objs = []
    for src in SOURCES:
        if src not in HOST_SOURCES:
            objs.append(OBJ / (src + ".o"))
            continue
        obj = out.parent / (src + ".san.o")
        flags = [f for f in FLAGS if f != "-O3"] + ["-O1"]
        r = subprocess.run([hipcc, *flags, *san, "-c", str(CSRC / src), "-o", str(obj)], capture_output=True,
                           text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc (sanitized) failed on {src}:\n{r.stderr}")
        objs.append(obj)
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address",
                        "-fsanitize=undefined", "-shared-libsan", "-o", str(out), *map(str, objs)],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link (sanitized) failed:\n{r.stderr}")
    return out


if __name__ == "__main__":
    print(build(verbose=True))
