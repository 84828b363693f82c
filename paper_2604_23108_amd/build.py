"""Builds the two shared libraries in-tree with hipcc for gfx950: libmohge.so (the C-ABI layer
library, include/mohge.h) and libmohge_bench.so (measurement and test aids, include/mohge_bench.h,
linked against the first)."""
from __future__ import annotations

import concurrent.futures as cf
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libmohge.so")
BENCH_LIB = os.path.join(HERE, "libmohge_bench.so")
OBJDIR = os.path.join(HERE, "_build")

SOURCES = ["api.hip", "route.hip", "permute.hip", "ffn.hip", "ffn_tiled.hip", "ffn_skinny.hip",
           "combine.hip", "aux_loss.hip", "ffn_bwd.hip", "route_bwd.hip", "decode_layer.hip"]
BENCH_SOURCES = ["bench_api.hip", "box_probe.hip"]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", INCLUDE, "-I", CSRC,
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJDIR, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    p = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in p.stderr.splitlines() if noise not in l)
    if p.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def _link(out: str, objs, extra=()) -> None:
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs, *extra]
    p = subprocess.run(cmd, capture_output=True, text=True)
    if p.returncode != 0:
        raise RuntimeError("link failed:\n" + p.stderr)


def build(verbose: bool = False) -> str:
    os.makedirs(OBJDIR, exist_ok=True)
    with cf.ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(_compile, SOURCES + BENCH_SOURCES))
    _link(LIB, objs[:len(SOURCES)])
    # the benchmark library finds libmohge.so next to itself
    _link(BENCH_LIB, objs[len(SOURCES):], ["-L", HERE, "-lmohge", "-Wl,-rpath,$ORIGIN"])
    if verbose:
        print("built", LIB, "and", BENCH_LIB)
    return LIB


# ---- host code under AddressSanitizer + UndefinedBehaviorSanitizer -------------------------------
# Separate files (never loaded by the package): the same sources with the HOST pass instrumented
# (device code is compiled as usual; sanitizers for GPU code are not used).  A process that loads
# them needs the sanitizer runtime first in its library list: run it with LD_PRELOAD=asan_runtime().
SAN_DIR = os.path.join(HERE, "_build_san")
SAN_LIB = os.path.join(SAN_DIR, "libmohge.so")
SAN_BENCH_LIB = os.path.join(SAN_DIR, "libmohge_bench.so")
SAN_FLAGS = ["-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]


def asan_runtime() -> str:
    """Path of the shared AddressSanitizer runtime of the compiler hipcc drives ('' if absent)."""
    p = subprocess.run(["hipcc", "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    path = p.stdout.strip()
    return path if p.returncode == 0 and os.path.isabs(path) and os.path.exists(path) else ""


def _compile_san(src: str) -> str:
    obj = os.path.join(SAN_DIR, src.replace(".hip", ".o"))
    p = subprocess.run(["hipcc", *FLAGS, *SAN_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj],
                       capture_output=True, text=True)
    if p.returncode != 0:
        raise RuntimeError(f"hipcc (sanitized host pass) failed for {src}:\n{p.stderr}")
    return obj


def build_sanitized() -> str:
    os.makedirs(SAN_DIR, exist_ok=True)
    with cf.ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(_compile_san, SOURCES + BENCH_SOURCES))
    san = ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan"]
    _link(SAN_LIB, objs[:len(SOURCES)], san)
    _link(SAN_BENCH_LIB, objs[len(SOURCES):], san + ["-L", SAN_DIR, "-lmohge", "-Wl,-rpath,$ORIGIN"])
    return SAN_LIB


if __name__ == "__main__":
    build(verbose=True)
