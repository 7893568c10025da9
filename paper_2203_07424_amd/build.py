"""Builds the gfx950 library in-tree with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "librec_mi355x.so")

SOURCES = ["scan.hip", "pool.hip", "pool_hot.hip", "gemm.hip", "gemm_big.hip", "mlp_chain.hip", "interact.hip", "synth_fill.hip", "probe.hip", "rec_api.hip"]

# The packed-fp32 target feature is switched off for all device code.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc() -> str:
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


# Host half under AddressSanitizer and UndefinedBehaviorSanitizer (device code
# as usual): for CPU-only checks of argument validation and model bookkeeping.
OBJ_SAN = os.path.join(PKG, "_build_san")
LIB_SAN = os.path.join(PKG, "librec_mi355x_hostsan.so")
SAN_FLAGS = ["-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer"]


def _compile(src: str, force: bool, sanitize: bool = False) -> str:
    s = os.path.join(CSRC, src)
    o = os.path.join(OBJ_SAN if sanitize else OBJ, src + ".o")
    deps = [s, os.path.join(CSRC, "rec_internal.h"), os.path.join(CSRC, "mlp_chain_body.h"),
            os.path.join(ROOT, "include", "rec.h"),
            os.path.join(ROOT, "include", "rec_synth.h"), os.path.join(ROOT, "include", "rec_probe.h"),
            os.path.abspath(__file__)]
    if not force and os.path.exists(o) and all(os.path.getmtime(o) >= os.path.getmtime(d) for d in deps):
        return o
    r = subprocess.run([_hipcc(), *FLAGS, *(SAN_FLAGS if sanitize else []), "-c", s, "-o", o],
                       capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return o


def build(force: bool = True, jobs: int = 6) -> str:
    """Compile every kernel for gfx950 and link the shared library."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    r = subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


def build_host_sanitized(force: bool = False, jobs: int = 6) -> str:
    """The same library with its host code instrumented.  A process that loads it
    needs clang's sanitizer runtime preloaded (sanitizer_runtime())."""
    os.makedirs(OBJ_SAN, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, True), SOURCES))
    r = subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address",
                        "-fsanitize=undefined", "-shared-libsan", "-o", LIB_SAN, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB_SAN


def sanitizer_runtime() -> str:
    """Path of the AddressSanitizer runtime the instrumented host code needs."""
    r = subprocess.run([_hipcc(), "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    return r.stdout.strip()


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
