"""Builds ``libslicegcn.so`` (the HIP kernels and their C ABI) for gfx950 with hipcc.

Cross-compiles without a GPU.  The library is written next to this file so that it travels
with the source tree; it is never installed elsewhere.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libslicegcn.so")
SOURCES = ["build_csr.hip", "order.hip", "spmm.hip", "dense.hip", "misc.hip", "loss.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed fp32 instructions stay off for every kernel in this library
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the HIP library cannot be built")
    return exe


# host code only: the device code is compiled as always (sanitizers do not run on the GPU here)
# (the checks clang's own runtime alone provides are left out: the tests preload gcc's sanitizer runtimes, which the
# oracle's sanitized build shares)
SANITIZE_HOST = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize=function",
                 "-Xarch_host", "-fno-sanitize=vptr", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
LIB_SANITIZED = os.path.join(PKG, "libslicegcn_hostsan.so")


def _compile(src: str, sanitize_host: bool = False) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".san.o" if sanitize_host else ".o"))
    cmd = [_hipcc(), *FLAGS, *(SANITIZE_HOST if sanitize_host else []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}")
    noise = "is not a recognized feature for this target"
    out = "\n".join(l for l in r.stdout.splitlines() if noise not in l and l.strip())
    if out:
        sys.stderr.write(out + "\n")
    return obj


def build(verbose: bool = True, sanitize_host: bool = False) -> str:
    """Compile every source and link the shared library.  Always rebuilds.  ``sanitize_host`` builds a second
    library whose host code carries AddressSanitizer / UndefinedBehaviorSanitizer checks (for the CPU-only tests
    of argument validation; load it with SLICEGCN_SANITIZE=1 and the sanitizer runtime preloaded)."""
    os.makedirs(OBJ, exist_ok=True)
    lib = LIB_SANITIZED if sanitize_host else LIB
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as pool:
        objs = list(pool.map(lambda s: _compile(s, sanitize_host), SOURCES))
    tmp = lib + f".tmp{os.getpid()}"
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *(["-Wl,--allow-shlib-undefined"] if sanitize_host else []),  # the sanitizer runtime comes from the preloaded libraries
           "-o", tmp, *objs]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}")
    os.replace(tmp, lib)
    if verbose:
        print(f"built {lib}")
    return lib


if __name__ == "__main__":
    build(sanitize_host="--sanitize-host" in sys.argv[1:])
