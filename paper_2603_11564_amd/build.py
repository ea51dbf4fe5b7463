"""Builds libdapq.so (the HIP kernels and their C ABI) for gfx950, in-tree, with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libdapq.so")
# measurement support for `bench.py --ceilings` (stream and instruction-issue probes); not part of the eviction path
CEILING_LIB = os.path.join(PKG, "libdapq_ceiling.so")
CEILING_SOURCES = ["ceiling.hip"]
SOURCES = ["common.hip", "rope.hip", "score.hip", "pool.hip", "topk.hip", "gather.hip", "recall.hip", "decode.hip", "qproj.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    # packed fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # MFMA results live in ordinary vector registers: the vector ALU reads every one of them
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
    '-DDAPQ_API=__attribute__((visibility("default")))',
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


# Host-side sanitizers for the library's host code (argument checks, launch plans, workspace carving); the device
# code is compiled as usual.  Used by tests/test_host_sanitizers.py, which runs the host boundary tests against it.
SANITIZE_FLAGS = ["-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                  "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
SANITIZED_LIB = os.path.join(PKG, "_build", "san", "libdapq_san.so")


def asan_runtime() -> str:
    """Path of the AddressSanitizer runtime a process must preload to use the sanitized library."""
    r = subprocess.run([_hipcc(), "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    path = r.stdout.strip()
    if r.returncode != 0 or not os.path.isabs(path) or not os.path.exists(path):
        raise RuntimeError("the AddressSanitizer runtime of hipcc's clang was not found")
    return path


def build_sanitized(verbose: bool = False) -> str:
    """libdapq.so again with AddressSanitizer and UndefinedBehaviorSanitizer on its host code; returns its path."""
    hipcc = _hipcc()
    objdir = os.path.dirname(SANITIZED_LIB)
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src: str) -> str:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        r = subprocess.run([hipcc, *FLAGS, *SANITIZE_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj],
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src} (sanitized):\n{r.stderr[-4000:]}")
        if verbose:
            print(f"compiled {src} (sanitized host code)", flush=True)
        return obj

    with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
                        "-shared-libsan", "-o", SANITIZED_LIB, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link of {os.path.basename(SANITIZED_LIB)} failed:\n{r.stderr[-4000:]}")
    return SANITIZED_LIB


def build(verbose: bool = False) -> str:
    """Compile every translation unit and link the shared library; returns its path."""
    hipcc = _hipcc()
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src: str) -> str:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr[-4000:]}")
        if verbose:
            print(f"compiled {src}", flush=True)
        return obj

    with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(compile_one, SOURCES + CEILING_SOURCES))
    for lib, lib_objs in ((LIB, objs[:len(SOURCES)]), (CEILING_LIB, objs[len(SOURCES):])):
        r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *lib_objs],
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link of {os.path.basename(lib)} failed:\n{r.stderr[-4000:]}")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
