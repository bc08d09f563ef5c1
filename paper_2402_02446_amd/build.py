"""Builds liblqer.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree, and beside it
liblqer_probes.so: the benchmark's peak probes (streaming read, copy, MFMA loop), which are not
part of the library.

    python -m paper_2402_02446_amd.build

Objects go to paper_2402_02446_amd/_build/, the libraries to paper_2402_02446_amd/.
hipcc cross-compiles without a GPU.
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
BUILD = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "liblqer.so")
PROBES_LIB = os.path.join(PKG, "liblqer_probes.so")
PROBES_SOURCES = ["bench_probes.hip"]

SOURCES = ["lqer_host.cpp", "build_factors.cpp", "kernels_quant.hip", "kernels_prep.hip",
           "kernels_stream.hip", "kernels_tiled.hip", "kernels_build.hip", "static_entry.hip", "kernels_int.hip", "int_host.cpp"]

COMMON = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-x", "hip",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wno-unused-command-line-argument",
          "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: cannot build liblqer.so")
    return exe


def _compile(src: str, extra) -> str:
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *COMMON, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(extra_flags=(), verbose: bool = True) -> str:
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        all_objs = list(ex.map(lambda s: _compile(s, list(extra_flags)), SOURCES + PROBES_SOURCES))
    for lib, objs in ((LIB, all_objs[:len(SOURCES)]), (PROBES_LIB, all_objs[len(SOURCES):])):
        cmd = [_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", lib, *objs, "-lpthread"]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("link failed:\n" + res.stderr)
        if verbose:
            print(f"built {lib}")
    return LIB


HOST_SOURCES = ["lqer_host.cpp", "build_factors.cpp", "int_host.cpp"]
ASAN_EXE = os.path.join(BUILD, "host_selftest_asan")


def build_host_asan() -> str:
    """The library's host sources and csrc/selftest_main.cpp compiled with AddressSanitizer and UBSan (host code only;
    the kernel objects of the normal build are linked in unchanged): _build/host_selftest_asan.  Needs build() first."""
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    objs = []
    for src in HOST_SOURCES + ["selftest_main.cpp"]:
        obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".asan.o")
        cmd = [_hipcc(), *COMMON, *san, "-c", os.path.join(CSRC, src), "-o", obj]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc (sanitizers) failed on {src}:\n{res.stderr}")
        objs.append(obj)
    kern = [os.path.join(BUILD, os.path.splitext(s)[0] + ".o") for s in SOURCES if s not in HOST_SOURCES]
    cmd = [_hipcc(), "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
           "-o", ASAN_EXE, *objs, *kern, "-lpthread"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link (sanitizers) failed:\n" + res.stderr)
    return ASAN_EXE


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
