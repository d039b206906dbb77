"""Compiles the HIP sources into paper_2506_15969_amd/lib/liblazyev.so (the decode path) and
liblazyev_bench.so (plain streaming probes for measurements) for gfx950.

hipcc cross-compiles without a GPU.  Run as `python -m paper_2506_15969_amd.build`.
"""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIBDIR = os.path.join(PKG, "lib")
LIB = os.path.join(LIBDIR, "liblazyev.so")
INCLUDE = os.path.join(os.path.dirname(PKG), "include")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-I" + INCLUDE,
          # packed-fp32 VALU forms are kept out of all device code
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# the eviction file holds the bit-reproducible binary64 score: no fused multiply-add there
SOURCES = {"decode_kernels.hip": [], "decode_fused.hip": ["-mllvm", "-amdgpu-kernarg-preload-count=13"], "evict_kernels.hip": ["-ffp-contract=off"],
           "lazyev_api.hip": [], "prefill_kernels.hip": []}
# measuring aids (plain streaming probes): a library of their own, not part of the path
BENCH_LIB = os.path.join(LIBDIR, "liblazyev_bench.so")
BENCH_SOURCES = {"probe_kernels.hip": []}
# the same library with the fused decode kernel instrumented (per-block time stamps of the last
# launch; bench.py --timeline reads them): a measuring build, never what the binding loads by default
TIMELINE_LIB = os.path.join(LIBDIR, "liblazyev_timeline.so")
TIMELINE_FLAGS = ["-DLAZYEV_TIMELINE"]


def _compile(item):
    name, extra = item
    obj = os.path.join(LIBDIR, name.replace(".hip", "_timeline.o" if TIMELINE_FLAGS[0] in extra else ".o"))
    cmd = [HIPCC, *COMMON, *extra, "-c", os.path.join(CSRC, name), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (name, r.stderr))
    return obj


def build_library(verbose: bool = True) -> str:
    os.makedirs(LIBDIR, exist_ok=True)
    fused = "decode_fused.hip"
    jobs = list(SOURCES.items()) + list(BENCH_SOURCES.items()) + [(fused, SOURCES[fused] + TIMELINE_FLAGS)]
    with ThreadPoolExecutor(max_workers=len(jobs)) as ex:
        objs = list(ex.map(_compile, jobs))
    path_objs = objs[:len(SOURCES)]
    timeline_objs = [objs[-1] if o.endswith("decode_fused.o") else o for o in path_objs]
    for lib, group in ((LIB, path_objs), (BENCH_LIB, objs[len(SOURCES):-1]), (TIMELINE_LIB, timeline_objs)):
        r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *group, "-o", lib],
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
        if verbose:
            print("built", lib)
    build_c_example(verbose)
    return LIB


def build_c_example(verbose: bool = True) -> str:
    """csrc/abi_example.c: the C ABI used from plain C99 with gcc (no C++, no Python); the GPU
    test tests/test_gpu_c_abi.py runs it."""
    exe = os.path.join(LIBDIR, "abi_example")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = [os.environ.get("CC", "gcc"), "-std=c99", "-O1", "-Wall", "-Wextra", "-D__HIP_PLATFORM_AMD__",
           "-I" + os.path.join(rocm, "include"), "-I" + INCLUDE, os.path.join(CSRC, "abi_example.c"),
           "-o", exe, "-L" + LIBDIR, "-llazyev", "-L" + os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("C example failed to build:\n" + r.stderr)
    if verbose:
        print("built", exe)
    return exe


if __name__ == "__main__":
    build_library()
