"""Builds libhfr.so in-tree with hipcc for gfx950 (cross-compiles without a GPU).

    python -m paper_2408_14158_amd.build [--incremental]
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhfr.so")
OBJ_DIR = os.path.join(HERE, "_build")

# slowest first (measured compile times): the pool starts them in this order, so the long units do not
# end up alone at the tail of the build
_TYPES = ["bf16", "e4m3", "e5m2", "f16", "f32"]
SOURCES = (["hfr_launch_%s_skewed.hip" % t for t in _TYPES[:4]] + ["hfr_launch_bf16.hip"] +
           ["hfr_launch_%s_skewed3.hip" % t for t in _TYPES[:4]] + ["hfr_launch_f32_skewed.hip"] +
           ["hfr_launch_e4m3.hip", "hfr_launch_e5m2.hip", "hfr_launch_f16.hip", "hfr_launch_f32_skewed3.hip"] +
           ["hfr_launch_bf16_many.hip", "hfr_launch_copy.hip", "hfr_launch_f32.hip"] +
           ["hfr_launch_%s_many.hip" % t for t in ("e4m3", "e5m2", "f16", "f32")] +
           ["hfr_launch_%s_list.hip" % t for t in _TYPES] +
           ["hfr_noalloc.hip", "hfr_api.cpp", "hfr_sched.cpp"])

# -ffp-contract=off: the add and the scale multiply must stay two roundings.
# packed-fp32 instructions are switched off for the device pass.
COMMON = ["-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-fno-fast-math", "-Wall"]
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _headers_mtime() -> float:
    inc = os.path.join(os.path.dirname(HERE), "include")
    hs = [os.path.join(d, f) for d in (CSRC, inc) for f in os.listdir(d) if f.endswith(".h")]
    return max(os.path.getmtime(h) for h in hs)


def _compile(src: str, incremental: bool = False) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    if incremental and os.path.exists(obj):
        # a host-only unit sees the plain headers only; a device unit every header
        newest = max(os.path.getmtime(path), _headers_mtime() if src.endswith(".hip") else max(
            os.path.getmtime(os.path.join(CSRC, "hfr_internal.h")),
            os.path.getmtime(os.path.join(os.path.dirname(HERE), "include", "hfr.h"))))
        if os.path.getmtime(obj) > newest:
            return obj
    if src.endswith(".hip"):
        cmd = [hipcc(), *COMMON, *DEVICE, "-c", path, "-o", obj]
    else:
        # host-only translation units: HIP headers, no device pass
        cmd = [hipcc(), *COMMON, "-x", "c++", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
               "-c", path, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("compile failed: %s\n%s" % (" ".join(cmd), r.stderr))
    return obj


def build(verbose: bool = True, incremental: bool = False) -> str:
    """Compiles every translation unit (incremental=True: only those older than
    their source or a header they include) and links libhfr.so."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(lambda src: _compile(src, incremental), SOURCES))
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed: %s\n%s" % (" ".join(cmd), r.stderr))
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


PROBE_LIB = os.path.join(HERE, "libhfr_probe.so")


def build_probe(verbose: bool = True) -> str:
    """The benchmark's streaming probes (csrc/hfr_probe.hip), a library of their own."""
    tmp = PROBE_LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), "-O3", "-std=c++17", "-fPIC", "-Wall", *DEVICE, "-shared",
           os.path.join(CSRC, "hfr_probe.hip"), "-o", tmp]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("probe build failed: %s\n%s" % (" ".join(cmd), r.stderr))
    os.replace(tmp, PROBE_LIB)
    if verbose:
        print("built", PROBE_LIB)
    return PROBE_LIB


EXAMPLE_SRC = os.path.join(HERE, "examples", "c_abi_example.c")
EXAMPLE_BIN = os.path.join(OBJ_DIR, "c_abi_example")


def build_example(verbose: bool = True) -> str:
    """The plain-C example program, linked against libhfr.so and the ROCm HIP runtime."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c99", "-O2", "-Wall", "-Wextra", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(os.path.dirname(HERE), "include"), "-I", os.path.join(rocm, "include"),
           EXAMPLE_SRC, "-o", EXAMPLE_BIN, "-L", HERE, "-lhfr", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/..", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("example build failed: %s\n%s" % (" ".join(cmd), r.stderr))
    if verbose:
        print("built", EXAMPLE_BIN)
    return EXAMPLE_BIN


if __name__ == "__main__":
    build(incremental="--incremental" in sys.argv[1:])
    build_probe()
    build_example()
    sys.exit(0)
