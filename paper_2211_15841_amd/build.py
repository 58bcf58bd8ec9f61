"""Builds libdmoe.so (the C-ABI library of include/dmoe.h) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdmoe.so")
SOURCES = ["api.hip", "bsmm_api.hip", "routing.hip", "permute.hip", "bsmm.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    # packed-fp32 VALU forms are kept out of all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    # the direct-to-LDS load asm names m0 (a reserved register it rewrites) as clobbered; the note about that is expected
    "-Wno-inline-asm",
]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                     if "packed-fp32-ops" not in l or "error" in l)
    if r.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), msgs))
    return msgs


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source and link libdmoe.so.  Always recompiles when force=True."""
    os.makedirs(BUILD, exist_ok=True)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(HERE, "..", "include", "dmoe.h")]
    newest = max(os.path.getmtime(p) for p in deps)
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= newest:
        return LIB
    objs = [os.path.join(BUILD, s.replace(".hip", ".o")) for s in SOURCES]

    def compile_one(pair):
        src, obj = pair
        return _run([HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])

    with ThreadPoolExecutor(max_workers=4) as ex:
        outs = list(ex.map(compile_one, zip(SOURCES, objs)))
    if verbose:
        for o in outs:
            if o.strip():
                print(o, file=sys.stderr)
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


HOST_CHECKED_LIB = os.path.join(BUILD, "libdmoe_hostcheck.so")
# the host pass of the two C-ABI source files under the undefined-behaviour sanitizer in trapping form (no runtime
# library needed: a signed overflow, an out-of-bounds index of a fixed array, a bad shift or a misaligned access in the
# size and layout arithmetic ends the process); device code is compiled as always
HOST_CHECK_FLAGS = ["-Xarch_host", "-fsanitize=undefined,bounds", "-Xarch_host", "-fsanitize-trap=all",
                    "-Xarch_host", "-fno-sanitize=function,vptr"]


def build_host_checked() -> str:
    """libdmoe_hostcheck.so: api.hip and bsmm_api.hip with their host code sanitized, the kernel files as in libdmoe.so."""
    os.makedirs(BUILD, exist_ok=True)
    objs = []
    for src in SOURCES:
        checked = src in ("api.hip", "bsmm_api.hip")
        obj = os.path.join(BUILD, src.replace(".hip", ".hostcheck.o" if checked else ".o"))
        if checked or not os.path.exists(obj):
            _run([HIPCC, *FLAGS, *(HOST_CHECK_FLAGS if checked else []), "-c", os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", HOST_CHECKED_LIB, *objs])
    return HOST_CHECKED_LIB


VENDOR_BENCH = os.path.join(BUILD, "bench_vendor_bmm")


def build_vendor_bench() -> str:
    """Compile the stand-alone rocBLAS batched-GEMM timing program (the vendor side of the Figure-9 comparison)."""
    os.makedirs(BUILD, exist_ok=True)
    src = os.path.join(HERE, "..", "bench_vendor_bmm.cpp")
    _run([HIPCC, "--offload-arch=gfx950", "-O2", "-Wno-unused-result", src, "-L/opt/rocm/lib", "-lrocblas",
          "-Wl,-rpath,/opt/rocm/lib", "-o", VENDOR_BENCH])
    return VENDOR_BENCH


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
    print(build_vendor_bench())
