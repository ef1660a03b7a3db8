"""Builds libkvswap.so (HIP kernels + host engine + C ABI) for gfx950, in-tree.

Usage: ``python -m paper_2411_18424_amd.build``.  hipcc cross-compiles without a GPU.
"""

from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkvswap.so")
SOURCES = ["kv_kernels.hip", "kv_engine.cpp", "kv_reuse.cpp", "kvswap.cpp", "kv_probe.cpp", "kv_manager.cpp"]

# -packed-fp32-ops is switched off on purpose: packed fp32 forms are not trusted on the
# target machines.  (The library does no floating point at all, the flag is policy.)
HIP_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-pthread",
]


def build_lib(verbose: bool = True) -> str:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        raise RuntimeError("hipcc not found: cannot build libkvswap.so")
    tmp = LIB + ".tmp"
    cmd = [hipcc] + HIP_FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "packed-fp32-ops" not in l and l.strip())
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out:
        print(out, flush=True)
    os.replace(tmp, LIB)
    build_host_tests(hipcc, verbose)
    return LIB


# C / C++ callers of the ABI that the GPU tests run as programs of their own (tests/host/*.cpp):
# built here, next to the library, so that nothing is compiled on the GPU machine.
HOST_TESTS = ["host_read_check"]


def build_host_tests(hipcc: str, verbose: bool = True) -> None:
    root = os.path.dirname(HERE)
    tdir = os.path.join(root, "tests", "host")
    for name in HOST_TESTS:
        src = os.path.join(tdir, name + ".cpp")
        if not os.path.exists(src):
            continue
        exe = os.path.join(tdir, name + ".bin")
        cmd = [hipcc, "-O1", "-std=c++17", "--offload-arch=gfx950", "-Wall", "-Wno-unused-command-line-argument",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               src, "-L" + HERE, "-lkvswap", "-Wl,-rpath," + HERE, "-Wl,-rpath,$ORIGIN/../../paper_2411_18424_amd",
               "-o", exe]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (name, res.stdout))


if __name__ == "__main__":
    print(build_lib())
    sys.exit(0)
