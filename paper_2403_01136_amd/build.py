"""Build liblpq.so (the HIP library behind include/lpq.h) for gfx950 with hipcc.

Usage: python -m paper_2403_01136_amd.build   (or build_library() from Python).
The library is built in-tree next to this file; it links only against the HIP runtime.
"""
import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblpq.so")
SOURCES = ["lpq_api.cpp", "lpq_quantize.hip", "lpq_decode.hip", "lpq_prefill.hip", "lpq_layer.hip", "lpq_indicator.hip", "lpq_planner.cpp"]
# packed-fp32 VALU forms are switched off for every device function of this library
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-attributes"]


def _compile(src, extra):
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc"] + FLAGS + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
    subprocess.check_call(cmd)
    return obj


def build_library(extra_flags=(), verbose=False):
    hipcc = subprocess.run(["which", "hipcc"], capture_output=True, text=True).stdout.strip()
    if not hipcc:
        raise RuntimeError("hipcc not found on PATH; the HIP library cannot be built")
    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(lambda s: _compile(s, list(extra_flags)), SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs + ["-Wl,-rpath,/opt/rocm/lib"]
    subprocess.check_call(cmd)
    if verbose:
        print("built", LIB)
    return LIB


def build_probe(verbose=False):
    """The issue-rate probe (csrc/probe_issue_rates.hip): a stand-alone measuring tool, not linked into the library."""
    exe = os.path.join(HERE, "probe_issue_rates")
    subprocess.check_call(["hipcc"] + [f for f in FLAGS if f != "-fPIC"] + [os.path.join(CSRC, "probe_issue_rates.hip"), "-o", exe])
    if verbose:
        print("built", exe)
    return exe


if __name__ == "__main__":
    build_library(sys.argv[1:], verbose=True)
    build_probe(verbose=True)
