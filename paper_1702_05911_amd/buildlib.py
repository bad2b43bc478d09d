"""Compiles the HIP sources in csrc/ into libpqt.so for gfx950 (cross-compiles without a GPU)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = ("pqt_api.hip", "traverse.hip", "rank_bins.hip", "rerank.hip", "exact_rerank.hip", "builder.hip", "brute_force.hip", "peaks.hip")
OUTPUT = os.path.join(HERE, "libpqt.so")


def build_library(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           # packed fp32 instructions are kept off for all device code
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-o", OUTPUT] + [os.path.join(HERE, "csrc", s) for s in SOURCES]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout + res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr)
    return OUTPUT


if __name__ == "__main__":
    print(build_library(verbose=True))
