"""Compiles the HIP sources in csrc/ into libpqt.so for gfx950 (cross-compiles without a GPU)."""
import os
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = ("pqt_api.hip", "pqt_host.cpp", "traverse.hip", "rank_bins.hip", "rerank.hip",
           # the re-rank kernel, one translation unit per code width (they compile side by side)
           "rerank_table2.hip", "rerank_table0.hip", "rerank_table1.hip", "rerank_table4.hip", "rerank_table8.hip",
           "rerank_pair_bytes.hip", "rerank_pair2.hip", "rerank_pair4.hip", "rerank_pair8.hip",
           "exact_rerank.hip", "builder.hip", "train.hip", "brute_force.hip", "peaks.hip")
OUTPUT = os.path.join(HERE, "libpqt.so")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # packed fp32 instructions are kept off for all device code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# host-only sources (no GPU code in them; the same files also build into the CPU sanitizer test program)
HOST_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-ffp-contract=off"]


def build_library(verbose=False, jobs=None):
    """One hipcc process per source file (they are independent translation units), then the link."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    jobs = jobs or min(len(SOURCES), os.cpu_count() or 1, 16)
    log = []

    def run(cmd):
        res = subprocess.run(cmd, capture_output=True, text=True)
        log.append(res.stdout + res.stderr)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + res.stderr)

    with tempfile.TemporaryDirectory(prefix="pqt_build_") as tmp:
        objects = [os.path.join(tmp, os.path.splitext(s)[0] + ".o") for s in SOURCES]
        with ThreadPoolExecutor(max_workers=jobs) as pool:
            list(pool.map(lambda so: run([hipcc] + (HOST_FLAGS if so[0].endswith(".cpp") else FLAGS) +
                                         ["-c", os.path.join(HERE, "csrc", so[0]), "-o", so[1]]),
                          zip(SOURCES, objects)))
        run([hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", "-o", OUTPUT] + objects)
    if verbose:
        print("".join(log))
    return OUTPUT


if __name__ == "__main__":
    print(build_library(verbose=True))
