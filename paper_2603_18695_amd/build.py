"""Build libks_scan.so in-tree with hipcc for gfx950 (no GPU needed)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libks_scan.so")
# a pair defined outside the library, as a caller would (examples/user_pair.hip); the GPU tests load it
USER_SRC = os.path.join(HERE, "examples", "user_pair.hip")
USER_LIB = os.path.join(HERE, "examples", "libks_user_pair.so")
# the C ABI from a program without Python (examples/scan_from_c.cpp); a GPU test runs it
C_EXAMPLE_SRC = os.path.join(HERE, "examples", "scan_from_c.cpp")
C_EXAMPLE = os.path.join(HERE, "examples", "scan_from_c")
SOURCES = ["ks_scan.hip", "ks_pairs_i32.hip", "ks_pairs_i64.hip", "ks_pairs_float.hip", "ks_pairs_struct.hip",
           "ks_pairs_mapped.hip", "ks_pairs_bytes.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    cmd = [_hipcc(), *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    """Compile every HIP source and link the shared library; returns its path."""
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as pool:
        objs = list(pool.map(_compile, SOURCES))
    cmd = [_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    cmd = [_hipcc(), *FLAGS, "-shared", "-I", CSRC, USER_SRC, "-L", HERE, "-lks_scan", "-Wl,-rpath,$ORIGIN/..",
           "-o", USER_LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("building the user-pair example failed:\n" + r.stderr)
    cmd = [_hipcc(), "-O2", "--offload-arch=gfx950", "-I", os.path.join(os.path.dirname(HERE), "include"), C_EXAMPLE_SRC,
           "-L", HERE, "-lks_scan", "-Wl,-rpath,$ORIGIN/..", "-o", C_EXAMPLE]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("building the C example failed:\n" + r.stderr)
    if verbose:
        print(f"built {LIB}, {USER_LIB} and {C_EXAMPLE}")
    return LIB


if __name__ == "__main__":
    build()
