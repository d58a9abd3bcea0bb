"""Builds the HIP library in-tree for gfx950 (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
REPO_DIR = os.path.dirname(PKG_DIR)
LIB_PATH = os.path.join(PKG_DIR, "libhe_fedavg.so")
SOURCES = [os.path.join(PKG_DIR, "csrc", "he_fedavg.hip")]
# measurement helper of bench.py --issue-rates (register-only instruction-rate loops): a library of its own
RATES_LIB_PATH = os.path.join(PKG_DIR, "libhe_issue_rates.so")
RATES_SOURCES = [os.path.join(PKG_DIR, "csrc", "he_issue_rates.hip")]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build_library(verbose: bool = False) -> str:
    _compile(LIB_PATH, SOURCES, verbose)
    _compile(RATES_LIB_PATH, RATES_SOURCES, verbose)
    return LIB_PATH


def _compile(lib_path, sources, verbose):
    cmd = [
        hipcc_path(), "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
        # No packed-fp32 code generation on the device (checked on the ISA: a float2 multiply-add compiles to v_pk_fma_f32
        # without the flag and to two scalar instructions with it).  The x86 host pass does not know the feature and
        # says so once per pass ("not a recognized feature for this target"): that line is filtered below.
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wall", "-Wno-unused-function",
        "-I", os.path.join(REPO_DIR, "include"), "-I", os.path.join(PKG_DIR, "csrc"),
        "-o", lib_path, *sources,
    ]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    noise = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"
    rest = "\n".join(l for l in res.stderr.splitlines() if l.strip() and l.strip() != noise)
    if verbose and rest:
        print(rest)


if __name__ == "__main__":
    print(build_library(verbose=True))
