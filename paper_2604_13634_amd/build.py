"""Build libcsd.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libcsd.so")
SOURCES = ["csd_verify.hip", "csd_sampled.hip", "csd_ocm.hip", "csd_api.hip"]
PROBE_LIB = os.path.join(PKG, "libcsd_probe.so")
PROBE_SOURCES = ["read_probe.hip"]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # no hand-written or compiler-made packed fp32 arithmetic
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # logits are never NaN: lets max/compare compile without quieting moves (device code only)
    "-Xarch_device", "-fno-honor-nans",
    "-Wno-unused-command-line-argument",
]


def _hipcc(sources, lib: str, verbose: bool) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-o", lib]
    cmd += [os.path.join(CSRC, s) for s in sources]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "is not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return lib


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source of the verification library into paper_2604_13634_amd/libcsd.so; returns its path."""
    return _hipcc(SOURCES, LIB, verbose)


def build_probe(verbose: bool = False) -> str:
    """Compile the benchmark's read-only bandwidth probe into its own small library (not part of the C ABI)."""
    return _hipcc(PROBE_SOURCES, PROBE_LIB, verbose)


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_probe(verbose=True))
