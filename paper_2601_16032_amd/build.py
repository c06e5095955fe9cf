"""Compile the HIP sources in csrc/ into libsawattn.so (in-tree, next to this file) for gfx950."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(_HERE), "include")
LIB_PATH = os.path.join(_HERE, "libsawattn.so")
PROBE_LIB_PATH = os.path.join(_HERE, "libsawattn_probe.so")   # the benchmark's matrix-rate probe, not part of the path

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17",
    # packed fp32 arithmetic is switched off on purpose (device code only; the host pass warns
    # that it does not know the feature, which is harmless)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-shared", "-fPIC",
]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    for source, target in (("attn_fwd.hip", LIB_PATH), ("mfma_probe.hip", PROBE_LIB_PATH)):
        cmd = [hipcc, *HIPCC_FLAGS, "-I", INCLUDE, "-I", CSRC, os.path.join(CSRC, source), "-o", target]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
        if verbose:
            print(" ".join(cmd))
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
