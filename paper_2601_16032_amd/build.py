"""Compile the HIP sources in csrc/ into libsawattn.so (in-tree, next to this file) for gfx950."""
from __future__ import annotations

import os
import re
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


def kernel_resources(remarks: str) -> dict:
    """{mangled kernel name: {"VGPRs": n, "AGPRs": n, "ScratchSize": bytes per lane, ...}} from the compiler's
    -Rpass-analysis=kernel-resource-usage remarks."""
    out, cur = {}, None
    for line in remarks.splitlines():
        m = re.search(r"remark:\s+Function Name: (\S+)", line)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        m = re.search(r"remark:\s+([A-Za-z ]+?)(?: \[[^\]]*\])?: (\d+) \[-Rpass", line)
        if m and cur is not None:
            cur[m.group(1).strip()] = int(m.group(2))
    return out


def check_wide_kernels(resources: dict) -> None:
    """The kernels with 64 rows per wavefront (fourth template argument 2) issue their MFMAs as inline assembly with
    hand-placed wait states.  That is only sound while the compiler keeps every accumulator where the source puts
    it: a spill would copy registers that an MFMA in flight is still writing.  Refuse a build in which one of them
    needs scratch memory."""
    wide = {k: v for k, v in resources.items() if "attn_fwd_kernel" in k and "ELi2ELb" in k}
    if len(wide) != 4:
        raise RuntimeError(f"expected the resource usage of 4 kernels with 64 rows per wavefront, found {sorted(wide)}")
    bad = {k: v["ScratchSize"] for k, v in wide.items() if v.get("ScratchSize", -1) != 0}
    if bad:
        raise RuntimeError(f"kernels with 64 rows per wavefront must not use scratch memory (bytes per lane): {bad}")


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    for source, target in (("attn_fwd.hip", LIB_PATH), ("mfma_probe.hip", PROBE_LIB_PATH)):
        cmd = [hipcc, *HIPCC_FLAGS, "-Rpass-analysis=kernel-resource-usage", "-I", INCLUDE, "-I", CSRC,
               os.path.join(CSRC, source), "-o", target]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
        if source == "attn_fwd.hip":
            try:
                check_wide_kernels(kernel_resources(res.stderr))
            except RuntimeError:
                os.remove(target)      # never leave a library behind that must not be used
                raise
        if verbose:
            print(" ".join(cmd))
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
