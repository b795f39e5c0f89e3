"""Build libtf.so (the C-ABI library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtf.so")
SOURCES = ["tf_api.hip", "gemm_generic.hip", "gemm_mfma_bf16.hip", "elementwise.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 VALU forms
    "-Wall", "-Wno-unused-command-line-argument",
    "-Rpass-analysis=kernel-resource-usage",      # per-kernel register / scratch report, checked below
]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra = os.environ.get("TF_BUILD_FLAGS", "").split()      # developer experiments, e.g. -DTF_GEMM_WN=4
    cmd = [hipcc] + HIPCC_FLAGS + extra + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    remarks = [l for l in err.splitlines() if "-Rpass-analysis=kernel-resource-usage" in l]
    err = "\n".join(l for l in err.splitlines() if "-Rpass-analysis=kernel-resource-usage" not in l)
    if remarks:   # source-context lines that clang prints under every remark
        err = "\n".join(l for l in err.splitlines() if not re.match(r"^\s*(\d+\s*)?\|", l))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    # The staged registers of the GEMM kernels must stay in registers: a kernel that uses
    # scratch memory has lost an order of magnitude of speed, so treat it as a build error.
    name = None
    for l in remarks:
        m = re.search(r"Function Name: (\S+)", l)
        if m:
            name = m.group(1)
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", l)
        if m and int(m.group(1)) != 0:
            raise RuntimeError(f"kernel {name} uses {m.group(1)} bytes/lane of scratch memory")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
