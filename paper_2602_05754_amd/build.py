"""Build libtf.so (the C-ABI library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtf.so")
SOURCES = ["tf_api.hip", "gemm_generic.hip", "gemm_mfma_bf16.hip", "elementwise.hip", "selection.hip", "schedule_lp.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 VALU forms
    "-Wall", "-Wno-unused-command-line-argument",
    "-Wno-inline-asm",          # the direct-to-LDS loads name M0 in their clobber list on purpose
    "-Rpass-analysis=kernel-resource-usage",      # per-kernel register / scratch report, checked below
]


# Scalar instructions that read the carry / condition bit SCC, and those that leave it alone.
_SCC_READERS = re.compile(r"^(s_addc_u32|s_subb_u32|s_cselect_b32|s_cselect_b64|s_cmov_b32|s_cmov_b64|"
                          r"s_cbranch_scc0|s_cbranch_scc1)\b")
_SCC_KEEPERS = re.compile(r"^(s_mov|s_movk|s_cmov|s_cselect|s_mul_i32|s_mul_hi|s_load|s_buffer_load|s_waitcnt|s_nop|"
                          r"s_barrier|s_branch|s_cbranch|s_sleep|s_setprio|s_getpc|s_setpc|s_swappc|s_sext|s_pack|"
                          r"s_bitset|s_ff1|s_ff0|s_flbit|s_brev|s_endpgm|s_sendmsg|s_getreg|s_setreg|s_memtime|"
                          r"s_memrealtime|s_dcache|s_icache|s_lshl1_add|s_lshl2_add|s_lshl3_add|s_lshl4_add)")


def scc_hazards(asm_text: str) -> list:
    """Inline assembly placed between a writer and a reader of SCC.

    The direct-to-LDS loads of the GEMM kernel are inline assembly that sets SCC.  The
    compiler is told so (clobber list), which keeps it from putting such a statement between,
    say, the s_add_u32 and the s_addc_u32 of a 64-bit address addition; a lost carry there is
    a wild global address.  This scan of the generated code is the belt to those braces: it
    walks every function linearly and reports each reader of SCC whose nearest preceding
    scalar instruction that writes SCC lies before an inline-assembly block that sets SCC itself.
    Returns a list of (function, line number, instruction)."""
    bad = []
    func = None
    in_asm = False
    asm_since_write = False
    for ln, raw in enumerate(asm_text.splitlines(), 1):
        line = raw.strip()
        if not line or line.startswith(";") and "ASM" not in line:
            continue
        if re.match(r"^[A-Za-z_.$][\w.$]*:", line) and not line.startswith(".L"):
            func = line.split(":")[0]
            asm_since_write = False
            continue
        if "#ASMSTART" in line:
            in_asm = True
            continue
        if "#ASMEND" in line:
            in_asm = False
            continue
        if in_asm:
            # only assembly that itself sets SCC can lose a carry (a vector addition without carry,
            # a plain move or a load leaves it alone)
            if line.startswith("s_") and not _SCC_KEEPERS.match(line.split()[0]):
                asm_since_write = True
            continue
        if not line.startswith("s_"):
            continue
        op = line.split()[0]
        if _SCC_READERS.match(op) and asm_since_write:
            bad.append((func, ln, line))
        if not _SCC_KEEPERS.match(op):      # every other scalar ALU / compare instruction writes SCC
            asm_since_write = False
    return bad


def check_scc(hipcc: str, extra: list) -> None:
    src = os.path.join(CSRC, "gemm_mfma_bf16.hip")
    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared", "-Rpass-analysis=kernel-resource-usage")]
    cmd = [hipcc] + flags + extra + ["-S", "--cuda-device-only", src, "-o", "-"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc -S failed:\n" + res.stderr)
    bad = scc_hazards(res.stdout)
    if bad:
        raise RuntimeError("inline assembly between a writer and a reader of SCC:\n" +
                           "\n".join(f"  {f} line {ln}: {ins}" for f, ln, ins in bad[:10]))


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra = os.environ.get("TF_BUILD_FLAGS", "").split()      # developer experiments
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
    check_scc(hipcc, extra)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
