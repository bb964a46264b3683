"""Builds libsvf.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import re
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libsvf.so")

SOURCES = ["svf_api.hip", "block_reps.hip", "score_select.hip", "verify_attn_valu.hip", "verify_attn_mfma.hip",
           "analytics.hip", "retrieval_variants.hip", "sparse_ffn.hip", "svf_ffn_api.hip", "spec_rules.hip"]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # packed fp32 instruction forms are kept out of the generated code on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    # per-kernel register / scratch report on stderr, checked below
    "-Rpass-analysis=kernel-resource-usage",
]

# Kernels that must not use scratch memory (a private segment makes every dispatch slower, and an
# array the compiler moved there turns register accesses into memory round trips).
NO_SCRATCH = ("verify_attn_mfma_kernel", "verify_attn_mfma_rows_kernel", "retrieve_only_kernel")


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build_lib(verbose: bool = True) -> str:
    """Compile every HIP source into paper_2512_21911_amd/libsvf.so; returns its path."""
    cmd = [hipcc_path(), *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    lines = [l for l in res.stderr.splitlines() if noise not in l]
    remarks = [l for l in lines if "remark:" in l]
    # (a remark is followed by the source line it points at and a caret line)
    context = re.compile(r"^\s*(\d+\s*)?\|")
    err = "\n".join(l for l in lines if "remark:" not in l and not context.match(l))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + "\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    # the report names a kernel ("Function Name: ...") and then lists its resources
    name = None
    for l in remarks:
        if "Function Name:" in l:
            name = l.split("Function Name:")[1].split("[-Rpass")[0].strip()
        elif "ScratchSize [bytes/lane]:" in l and name and any(k in name for k in NO_SCRATCH):
            size = int(l.split("ScratchSize [bytes/lane]:")[1].split()[0])
            if size != 0:
                raise RuntimeError(f"{name} uses {size} bytes of scratch memory per lane")
    return LIB_PATH


if __name__ == "__main__":
    build_lib()
