"""Build libechokv.so (HIP, gfx950) in-tree.  (The oracle is NumPy: there is no C to compile for it.)"""
from __future__ import annotations

import os
import re
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libechokv.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    "-Rpass-analysis=kernel-resource-usage",
]

# Kernels that count their own outstanding global loads (manual s_waitcnt vmcnt(N) around
# global -> LDS copies).  Register spills and stack objects go through the same counter, so any
# scratch memory in one of them would make those waits meaningless: the build refuses it.
NO_SPILL_KERNELS = ("fused_decode_dma_kernel", "prefill_attn_dma_kernel", "absorbed13scores_kernel")


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found; libechokv needs the ROCm toolchain")


def build_library(verbose: bool = False, extra_flags=()) -> str:
    """Compile every HIP source into libechokv.so.  Always recompiles."""
    srcs = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith(".hip")]
    cmd = [hipcc_path(), *HIPCC_FLAGS, *extra_flags, "-I", os.path.join(HERE, "..", "include"),
           "-o", LIB_PATH + ".tmp", *srcs]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError("hipcc failed building libechokv.so")
    spilled = check_spills(res.stdout + res.stderr)
    if spilled:
        raise RuntimeError("scratch memory (spills or stack objects) in kernels that count their own loads: "
                           + ", ".join(f"{k} ({n})" for k, n in spilled))
    os.replace(LIB_PATH + ".tmp", LIB_PATH)
    return LIB_PATH


def check_spills(remarks: str):
    """(kernel, amount) for every NO_SPILL_KERNELS instance that spills registers or keeps objects
    in scratch memory, from the compiler's resource-usage remarks."""
    bad, cur = [], None
    for line in remarks.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            cur = m.group(1)
            continue
        m = re.search(r"(?:VGPRs Spill|ScratchSize \[bytes/lane\]): (\d+)", line)
        if m and cur and int(m.group(1)) > 0 and any(k in cur for k in NO_SPILL_KERNELS):
            bad.append((cur, int(m.group(1))))
    return bad


if __name__ == "__main__":
    print(build_library(verbose=True))
