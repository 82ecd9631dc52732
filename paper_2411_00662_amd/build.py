"""Builds libmonta.so (HIP, gfx950) in-tree with hipcc.  Cross-compiles without a GPU."""
from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
SRC = os.path.join(PKG, "csrc", "monta.hip")
DEPS = [SRC, os.path.join(PKG, "csrc", "monta_kernels.hpp"), os.path.join(PKG, "csrc", "monta_planner.hpp"),
        os.path.join(ROOT, "include", "monta.h")]
LIB = os.path.join(PKG, "libmonta.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed fp32 instructions out of scalar float code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra",
]


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile the library.  With force=False an up-to-date library is kept."""
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in DEPS):
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-Rpass-analysis=kernel-resource-usage", "-I" + os.path.join(ROOT, "include"),
           "-o", LIB, SRC]
    res = subprocess.run(cmd, capture_output=True, text=True)
    failed = res.returncode != 0
    if verbose or failed:
        print(" ".join(cmd))
        print(res.stdout)
        print("\n".join(l for l in res.stderr.splitlines() if failed or "remark:" not in l))
    if failed:
        raise RuntimeError("hipcc failed building libmonta.so")
    spills = scratch_users(res.stderr)
    if spills:
        # a kernel that spills registers to scratch memory still computes the right thing, many times slower (an
        # innocent-looking edit of the expert kernel once did that): refuse the build rather than ship it
        os.remove(LIB)
        raise RuntimeError("kernels spill registers to scratch: " + ", ".join(f"{k} ({v} B/lane)" for k, v in spills))
    return LIB


def scratch_users(remarks: str):
    """(kernel, bytes per lane) for every kernel whose resource-usage remark reports scratch memory."""
    out, name = [], None
    for line in remarks.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split("[")[0].strip()
        elif "ScratchSize [bytes/lane]:" in line and name:
            n = int(line.split("ScratchSize [bytes/lane]:")[1].split("[")[0].strip())
            if n > 0:
                out.append((name, n))
    return out


if __name__ == "__main__":
    print(build(verbose=True))
