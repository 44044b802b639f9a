"""Builds libcce.so (HIP, gfx950) in-tree with hipcc.  No GPU is needed to compile."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libcce.so")
SOURCES = [os.path.join(CSRC, "cce_kernels.hip"), os.path.join(CSRC, "aux_kernels.hip")]
HEADERS = [os.path.join(CSRC, "gemm_core.h"), os.path.join(CSRC, "host_util.h"), os.path.join(CSRC, "plan.h"), os.path.join(CSRC, "wg_map.h"),
           os.path.join(os.path.dirname(PKG_DIR), "include", "cce.h"),
           os.path.join(os.path.dirname(PKG_DIR), "include", "cce_aux.h"),
           os.path.join(os.path.dirname(PKG_DIR), "include", "cce_shard.h"),
           os.path.join(os.path.dirname(PKG_DIR), "include", "cce_fp8.h"),
           os.path.join(os.path.dirname(PKG_DIR), "include", "cce_compact.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-Wno-inline-asm",          # the M0 clobber of the global->LDS load is intentional
]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = True, extra_flags: list[str] | None = None) -> str:
    """Compile every HIP source into libcce.so; always recompiles."""
    cmd = [hipcc_path(), *HIPCC_FLAGS, *(extra_flags or []), *SOURCES, "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (res.stdout + res.stderr).splitlines()
                    if "packed-fp32-ops" not in l)
    if verbose and out.strip():
        print(out)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{out}")
    return LIB_PATH


def is_built() -> bool:
    return os.path.exists(LIB_PATH)


if __name__ == "__main__":
    build()
    sys.exit(0)
