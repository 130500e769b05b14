"""Build the gfx950 shared library (C ABI in include/moe.h) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libmoe_gfx950.so")
SOURCES = ["moe_api.hip", "route.hip", "dispatch.hip", "ffn.hip", "combine.hip", "plan.hip", "probe.hip"]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the MoE library cannot be built")
    return exe


def build(verbose: bool = False, keep_asm_dir: str | None = None) -> str:
    """Compile every HIP source for gfx950 into libmoe_gfx950.so; returns its path."""
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-I" + os.path.join(ROOT, "include"),
           # packed fp32 instructions are kept off on the test machines
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument"]
    if keep_asm_dir:
        os.makedirs(keep_asm_dir, exist_ok=True)
        cmd += ["-save-temps=obj"]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    tmp = LIB_PATH + ".tmp"
    out = os.path.join(keep_asm_dir, "libmoe_gfx950.so") if keep_asm_dir else tmp
    cmd += ["-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    log = "\n".join(l for l in (res.stdout + res.stderr).splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + log)
    if verbose and log.strip():
        print(log)
    if keep_asm_dir:
        shutil.copyfile(out, tmp)
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True, keep_asm_dir=sys.argv[1] if len(sys.argv) > 1 else None))
