"""Build the gfx950 shared library (C ABI in include/moe.h) in-tree with hipcc."""
from __future__ import annotations

import hashlib
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libmoe_gfx950.so")
STAMP_PATH = LIB_PATH + ".srchash"
OBJ_DIR = os.path.join(ROOT, "_build", "obj")
SOURCES = ["moe_api.hip", "route.hip", "dispatch.hip", "ffn.hip", "combine.hip", "plan.hip", "probe.hip"]
HEADERS = [os.path.join(CSRC, "moe_internal.h"), os.path.join(ROOT, "include", "moe.h")]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the MoE library cannot be built")
    return exe


def source_hash() -> str:
    """Hash of every file the library is compiled from (what a built library is checked against)."""
    h = hashlib.sha256()
    for path in [os.path.join(CSRC, s) for s in SOURCES] + HEADERS:
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def is_current() -> bool:
    """True if a built library exists and was built from the sources as they are now."""
    if not (os.path.exists(LIB_PATH) and os.path.exists(STAMP_PATH)):
        return False
    with open(STAMP_PATH) as fh:
        return fh.read().strip() == source_hash()


def _flags() -> list:
    return ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + os.path.join(ROOT, "include"),
            # packed fp32 instructions are kept off on the test machines
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wno-unused-command-line-argument"]


def _run(cmd) -> str:
    res = subprocess.run(cmd, capture_output=True, text=True)
    log = "\n".join(l for l in (res.stdout + res.stderr).splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + log)
    return log


def build(verbose: bool = False, jobs: int = 8) -> str:
    """Compile every HIP source for gfx950 (one hipcc per file, in parallel) and link
    libmoe_gfx950.so; returns its path. Always compiles everything."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    stamp = source_hash()
    objs = [os.path.join(OBJ_DIR, s.replace(".hip", ".o")) for s in SOURCES]

    def compile_one(pair):
        src, obj = pair
        return _run([hipcc()] + _flags() + ["-c", os.path.join(CSRC, src), "-o", obj])

    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(SOURCES)))) as pool:
        logs = list(pool.map(compile_one, zip(SOURCES, objs)))
    tmp = LIB_PATH + ".tmp"
    logs.append(_run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", tmp]))
    os.replace(tmp, LIB_PATH)
    with open(STAMP_PATH, "w") as fh:
        fh.write(stamp + "\n")
    if verbose:
        text = "\n".join(l for l in logs if l.strip())
        if text:
            print(text)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
