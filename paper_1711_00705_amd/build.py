"""Builds libmc.so (the C-ABI HIP library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libmc.so")
SOURCES = ("mc_layout.cpp", "mc_pack.hip", "mc_reduce_update.hip", "mc_fused.hip", "mc_packets.hip", "mc_schedule.hip",
           "mc_copy.hip", "mc_trees.cpp")
HIPCC_FLAGS = (
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # every add / multiply of the update is rounded on its own: no fused multiply-add
    "-ffp-contract=off",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # leading scalar kernel arguments arrive in registers at wavefront start instead of through loads
    "-mllvm", "-amdgpu-kernarg-preload-count=14",
    "-Wall", "-Wno-unused-command-line-argument",
)


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "packed-fp32-ops"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)


def build_library(verbose: bool = False) -> str:
    """Compile every source of the library (in parallel, one object each) and link them; always
    recompiles.  Returns the .so path."""
    import shutil
    import tempfile
    from concurrent.futures import ThreadPoolExecutor
    tmpdir = tempfile.mkdtemp(prefix="mc_build_")
    try:
        compile_flags = [f for f in HIPCC_FLAGS if f != "-shared"]
        inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]

        def compile_one(src):
            obj = os.path.join(tmpdir, src + ".o")
            _run([hipcc(), *compile_flags, *inc, "-c", os.path.join(CSRC, src), "-o", obj], verbose)
            return obj
        with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
            objs = list(pool.map(compile_one, SOURCES))
        tmp = LIB + ".tmp%d" % os.getpid()
        try:
            _run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-Wno-unused-command-line-argument",
                  "-o", tmp, *objs], verbose)
            os.replace(tmp, LIB)
        finally:
            if os.path.exists(tmp):
                os.remove(tmp)
    finally:
        shutil.rmtree(tmpdir, ignore_errors=True)
    return LIB


def library_path(build_if_missing: bool = True) -> str:
    """Path of the built library; builds it only when none is there."""
    if not os.path.exists(LIB):
        if not build_if_missing:
            raise FileNotFoundError(LIB)
        build_library()
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
