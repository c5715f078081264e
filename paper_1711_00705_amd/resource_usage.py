"""Per-kernel register, scratch and occupancy figures as the compiler reports them.

Compiles each HIP source of the library for gfx950 (device side only) with
`-Rpass-analysis=kernel-resource-usage` and prints one table row per kernel instance.  Needs no
GPU.  `python -m paper_1711_00705_amd.resource_usage > profiles/kernel_resource_usage.txt`
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

from . import build as b

FIELDS = ("VGPRs", "AGPRs", "TotalSGPRs", "ScratchSize [bytes/lane]", "Occupancy [waves/SIMD]",
          "VGPRs Spill", "SGPRs Spill", "LDS Size [bytes/block]")


def demangle(names):
    import shutil
    filt = shutil.which("c++filt") or shutil.which("llvm-cxxfilt")
    if not filt:
        return names
    res = subprocess.run([filt], input="\n".join(names), capture_output=True, text=True)
    out = res.stdout.splitlines()
    return out if len(out) == len(names) else names


def short(name: str) -> str:
    name = name.replace("(anonymous namespace)::", "")
    name = re.sub(r"^void ", "", name)
    name = re.sub(r"\(.*$", "", name)          # drop the argument list
    return name


def remarks(source: str):
    with tempfile.TemporaryDirectory() as tmp:
        cmd = [b.hipcc(), *[f for f in b.HIPCC_FLAGS if f != "-shared"], "--offload-device-only", "-c",
               "-Rpass-analysis=kernel-resource-usage", "-I", os.path.join(b.ROOT, "include"), "-I", b.CSRC,
               os.path.join(b.CSRC, source), "-o", os.path.join(tmp, "x.o")]
        res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(res.stderr)
    rows, cur = [], None
    for line in res.stderr.splitlines():
        m = re.search(r"remark:\s+Function Name: (\S+)", line)
        if m:
            cur = {"name": m.group(1)}
            rows.append(cur)
            continue
        m = re.search(r"remark:\s+([A-Za-z][^:]*): (\S+) \[-Rpass-analysis", line)
        if m and cur is not None:
            cur[m.group(1).strip()] = m.group(2)
    return rows


def collect():
    """[(source, [(kernel name, {field: value})])] for every HIP source of the library."""
    sources = [s for s in b.SOURCES if s.endswith(".hip")]
    with ThreadPoolExecutor(max_workers=4) as pool:
        per_source = list(pool.map(remarks, sources))
    return sources, per_source


def main() -> None:
    sources, per_source = collect()
    print("Kernel resource usage reported by hipcc -Rpass-analysis=kernel-resource-usage for gfx950")
    print("(python -m paper_1711_00705_amd.resource_usage; flags: " + " ".join(b.HIPCC_FLAGS) + ")")
    print("Template arguments: reduce_update_kernel / fused_step_kernel <terms (0 = run-time count), vectors per")
    print("thread, threads, mode (0 sum only, 1 update + g, 2 update, 3 per segment), streamed state>;")
    print("reduce_update_direct_kernel / fused_direct_kernel / fused_unit_kernel <terms, mode, streamed state>;")
    print("gather_scatter_kernel <unpack, stream tensors, stream flat, vectors per thread>.")
    print()
    head = ("kernel", "VGPR", "AGPR", "SGPR", "scratch B/lane", "waves/SIMD", "VGPR spill", "SGPR spill", "LDS B")
    for src, rows in zip(sources, per_source):
        names = [short(n) for n in demangle([r["name"] for r in rows])]
        print(f"== {src}: {len(rows)} kernel instances")
        print("%-58s %5s %5s %5s %14s %10s %10s %10s %6s" % head)
        for n, r in sorted(zip(names, rows), key=lambda x: x[0]):
            print("%-58s %5s %5s %5s %14s %10s %10s %10s %6s" % ((n,) + tuple(r.get(f, "?") for f in FIELDS)))
        worst = max(int(r.get("ScratchSize [bytes/lane]", 0)) for r in rows) if rows else 0
        low = min(int(r.get("Occupancy [waves/SIMD]", 8)) for r in rows) if rows else 0
        print(f"-- largest scratch {worst} B/lane, lowest occupancy {low} waves/SIMD")
        print()


if __name__ == "__main__":
    sys.exit(main())
