"""MI355X-native per-rank multi-colour reduce + SGD update (arXiv 1711.00705, Sections 3 and 4.2).

``paper_1711_00705_amd.mc`` is the binding of the C-ABI HIP library (include/mc.h);
``paper_1711_00705_amd.workloads`` holds the seeded synthetic inputs;
``paper_1711_00705_amd.build`` compiles the library with hipcc for gfx950.
Importing the package itself loads nothing.
"""
__all__ = ["mc", "workloads", "build"]
