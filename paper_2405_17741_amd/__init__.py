"""Per-token LoRA expert switch for AMD MI355X (gfx950): Python binding of liblsw.

`binding` mirrors include/lsw.h one to one; `inputs` draws the seeded synthetic
workloads; `build` compiles the HIP library in-tree.  Importing the package does not
load the library; the first call through `binding` does, and fails loudly if it is missing.
"""
__all__ = ["binding", "inputs", "build"]
