"""MI355X-native Partial FC (PFC) training step (arXiv 2203.15565, Sec. 3.2).

`binding` wraps the C-ABI library libpfc.so (hand-written HIP for gfx950); `workloads`
draws the seeded synthetic inputs.  Importing the package loads nothing native; the first
use of `binding` loads the library and raises if it has not been built.
"""
__all__ = ["binding", "workloads", "build"]
