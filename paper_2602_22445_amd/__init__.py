"""ftred: correction-based fault-tolerant reduce / allreduce, simulated at scale on one MI355X.

`paper_2602_22445_amd.binding` is the thin ctypes layer over the C-ABI library
(`libftred.so`, hand-written HIP for gfx950); `paper_2602_22445_amd.workloads`
holds the seeded synthetic inputs.  Importing the package does not load the
library; `binding.lib()` does, and raises if it has not been built.
"""
__all__ = ["binding", "workloads", "build"]
