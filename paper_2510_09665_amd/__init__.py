"""MI355X-native KV-cache chunk mover: paged GPU KV <-> contiguous 256-token chunks in
pinned host memory (the batched store / retrieve path of the paper's section 5.1).

`paper_2510_09665_amd.lmc` is the ctypes binding of the C-ABI library built from
csrc/; `paper_2510_09665_amd.workloads` draws the seeded synthetic inputs.  Importing
the package loads neither.
"""
__all__ = ["lmc", "workloads", "build"]
