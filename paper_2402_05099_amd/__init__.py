"""MI355X-native shared-prefix decode attention (Hydragen, arXiv 2402.05099): HIP kernels behind a C ABI.

`binding` mirrors include/hydragen.h; `workloads` makes the seeded synthetic inputs; `device` moves them to
the GPU; `build` compiles the shared library in-tree.  Importing this package loads nothing native.
"""
