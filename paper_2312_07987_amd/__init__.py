"""SwitchHead attention layer (arXiv 2312.07987) for one MI355X: hand-written HIP kernels
behind a C ABI (include/switchhead.h), with this thin ctypes binding on top.

Importing the package does not load the library; `paper_2312_07987_amd.binding` loads
it on first use and raises if it has not been built (there is no fallback path).
"""
