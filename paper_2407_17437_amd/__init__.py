"""Truly sparse MLP training step for MI355X (gfx950): CSR SpMM / transposed SpMM /
SDDMM / momentum update kernels behind a C-ABI library, with a thin ctypes binding.

`workloads` (seeded synthetic inputs, numpy only) can be imported without the
compiled library; `binding` loads the HIP library on first use and raises if it
has not been built.
"""
