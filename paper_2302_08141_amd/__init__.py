"""Plan scoring for automatic parallelization on MI355X (gfx950).

The package holds the HIP kernels behind a C-ABI library (`csrc/`), a thin
ctypes binding with the same entry-point names (`binding.py`), and seeded
synthetic search inputs (`workloads/`).  Nothing here falls back to the CPU:
using the binding without the built library raises.
"""
