"""OD-SGD parameter-update engine for MI355X (gfx950).

The package holds the HIP kernels and C-ABI library (csrc/), a thin ctypes
binding (binding.py) and the seeded synthetic workloads (workloads.py).
Importing the package does not load the GPU library; the binding loads it on
first use and raises if it has not been built.
"""
