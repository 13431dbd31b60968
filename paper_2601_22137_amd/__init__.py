"""MI355X-native PRISM hot path: HIP kernels behind a C-ABI (csrc/, include/prism.h)
and a thin ctypes binding (prism.py).  workloads.py holds the seeded input recipes."""
