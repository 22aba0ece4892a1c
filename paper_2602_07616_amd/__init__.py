"""MI355X-native batch-decode MoE layer with SERE expert re-routing.

The product is the HIP library `libsere.so` (C ABI in include/sere.h); this
package holds its sources (csrc/), the ctypes binding, the seeded synthetic
workload generator and small helpers to place a workload in HBM.
"""
from . import workloads  # noqa: F401  (numpy only; safe without a GPU)
