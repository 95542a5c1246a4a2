"""libheinsen for MI355X: x_t = a_t x_{t-1} + b_t as one fused log-space scan (HIP, gfx950).

The package holds the HIP sources (csrc/), the build script, the ctypes binding and the seeded
workload generators.  The binding is imported lazily so that the generators can be used without the
built library."""

__all__ = ["binding", "workloads", "build"]
