"""SALS decode-step attention for MI355X (gfx950): hand-written HIP kernels
behind a C ABI (``include/sals.h``), a thin ctypes binding, and seeded
synthetic workloads.  ``synth`` needs only numpy; ``binding`` needs torch and
the built library and fails loudly without them."""

__all__ = ["synth", "binding", "build", "roofline"]
