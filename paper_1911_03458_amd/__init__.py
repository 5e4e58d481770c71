"""MI355X-native ranged inner-product (MERIT transform) hot path.

`binding` wraps the C ABI of libmerit.so (include/merit.h); `workloads` holds
the seeded synthetic input generators; `build` compiles the HIP sources.
Importing this package loads nothing heavy; the library is loaded on first use.
"""
__all__ = ["binding", "workloads", "build"]
