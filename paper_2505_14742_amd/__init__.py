"""MI355X-native Quaff quantized-linear hot path (HIP kernels behind a C ABI).

Importing the package loads nothing heavy; `paper_2505_14742_amd.binding` loads
the HIP library on first use and raises if it has not been built.
"""
__all__ = ["synth", "binding"]
