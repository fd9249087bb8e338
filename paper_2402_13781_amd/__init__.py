"""MI355X-native ExDyna gradient-selection hot path (HIP kernels behind a C-ABI).

Importing the package does not load the HIP library; `binding` does, on first use,
and fails loudly when it is missing.
"""
__all__ = ["binding", "synthetic"]
