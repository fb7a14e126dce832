"""MI355X-native sparse format customization hot path (COO -> CSR/DCSR/DIA/BCSR/ELL,
hybrid decomposition, SpMV/SpMM) behind a C-ABI HIP library.

Importing the package loads nothing; `paper_2403_05802_amd.binding` loads the built
shared library on first use and raises if it is missing.
"""
__all__ = ["binding", "workloads", "build"]
