"""MI355X-native CAT-loss hot path of PARD-2 (HIP kernels behind a C ABI).

Importing the package loads nothing; `paper_2605_08632_amd.binding` loads the
HIP library on first use and raises if it has not been built.
"""
