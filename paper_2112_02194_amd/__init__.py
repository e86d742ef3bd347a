"""MI355X-native implicit-ALS half-epoch solve (hand-written HIP behind a C ABI).

The Python layer only marshals arguments: every step of the method runs in the
kernels of ``libals.so`` (sources under ``csrc/``).  Import ``paper_2112_02194_amd.binding``
for the functions; importing this package alone loads nothing.
"""
__all__ = ["binding", "build"]
