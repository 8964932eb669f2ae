"""MI355X-native masked (cache-enabled sparse) UNet step.

`paper_2305_17423_amd.binding` is the thin ctypes layer over the C-ABI library
built from csrc/ (see include/fise.h); `paper_2305_17423_amd.workloads` holds
the seeded synthetic input generators.  Importing the package loads neither.
"""
