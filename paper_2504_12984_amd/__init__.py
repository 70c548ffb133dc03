"""MI355X-native mixed-precision matmul  C = A . dequant(W)  for 1..8-bit weights.

The compute lives in the HIP library built from csrc/ (see include/qgemm.h for
the C ABI); `binding` is the thin ctypes layer over it.  Importing this package
does not load the library; `paper_2504_12984_amd.binding` does, and fails loudly
if it has not been built.
"""
