"""MI355X-native BLAS level-1 / level-2 kernels behind a C-ABI library (libmxblas.so).

``paper_2411_07211_amd.blas`` is the thin ctypes binding (same names as include/mxblas.h);
``paper_2411_07211_amd.synth`` holds the seeded input generators.  Nothing here falls back to a
CPU implementation: if the HIP library is missing, importing ``blas`` raises.
"""
