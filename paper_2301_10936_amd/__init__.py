"""MI355X-native hot path of permutation-invariant-transformation (PIT) dynamic sparse GEMM.

``paper_2301_10936_amd.pit``       -- thin ctypes binding of the C-ABI library (needs the built HIP library;
                                      importing it raises if the library is missing).
``paper_2301_10936_amd.workloads`` -- seeded synthetic input generators (no method arithmetic).
"""
