"""fp64 CPU oracle for the MGLU forward pass -- TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg import
this package; the GPU library and its Python binding never do.
"""
