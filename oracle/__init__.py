"""CPU oracle for the XCD-swizzled GEMM path.

TEST INFRASTRUCTURE ONLY.  Nothing here is part of the product: it is imported by the tests,
by the smoke check and by the benchmark's CPU-baseline leg, never by the library or its
Python binding, and it shares no code with them.  Everything is plain, slow and written to be
checked against the paper by eye.
"""
