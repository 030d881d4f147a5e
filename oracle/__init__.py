"""CPU oracle for the TAQ cross-attention block: test infrastructure only.

Nothing under this package is part of the product. Only tests, the smoke check
and the benchmark's CPU-baseline leg may import it; the HIP library and its
Python binding never do.
"""
