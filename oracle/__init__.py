"""CPU oracle for the V:N:M format and its sparse x dense product.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this directory; only the
test-suite, the smoke entry and the benchmark's CPU-baseline leg may call it.  It shares no
code, tables or helpers with the HIP library.
"""
