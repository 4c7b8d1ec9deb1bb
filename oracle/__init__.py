"""CPU oracle for layout-propagating GEMM chains.  TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 reference implementations written from the method's
definitions.  Only tests, the smoke check and the benchmark's CPU-baseline leg
may import this package; the product package never does, and this package
imports nothing from the product.
"""
