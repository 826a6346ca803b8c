"""CPU oracle for the structured tensor ops -- test infrastructure only.

Only tests, the smoke check and the CPU-baseline leg of the benchmark may import
this package.  It shares nothing with the GPU library.
"""
