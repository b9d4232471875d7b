"""CPU oracle for the additive-attention layer (test infrastructure only).

Nothing in the product path imports this package: only the tests, the smoke
check and the CPU-baseline leg of the benchmark do.  It shares no code with
the HIP kernels or their Python binding.
"""
