"""CPU fp64 oracle for the Strand-Interleaving layer step (test infrastructure only).

Nothing under this package is part of the product: only tests, the smoke check and
the CPU-baseline leg of the benchmark may import it.  It shares no code with the
HIP path and imports nothing from the product package.
"""
