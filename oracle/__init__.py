"""CPU oracle for the TRIM filter-then-refine scan.  Test infrastructure only.

Nothing under this directory is part of the product: only tests/, the smoke check and the
benchmark's reported CPU-baseline leg may import it, and it imports nothing from the
HIP package.
"""
