"""CPU oracle for the CoreInfer hot path.  TEST INFRASTRUCTURE ONLY.

Nothing under this package is part of the product: only the tests, the smoke
check and the benchmark's CPU-baseline leg may import it.  It shares no code
with the HIP library and imports nothing from it.
"""
