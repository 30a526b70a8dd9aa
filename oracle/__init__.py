"""CPU oracle for the fine-grained FP8 linear layer (test infrastructure only).

Nothing under this package is part of the product path.  Only the test-suite,
the smoke check and the ``cpu_baseline`` leg of the benchmark may import it.
"""
