"""CPU oracle for the LKV inference-time eviction path (test infrastructure only).

Nothing under this package is part of the product.  Only the tests, the smoke
check and the benchmark's ``cpu_baseline`` leg may import it; the HIP path
shares no code with it.
"""
