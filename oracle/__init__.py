"""CPU oracle for the DistFlashAttn per-worker hot path.

TEST INFRASTRUCTURE ONLY.  Nothing under this package is part of the product:
only the tests, the smoke check and the bench's `cpu_baseline` leg may import
it.  It shares no code with the HIP path and never imports it.
"""
