"""CPU oracle for the collective KV-reuse step.  TEST INFRASTRUCTURE ONLY.

Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may
import this package; the product path never does.
"""
