"""CPU fp64 oracle for decode-phase attention over a KV cache.

TEST INFRASTRUCTURE ONLY.  Nothing under this directory is part of the product
path: only the tests, the smoke check and the benchmark's cpu_baseline leg may
import it.  It shares no code with the HIP library and never imports it.
"""
